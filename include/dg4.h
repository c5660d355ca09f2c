/*
 * dg4 - sparse graph-attention layer over And-Inverter Graphs on AMD MI355X.
 *
 * C ABI of the data-parallel hot path of DeepGate4 (arXiv 2502.01681): node
 * features plus an AIG edge list with inverter flags in, gate embeddings out.
 *
 * Conventions for every call
 *   - returns 0 (DG4_OK) or a negative dg4_status; nothing throws or aborts
 *     across the boundary; on error the outputs are left untouched unless a
 *     device error (DG4_EHIP) struck after work had been queued.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP
 *     device memory of the current device, owned by the caller. The library
 *     allocates device memory only inside a dg4_graph (its neighbour tables),
 *     on the first device call that uses the graph or in dg4_graph_upload.
 *   - rows of X, H, Q, K, V, A are indexed by ORIGINAL node id, row-major,
 *     `hidden` elements each, element type cfg->dtype (float or bfloat16).
 *     Device tensors and weight matrices start on a 16-byte boundary (EINVAL
 *     otherwise): rows are read and written as 16-byte pieces.
 *   - device calls are asynchronous on `stream` (a hipStream_t, may be NULL
 *     for the default stream) and touch no other stream.
 *   - a dg4_graph is immutable after construction; concurrent calls may share it.
 */
#ifndef DG4_H
#define DG4_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dg4_graph dg4_graph;

#define DG4_MAX_HOPS 8      /* deepest cone (the paper's k = 8): rows of at most 2^9 - 1 entries */

typedef enum { DG4_F32 = 0, DG4_BF16 = 1 } dg4_dtype;

typedef enum {
    DG4_OK = 0,
    DG4_EINVAL = -1,        /* null pointer, negative size, bad flag or bad config field   */
    DG4_ERANGE = -2,        /* node id outside [0, n_nodes)                                */
    DG4_EFANIN = -3,        /* in-degree above 2, or the same (src,dst) pair twice         */
    DG4_ECYCLE = -4,        /* the edge list is not a DAG (self loops included)            */
    DG4_EHINT = -5,         /* level_hint is not a topological levelling with PIs at 0     */
    DG4_EUNSUPPORTED = -6,  /* head dim != 32, hidden not 128/256, hops not 1..8, layers>16 */
    DG4_ENOMEM = -7,        /* host or device allocation failed                            */
    DG4_EWORKSPACE = -8,    /* workspace missing, misaligned (256 B) or too small          */
    DG4_EHIP = -9,          /* a HIP runtime call failed                                   */
    DG4_EABORTED = -10      /* dg4_layer_status: the last persistent sweep gave up on a    */
                            /* dependency wait; Hout is incomplete                         */
} dg4_status;

/* cfg->flags */
#define DG4_NO_EPILOGUE 1u  /* H = A*Wo without residual and LayerNorm (kernel tests)      */
#define DG4_PER_LEVEL   2u  /* dg4_layer_fwd: launch level by level instead of the single  */
                            /* persistent dataflow kernel (same results; for comparison).  */
                            /* Level-by-level sweeps over ALL levels of a graph built with */
                            /* a level_hint deeper than Eq. 1 go through the Eq. 1 levels  */
                            /* (fewer rounds, same bits; host-built graphs only)           */
#define DG4_BOUNDED_KV  4u  /* dg4_layer_fwd: keep no K|V store of finished gates. The K|V  */
                            /* rows of a level's distinct sources are projected from Hout   */
                            /* when the level is processed, so the workspace holds one      */
                            /* level's frontier only (Section 3.4: memory that does not     */
                            /* grow with the graph). Level-by-level launches; same results  */
                            /* bit for bit; the projection work is repeated per reader level */
#define DG4_FFN         8u  /* dg4_layer_fwd: every layer ends with the position-wise feed-  */
                            /* forward sub-block of the transformer (Section 3.5 keeps the   */
                            /* transformer structure around the attention):                  */
                            /* s <- LayerNorm(s + max(s W1, 0) W2).                          */
                            /* Not together with DG4_NO_EPILOGUE                             */
#define DG4_LEVEL_ORDER 16u /* dg4_layer_fwd: a sweep over ALL levels follows the graph's own  */
                            /* levels (the caller's level_hint, if one was given) instead of  */
                            /* the library's dependency-driven order. Same results bit for    */
                            /* bit; for comparisons of schedules                              */
#define DG4_PROFILE     32u /* dg4_layer_fwd: the specialised persistent kernel accumulates    */
                            /* per-phase timers, read back by dg4_layer_profile                */
#define DG4_TIME_SWEEP  64u /* dg4_layer_fwd: bracket the persistent kernel with two events on  */
                            /* the caller's stream, read back by dg4_sweep_elapsed_ms           */
#define DG4_WEIGHTS_PACKED 128u /* dg4_layer_fwd: the caller vouches that W holds the same      */
                            /* values as in its previous completed call with the same cfg       */
                            /* (apart from this flag), graph, level range and workspace, and    */
                            /* that nothing else wrote to the workspace since: the copies of    */
                            /* the weights in matrix-core operand order that call left in the   */
                            /* workspace are used again instead of being rebuilt                */

typedef struct {
    int32_t hidden;         /* d: 128 or 256                                               */
    int32_t heads;          /* d / 32                                                      */
    int32_t hops;           /* k of cone_k, must equal the graph's                         */
    int32_t n_layers;       /* 1..16 stacked layers (dg4_layer_fwd only; the paper uses 12) */
    int32_t dtype;          /* dg4_dtype of X, H, Q, K, V, A and of the weight matrices    */
    uint32_t flags;
    float ln_eps;           /* LayerNorm epsilon, e.g. 1e-5                                */
    uint32_t spin_limit;    /* persistent sweeps: polls of a "published" flag before a tile */
                            /* gives up and the sweep aborts (dg4_layer_status); 0 = the     */
                            /* default of 2^22 (seconds). Tests of the abort path use 1      */
} dg4_layer_cfg;

/*
 * Graph analysis (paper Section 3.2). HOST call, host pointers.
 *   - node type by in-degree: 0 primary input, 2 AND, 1 NOT/buffer; ids need
 *     not be topological. edge_inv[e] in {0,1} marks an inverted fanin edge.
 *   - level(v) by Eq. 1; or, if level_hint (n_nodes entries) is given, the hint
 *     after checking hint[PI] == 0 and hint[dst] > hint[src] for every edge. The
 *     level only names the ranges a sweep can be cut into (level_begin, level_end of
 *     dg4_layer_fwd) and orders the work of a partial sweep; embeddings do not depend on it.
 *   - order: node ids sorted by (level, id).
 *   - neighbour rows N(v) = cone_hops(v), v included, hops in 1..DG4_MAX_HOPS, at most
 *     2^(hops+1)-1 entries, ascending id, each with a relation code: 0 self, 1 direct fanin,
 *     2 direct inverted fanin, 3 ancestor first reached by >= 2 edges (the
 *     virtual edges of Section 3.5). The shortest path decides the code.
 * On success *out owns host copies of all tables; free with dg4_graph_free.
 * Errors: EINVAL, ERANGE, EFANIN, ECYCLE, EHINT, EUNSUPPORTED (hops), ENOMEM.
 */
int dg4_build_levels(int64_t n_nodes, int64_t n_edges,
                     const int32_t* edge_src, const int32_t* edge_dst, const uint8_t* edge_inv,
                     int32_t hops, const int32_t* level_hint /* nullable */,
                     dg4_graph** out);

/*
 * The same analysis (Section 3.2: levels by Eq. 1, cone rows; and the fanout counts of Eq. 2) run on
 * the GPU, for an edge list that is already in DEVICE memory: edge_src, edge_dst, edge_inv and
 * level_hint (nullable) are device pointers. Levels are found in rounds over the fanin table (a gate
 * is finished one round after its fanins), the (level, id) order by a stable sort, each cone row by a
 * backward search from its gate (up to three hops) or, for deeper cones, one hop at a time as a
 * merge of the fanins' rows (about 9 bytes per neighbour entry of temporary memory then). Every table of the resulting graph equals the host call's bit for
 * bit. Synchronous: waits on `stream`; temporary device memory (about 160 bytes per node and 5 per neighbour entry) is
 * allocated and released inside the call, and the tables are copied to host memory, where the graph
 * object keeps them. Errors as dg4_build_levels; if an edge list has defects of several kinds, the
 * kind reported may differ from the host call's (which reports the first in edge order), and an
 * invalid hint on a cyclic graph gives EHINT. Also EHIP.
 */
int dg4_build_levels_device(int64_t n_nodes, int64_t n_edges,
                            const int32_t* edge_src, const int32_t* edge_dst, const uint8_t* edge_inv,
                            int32_t hops, const int32_t* level_hint /* nullable */,
                            void* stream, dg4_graph** out);

/*
 * Graph analysis under the general partition and updating strategy (Section 3.3, Algorithm 1;
 * Section 3.4, Algorithm 2, at inference): cones of depth k = hops are collected at levels k,
 * k + stride, ... (stride < hops), then for every gate that nothing reads, then for every gate that
 * is still in no cone (the partition covers the whole circuit); the cones of a level form a list, in
 * that order, each part by ascending id, and are processed in mini-batches of batch_cones consecutive
 * cones, lists by ascending level. A gate is computed once, by the first mini-batch that holds it,
 * and marked; its neighbour row is what that mini-batch shows of its cone: the union, over the
 * mini-batch's cones c that hold v, of { u in c : u in cone_hops(v) }. Later mini-batches read it
 * from the historical embeddings. Since a marked gate never changes and every source of a gate lies
 * below it, the embeddings are those of one sweep in level order over these rows: the returned graph
 * is used with every other call exactly like one from dg4_build_levels (rows are subsets of that
 * call's rows, same order and codes), and its nnz counts the kept entries.
 * marks = 0 is the ablation without marks (Section 4.4): every mini-batch recomputes all the gates
 * of its cones from their initial features and reads nothing from earlier mini-batches; the last
 * result of a gate stands. The returned graph then has one node per (mini-batch, gate of it), a COPY,
 * numbered mini-batch after mini-batch and by ascending gate id inside one; dg4_graph_info gives the
 * number of copies as n_nodes. The caller runs the other calls on the copies: features X'[c] =
 * X[DG4_COPY_OF[c]], and the embedding of gate v is H'[DG4_LAST_COPY[v]]. The number of copies over
 * the number of gates is the work the marks save.
 * HOST call, host pointers. Errors as dg4_build_levels; EINVAL if stride < 1, stride >= hops,
 * batch_cones < 1 or marks not 0 / 1; EUNSUPPORTED if there would be 2^30 copies or more.
 */
int dg4_build_partitioned(int64_t n_nodes, int64_t n_edges,
                          const int32_t* edge_src, const int32_t* edge_dst, const uint8_t* edge_inv,
                          int32_t hops, const int32_t* level_hint /* nullable */,
                          int32_t stride, int32_t batch_cones, int32_t marks,
                          dg4_graph** out);

/*
 * dg4_build_partitioned with marks (Section 3.3, Algorithm 1; Section 3.4, Algorithm 2) on the GPU, for
 * an edge list in DEVICE memory (edge_src, edge_dst, edge_inv, level_hint: device pointers), on top of
 * dg4_build_levels_device: the kinds of roots, the members their cones cover and the left-over roots
 * per gate; the lists by a stable sort of the (level, id) order on (level, kind); the first mini-batch
 * of every gate by a minimum over the cones that hold it; the kept entries by merging a gate's row
 * with the rows of its mini-batch's roots (a wave per cone), then a compaction. Only the running
 * mini-batch numbers of the cones (one pass over the sorted roots) are formed on the host. Every
 * table, DG4_CONE_* and DG4_STAGE included, equals the host call's bit for bit. Synchronous on
 * `stream`; temporary device memory as dg4_build_levels_device plus about 22 bytes per node and one
 * byte per neighbour entry of the unrestricted cones. The ablation without marks is a host call only.
 * Errors as dg4_build_partitioned and dg4_build_levels_device.
 */
int dg4_build_partitioned_device(int64_t n_nodes, int64_t n_edges,
                                 const int32_t* edge_src, const int32_t* edge_dst, const uint8_t* edge_inv,
                                 int32_t hops, const int32_t* level_hint /* nullable */,
                                 int32_t stride, int32_t batch_cones,
                                 void* stream, dg4_graph** out);

/* Tables of a graph, borrowed host pointers valid until dg4_graph_free. */
typedef enum {
    DG4_LEVEL = 0,      /* int32  [n_nodes]                                    */
    DG4_ORDER = 1,      /* int32  [n_nodes]      ids by (level, id)            */
    DG4_LEVEL_PTR = 2,  /* int64  [n_levels + 1] first position of each level  */
    DG4_NBR_PTR = 3,    /* int64  [n_nodes + 1]                                */
    DG4_NBR_IDX = 4,    /* int32  [nnz]                                        */
    DG4_NBR_REL = 5,    /* uint8  [nnz]                                        */
    /* The order in which a sweep over ALL levels processes the gates on the device: tiles of at
     * most 16 gates (2, 4 or 8 on circuits with few gates per dependency level, where small tiles
     * shorten the chain from level to level), each gate after every gate of its neighbour row
     * (list scheduling over the real dependencies; the level only breaks ties). For inspection
     * and tests; the embeddings do not depend on it. Built on first request. */
    DG4_FLOW_ORDER = 6,     /* int32 [n_nodes]     node ids in processing order          */
    DG4_FLOW_TILE_PTR = 7,  /* int64 [n_tiles + 1] first position of each tile           */
    /* Fanout counts of the structural encoding (Section 3.5, Eq. 2), see dg4_struct_encode. */
    DG4_OUT_AND = 8,        /* int32 [n_nodes]                                           */
    DG4_OUT_NOT = 9,        /* int32 [n_nodes]                                           */
    /* The processing order of sweeps with DG4_FFN and of the streaming dataflow kernel: tiles 2k and
     * 2k+1 (at most 16 gates each; 8 on narrow circuits) form a pair without dependencies between
     * them (the second may be empty). Built on first request. For inspection and tests. */
    DG4_PAIR_ORDER = 10,    /* int32 [n_nodes]                                           */
    DG4_PAIR_TILE_PTR = 11, /* int64 [n_tiles + 1], n_tiles even                         */
    /* Graphs from dg4_build_partitioned only (EINVAL otherwise): Algorithm 1's lists and the
     * running number of the mini-batch that computes each gate. */
    DG4_CONE_ROOT = 12,        /* int32 [n_cones]      roots, list after list                */
    DG4_CONE_GROUP_LEVEL = 13, /* int32 [n_lists]      level of each list, ascending         */
    DG4_CONE_GROUP_PTR = 14,   /* int64 [n_lists + 1]  first cone of each list               */
    DG4_STAGE = 15,            /* int32 [n_nodes]      (marks = 1 only)                      */
    /* marks = 0 only: the gate each copy stands for, and each gate's copy in the last mini-batch
     * that holds it. */
    DG4_COPY_OF = 16,          /* int32 [n_copies]                                           */
    DG4_LAST_COPY = 17         /* int32 [n_gates]                                            */
} dg4_array;

int dg4_graph_array(const dg4_graph* g, int which, const void** host_ptr, int64_t* count);
int dg4_graph_info(const dg4_graph* g, int64_t* n_nodes, int64_t* n_levels, int64_t* nnz, int32_t* hops);

/* Copy the neighbour tables to the current device now (otherwise done lazily
 * by the first device call). EHIP / ENOMEM on failure. */
int dg4_graph_upload(dg4_graph* g);
void dg4_graph_free(dg4_graph* g);

/*
 * Bytes of device workspace the calls below need (256-byte aligned buffers).
 * dg4_layer_workspace_bytes covers dg4_layer_fwd: packed weights, the
 * projected self rows, the per-layer K/V store of finished gates and the
 * level-sorted copy of H. Negative dg4_status on a bad configuration.
 */
int64_t dg4_proj_workspace_bytes(const dg4_layer_cfg* cfg);
int64_t dg4_ffn_workspace_bytes(const dg4_layer_cfg* cfg);
int64_t dg4_layer_workspace_bytes(const dg4_layer_cfg* cfg, const dg4_graph* g);

/*
 * Structural encoding (Section 3.5, Eq. 2), added to the initial embeddings:
 *   Xout[v] = X[v] + Emb_l(level(v)) + Emb_and(OutAND(v)) + Emb_not(OutNOT(v)),  Emb(s) = s*w + b,
 * OutAND(v) / OutNOT(v) = numbers of AND / NOT gates among the direct fanouts of v. With inverters
 * as edge flags: a fanout with in-degree 1 is a NOT/buffer gate; all inverted edges from v into AND
 * gates stand for the ONE inverter of v (counted once), plain edges into AND gates count one each.
 * level(v) is the graph's level (Eq. 1 or the hint). fp32 arithmetic, one rounding to cfg->dtype.
 *   X, Xout [n, hidden] device (may be the same buffer); emb: device float [6, hidden] = w_l, b_l,
 *   w_and, b_and, w_not, b_not. cfg: hidden, heads, dtype are used.
 */
int dg4_struct_encode(const dg4_layer_cfg* cfg, dg4_graph* g, const void* X, const float* emb,
                      void* Xout, void* stream);

/*
 * Q = S Wq, K = S Wk, V = S Wv for rows [row_begin, row_end) of S (the
 * projection at the head of the attention block, Section 3.5; no biases).
 *   S [n, hidden] device; Wqkv [hidden, 3*hidden] device, row-major, columns
 *   Wq | Wk | Wv, same dtype; Q, K, V [n, hidden] device (rows outside the
 *   range untouched). bf16: bf16 inputs, fp32 accumulation, bf16 outputs.
 */
int dg4_qkv_proj(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                 const void* Wqkv, void* Q, void* K, void* V,
                 void* workspace, int64_t workspace_bytes, void* stream);

/*
 * dg4_qkv_proj for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc. Same arguments, meaning and results (bit for bit)
 * as dg4_qkv_proj, but no workspace: the packed copy of the weight goes into a device array inside
 * the library, dg4_static_scratch_bytes() = 512 KB per GPU, held until the process ends. The call
 * allocates and frees nothing. EWORKSPACE if the packed weight does not fit (fp32 with hidden 256:
 * 768 KB), before anything is queued. Every call on a GPU shares that GPU's array, so two calls that
 * overlap in time on one GPU (different streams or threads) race; calls on one stream are safe, each
 * rewrites what it reads.
 */
int64_t dg4_static_scratch_bytes(void);
int dg4_qkv_proj_static(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                        const void* Wqkv, void* Q, void* K, void* V, void* stream);

/*
 * The position-wise feed-forward sub-block that follows the attention sub-block in the
 * transformer layer (Section 3.5: the attention module is replaced, the rest of the transformer
 * structure is kept), for rows [row_begin, row_end) of S:
 *   Out[r] = LayerNorm(S[r] + max(S[r] W1, 0) W2)      (no biases, no affine, biased variance)
 *   S, Out [n, hidden] device (rows outside the range untouched; Out may not alias S);
 *   W1 [hidden, 4*hidden], W2 [4*hidden, hidden] device, row-major, cfg->dtype.
 * bf16: bf16 inputs and hidden activations, fp32 accumulation and LayerNorm, bf16 output.
 * workspace: dg4_ffn_workspace_bytes (the two weights in matrix-core operand order).
 */
int dg4_ffn_fwd(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                const void* W1, const void* W2, void* Out,
                void* workspace, int64_t workspace_bytes, void* stream);

/*
 * Attention restricted to the cone (Section 3.5), for destination rows
 * [row_begin, row_end): for each head h of 32 features
 *   s[u]   = <Q[v,h], K[u,h]> / sqrt(32) + rel_bias[h][rel(v,u)],  u in N(v)
 *   alpha  = softmax_u s[u]          (fp32; a single-source row has alpha = 1, Section 3.7)
 *   A[v,h] = sum_u alpha[u] V[u,h]
 * scores and alpha live in registers only. rel_bias: device float [heads, 4].
 */
int dg4_sparse_attn_fwd(const dg4_layer_cfg* cfg, dg4_graph* g, int64_t row_begin, int64_t row_end,
                        const void* Q, const void* K, const void* V, const float* rel_bias,
                        void* A, void* stream);

/*
 * The level sweep of the updating strategy (Section 3.4, Algorithm 2 with
 * every level a root level): for levels [level_begin, level_end) ascending,
 * every gate of the level is computed exactly once; its cone sources are read
 * at their FINAL embedding H (the historical embeddings of Fig. 2), the gate
 * itself at its running state. Per gate, for layer l = 0..n_layers-1 (all
 * layers of a gate before the next level):
 *   s_0 = X[v];  q, k_self, v_self = s_l Wqkv_l;  k_u, v_u = H[u] Wk_l, H[u] Wv_l
 *   a = attention as in dg4_sparse_attn_fwd;  s_{l+1} = LayerNorm(s_l + a Wo_l)
 * (no affine, biased variance) and H[v] = s_{n_layers}, stored in cfg->dtype.
 *   X [n, hidden] device; Hout [n, hidden] device. With level_begin > 0, Hout
 *   must already hold the rows of all lower levels (resume).
 *   W: HOST array of 3*n_layers DEVICE pointers: Wqkv_l [hidden,3*hidden],
 *   Wo_l [hidden,hidden] (cfg->dtype), rel_bias_l float [heads,4].
 * With DG4_FFN the layer is the whole transformer block: after the LayerNorm above,
 *   s_{l+1} <- LayerNorm(s_{l+1} + max(s_{l+1} W1_l, 0) W2_l)   (as in dg4_ffn_fwd),
 * and W holds 5*n_layers pointers: Wqkv_l, Wo_l, rel_bias_l, W1_l [hidden,4*hidden],
 * W2_l [4*hidden,hidden].
 * The workspace contents are scratch; nothing a caller may rely on persists between calls, except
 * under DG4_WEIGHTS_PACKED.
 * On a graph from dg4_build_partitioned the same sweep realises Algorithm 2 in general (the rows
 * of the graph are what each gate's first mini-batch shows of its cone).
 * The order in which a sweep over ALL levels visits the gates is the library's (dependency-driven
 * tiles in the persistent kernels, Eq. 1 levels in level-by-level launches) and does not change a
 * bit of the result; DG4_LEVEL_ORDER forces the graph's own levels (for comparisons).
 * Persistent sweeps (everything but DG4_PER_LEVEL, DG4_BOUNDED_KV and DG4_FFN on rows wider than 16
 * entries, which run level by level) hand tiles of gates to resident workgroups, which wait for the
 * tiles their gates read from. Should such a wait exceed cfg->spin_limit polls (it cannot, unless
 * the device is taken away from the kernel), the sweep stops, Hout is left incomplete, and the
 * call has long returned DG4_OK: dg4_layer_status tells.
 */
int dg4_layer_fwd(const dg4_layer_cfg* cfg, dg4_graph* g, const void* X, const void* const* W,
                  int32_t level_begin, int32_t level_end, void* Hout,
                  void* workspace, int64_t workspace_bytes, void* stream);

/*
 * Whether the last dg4_layer_fwd on `workspace` (same cfg and graph) ran to completion. Synchronous:
 * the caller has synchronised the stream; four bytes are copied from the workspace. DG4_OK, or
 * DG4_EABORTED if a persistent sweep gave up on a dependency wait (Hout is then incomplete).
 */
int dg4_layer_status(const dg4_layer_cfg* cfg, const dg4_graph* g, const void* workspace);

/*
 * Tracing aid for the persistent sweep kernel of dg4_layer_fwd. Synchronous:
 * copies from `workspace` (as left by the last dg4_layer_fwd with the same cfg
 * and graph, after the caller synchronised the stream) the abort flag of the
 * kernel's bounded dependency wait (0 = the sweep ran to completion) and, if
 * DG4_PROFILE was set in that call's cfg->flags, eight
 * per-phase timers in 10 ns ticks summed over workgroups: tiles with a late source (a count), dependency
 * wait, attention, output projection, LayerNorm, K|V projection, publish, feed-forward sub-block.
 */
int dg4_layer_profile(const dg4_layer_cfg* cfg, const dg4_graph* g, const void* workspace,
                      uint64_t* ticks8, uint32_t* aborted);

/*
 * Tracing aid: device time in milliseconds of the persistent sweep kernel of the most recent
 * dg4_layer_fwd (of any thread) that ran one with DG4_TIME_SWEEP in cfg->flags (two events recorded
 * on the caller's stream around that one kernel). Waits for the kernel. EINVAL if no such call
 * has been made.
 */
int dg4_sweep_elapsed_ms(float* ms);

const char* dg4_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* DG4_H */
