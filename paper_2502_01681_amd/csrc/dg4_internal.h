// Internal declarations shared by the host graph builder, the entry points and
// the kernel launchers. Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <memory>
#include <type_traits>
#include <mutex>
#include <vector>

#include "dg4.h"

// Neighbour rows on the device: fixed-width rows of packed 32-bit entries
// (relation code << 30 | index), padded with DG4_ELL_PAD. Width = 2^(hops+1), at least 8:
// one more than the largest cone (Section 3.2), so a row always ends in a pad.
#define DG4_ELL_PAD 0xFFFFFFFFu
// tiles of one dependency level that the schedule of the register-resident kernel aims to stay below (1.25 x the 256
// compute units: measured on circuits of 264 ... 3092 gates per level)
#define DG4_SCHED_TILES_PER_LEVEL 320
#define DG4_MAX_LAYERS 16        // the paper stacks 12 (Section 4.1)
#define DG4_TILE_ROWS 16          // gates per tile of the persistent sweep
#define DG4_MAX_SWEEP_GROUPS 1024 // most workgroups the persistent sweep is launched with (one per compute unit)

struct dg4_graph {
    int64_t n = 0, e = 0, nnz = 0;
    int32_t hops = 0, max_level = 0;
    std::vector<int32_t> level, order;           // order: ids by (level, id)
    std::vector<int32_t> pos;                    // pos[id] = position in the level-ordered device processing order (set at upload)
    std::vector<int32_t> sweep_order;            // its inverse: position -> id
    std::vector<int64_t> level_ptr, nbr_ptr;
    std::vector<int32_t> out_and, out_not;       // fanout counts of the structural encoding (Eq. 2)
    int32_t* d_struct = nullptr;                 // device [n][3]: level, OutAND, OutNOT (on first dg4_struct_encode)
    std::vector<int32_t> nbr_idx;
    std::vector<uint8_t> nbr_rel;
    // Partitioned graphs (dg4_build_partitioned): Algorithm 1's lists; with marks the mini-batch of
    // each gate; without marks the nodes are copies: the gate each stands for, each gate's last copy.
    int32_t stride = 0, batch_cones = 0;
    bool marks = true;
    std::vector<int32_t> cone_root, cone_group_level, stage;
    std::vector<int64_t> cone_group_ptr;
    std::vector<int32_t> copy_of, last_copy;
    // Graphs built with a caller's levelling that is deeper than Eq. 1: the Eq. 1 levels and the
    // tables of a (Eq. 1 level, id) order, for level-by-level sweeps over ALL levels, which then
    // take as many rounds of launches as the circuit is deep, not as the levelling is. Host part at
    // build time, device tables on first use.
    std::vector<int32_t> eq1_level;
    std::vector<int64_t> eq1_level_ptr;      // empty: no such order
    int32_t* d_order_eq1 = nullptr;          // [n] position -> node id
    uint32_t* d_ell_eq1 = nullptr;           // [n, ell_w] rows and entries by position in that order

    // device mirror (one device), created once under `mu`
    std::mutex mu;
    bool on_device = false;
    int device = -1;
    int ell_w = 0;
    uint32_t* d_ell_id = nullptr;    // [n, ell_w] rows and entries by node id
    uint32_t* d_ell_pos = nullptr;   // [n, ell_w] rows and entries by position
    int32_t* d_order = nullptr;      // [n] position -> node id in the device processing order
    // tiles of the persistent sweep: runs of <= DG4_TILE_ROWS positions inside one level
    std::vector<int64_t> level_tile_ptr;   // [n_levels + 1] first tile of each level
    uint2* d_tiles = nullptr;        // [n_tiles] (first position, rows)
    // the same with runs of <= 32 positions (the persistent kernel for every shape), and, for rows wider
    // than 16 entries, of <= wide_tile_rows positions (on first use)
    std::vector<int64_t> level_tile32_ptr;
    uint2* d_tiles32 = nullptr;
    int wide_tile_rows = 0;
    std::vector<int64_t> level_tilew_ptr;
    uint2* d_tilesw = nullptr;
    // A second processing order for sweeps over ALL levels: tiles filled by list scheduling over
    // the real dependencies (a gate goes as early as its sources allow, sources long finished
    // first), not level by level. Host copy (node ids in processing order, first position of
    // each tile), then device tables with the layout of the three above.
    // Frontier tables for sweeps without a K|V store (DG4_BOUNDED_KV), built on first use: per level
    // the distinct sources of its gates (node ids, ascending position), and neighbour rows whose
    // entries index that list.
    bool has_frontier = false;
    std::vector<int64_t> front_ptr;      // [n_levels + 1]
    int64_t front_max = 0;               // largest frontier of a level
    int32_t* d_front_id = nullptr;       // [front_ptr.back()] node ids
    uint32_t* d_ell_front = nullptr;     // [n, ell_w] by position, entries rel << 30 | index in the level's frontier
    std::vector<int32_t> flow_order;
    std::vector<int64_t> flow_tile_ptr;
    uint32_t* d_flow_ell = nullptr;
    int32_t* d_flow_order = nullptr;
    uint2* d_flow_tiles = nullptr;
    int64_t n_flow_tiles = 0;
    // The same kind of order with tiles in independent PAIRS (2k, 2k+1; the second may be empty),
    // for sweeps with the feed-forward sub-block; built on first use.
    std::vector<int32_t> pair_order;
    std::vector<int64_t> pair_tile_ptr;
    uint32_t* d_pair_ell = nullptr;
    int32_t* d_pair_order = nullptr;
    uint2* d_pair_tiles = nullptr;
    int64_t n_pair_tiles = 0;
};

// dg4_qkv_proj in two parts (dg4_api.cpp): the argument checks that do not concern the workspace, and
// the launches, which allocate nothing; shared with dg4_qkv_proj_static.
#define DG4_STATIC_SCRATCH_BYTES (512 * 1024)
int dg4_qkv_proj_check(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                       const void* Wqkv, const void* Q, const void* K, const void* V);
int dg4_qkv_proj_run(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                     const void* Wqkv, void* Q, void* K, void* V, void* packed, hipStream_t s);

int dg4_graph_ensure_device(dg4_graph* g);
int dg4_flow_schedule(dg4_graph* g);   // caller holds g->mu
int dg4_pair_schedule(dg4_graph* g);   // caller holds g->mu
int dg4_graph_ensure_frontier(dg4_graph* g);           // after dg4_graph_ensure_device
int dg4_graph_ensure_struct(dg4_graph* g);
int dg4_graph_ensure_pairs(dg4_graph* g);              // after dg4_graph_ensure_device
int dg4_graph_ensure_wide_tiles(dg4_graph* g);         // after dg4_graph_ensure_device; graphs with rows wider than 16 entries
int dg4_graph_ensure_eq1(dg4_graph* g);                // after dg4_graph_ensure_device; needs eq1_level_ptr

// ---- structural encoding (dg4_kernels.hip) ----
int dg4_launch_struct_encode(int dtype, int hidden, const void* x, const int32_t* feat, const float* emb, void* out,
                             int64_t n, hipStream_t s);

// ---- kernel launchers (dg4_kernels.hip). All return a hipError_t as int. ----

struct dg4_attn_args {
    const void* q; int64_t q_stride;        // row r of Q at q + r*q_stride elements
    const void* k_self; const void* v_self; int64_t self_stride;   // rows by destination row
    const void* k_src; const void* v_src; int64_t src_stride;      // rows by neighbour index
    const float* rel_bias;                  // [heads,4]
    const uint32_t* ell; int ell_w;
    void* a; int64_t a_stride;
    int64_t row_begin, row_end;
};
int dg4_launch_attn(int dtype, int hidden, const dg4_attn_args& a, hipStream_t s);

// Re-tile columns [col0, col0+n_cols) of a row-major weight with `ld` columns
// and k_dim rows into MFMA B-operand order (n_cols % 32 == 0).
int dg4_launch_pack_w(int dtype, const void* w, int ld, int col0, int n_cols, int k_dim, void* packed, hipStream_t s);

struct dg4_gemm_args {
    const void* a; int64_t a_stride;        // input rows; row r at a + idx(r)*a_stride
    const int32_t* a_gather;                // nullable: idx(r) = a_gather[r], else r
    const void* w_packed; int n_cols;       // packed [hidden, n_cols]
    // output: column block j (of `hidden` columns) of row r goes to
    // out[j] + oidx(r)*out_stride
    void* out[2 * DG4_MAX_LAYERS + 3]; int64_t out_stride;
    const int32_t* out_scatter;             // nullable: oidx(r) = out_scatter[r]
    int64_t row_begin, row_end;
    // epilogue (n_cols == hidden only): out = LN(resid + acc)
    int epilogue;                           // 0 plain, 1 residual + LayerNorm
    const void* resid; int64_t resid_stride; const int32_t* resid_gather;
    void* out2; int64_t out2_stride;        // nullable second copy, indexed by r
    float ln_eps;
    int split;                              // set by the launcher: waves of a workgroup share rows and split the columns
    // Optional second product behind the epilogue (shapes for which dg4_gemm_fuses_kv() holds):
    // [K | V] = y * kv_w_packed (packed [hidden, 2*hidden]) for the normalised rows y, row r to
    // kv_out + r*kv_stride. The same bits as a separate launch over the stored rows.
    const void* kv_w_packed; void* kv_out; int64_t kv_stride;
};
int dg4_launch_gemm(int dtype, int hidden, const dg4_gemm_args& a, hipStream_t s);
bool dg4_gemm_fuses_kv(int dtype, int hidden);
int dg4_launch_attn_gemm(int dtype, int hidden, const dg4_attn_args& att, const dg4_gemm_args& a, hipStream_t s);

// Feed-forward sub-block: out = LN(h + max(h W1, 0) W2) for rows [row_begin, row_end).
struct dg4_ffn_args {
    const void* h; int64_t h_stride;        // input rows, row r at h + r*h_stride
    const void* w1_packed;                  // W1 [hidden, 4*hidden] in dg4_launch_pack_w order
    const void* w2_packed;                  // W2 [4*hidden, hidden] in dg4_launch_pack_w2 order
    void* out; int64_t out_stride;          // row r goes to out + oidx(r)*out_stride
    const int32_t* out_scatter;             // nullable: oidx(r) = out_scatter[r], else r
    void* out2; int64_t out2_stride;        // nullable second copy, indexed by r
    int64_t row_begin, row_end;
    float ln_eps;
};
int dg4_launch_pack_w2(int dtype, const void* w2, int hidden, void* packed, hipStream_t s);
int dg4_launch_ffn(int dtype, int hidden, const dg4_ffn_args& a, hipStream_t s);
// bf16, hidden 256, many rows: W1 | W2 as ONE stream in w1_packed (dg4_launch_pack_ffn_bulk order), w2_packed unused
int dg4_launch_pack_ffn_bulk(const void* w1, const void* w2, void* packed, hipStream_t s);
int dg4_launch_ffn_bulk(const dg4_ffn_args& a, hipStream_t s);

// ---- persistent sweep (dg4_sweep.hip): bf16, hidden 256, one layer ----
struct dg4_sweep_args {
    const uint2* tiles; int64_t tile_begin; int64_t n_tiles;   // tile t of the sweep is tiles[tile_begin + t]
    const uint32_t* ell; int ell_w;        // neighbour rows by position
    const int32_t* order;                  // position -> node id
    const uint16_t* x;                     // [n, 256] by node id
    const uint16_t* qkv_self;              // [n, 768] by position: Q | K | V of x
    uint16_t* kv;                          // [n, 512] by position: K | V of the final embeddings
    uint16_t* h_out;                       // [n, 256] by node id
    const void* wo_packed; const void* wkv_packed;   // pack_wt order
    const void* ffn_packed;                // nullable: W1 | W2 of the feed-forward sub-block, dg4_launch_pack_ffn order (1 MB);
                                           // the tile table then lists PAIRS (2k, 2k+1) of mutually independent tiles
    uint16_t* park;                        // with ffn_packed: [workgroups, 16, 256] rows parked between the tiles of a pair
    const float* rel_bias;
    uint32_t* flags;                       // [n] by position: 1 = rows published
    uint32_t* ctrl;                        // [1] abort flag, [16..31] phase timers
    uint64_t* prof;                        // nullable: 8 phase timers (100 MHz ticks, summed over workgroups)
    float ln_eps; int epilogue;
    int eager_publish;                     // raise a tile's flags as soon as its rows are written (level-ordered tiles: readers are close)
    uint32_t spin_limit;
};
int dg4_launch_pack_wt(const void* w, int ld, int col0, int ntw, int waves, void* packed, hipStream_t s);
int dg4_launch_pack_ffn(const void* w1, const void* w2, void* packed, hipStream_t s);   // [256,1024], [1024,256] bf16
// flags[i] = i < done_below for i < n_flags; the control words (abort, ticket counter, timers) = 0
int dg4_launch_sweep_init(uint32_t* flags, uint32_t* ctrl, int64_t n_flags, int64_t done_below, hipStream_t s);
int dg4_launch_sweep(const dg4_sweep_args& a, hipStream_t s);

// ---- persistent dataflow sweep for every shape and any number of layers (dg4_flow.hip) ----
struct dg4_flow_args {
    const uint2* tiles; int64_t tile_begin; int64_t n_tiles;   // tile t is tiles[tile_begin + t] = (first position, rows <= 32) ...
    int pairs;                             // ... or (pairs != 0) entries 2t and 2t+1 of the table together
    int64_t n_pre; int64_t pre_rows;       // resumed sweeps: positions [0, pre_rows) are finished gates whose K | V come from h_out first, in n_pre = ceil(pre_rows / 32) extra tiles
    const uint32_t* ell; int ell_w;        // neighbour rows by position
    int tile_rows;                         // rows wider than 16 entries: most gates of a tile (2, 4, 8 or 16; no pairs)
    int tile_cap;                          // most gates of any tile of this launch: 16 (one block) or 32
    int layer_flags;                       // a gate's flag goes up layer by layer (its count of stored layers), not once at the end
    const int32_t* order;                  // position -> node id
    const void* x;                         // [n, d] by node id
    const void* qkv_self;                  // [n, 3d] by position: Q | K | V of x (layer 0)
    void* kv; int64_t kv_layer_stride;     // [layers][n, 2d] by position: K | V of the final embeddings; elements between layers
    void* h_out;                           // [n, d] by node id
    const void* wqkv_packed; const void* wo_packed; int64_t w_layer_stride;   // dg4_launch_pack_wa order; bytes from a layer's to the next's
    const void* wkv_packed;                // [layers][d, 2d] in dg4_launch_pack_wa order: K | V columns of every layer
    int ffn;                               // the feed-forward sub-block after every attention sub-block (rows of at most 16 entries)
    const void* w1_packed;                 // per layer W1 [d, 4d] in dg4_launch_pack_wa order ...
    const void* w2_packed;                 // ... and W2 [4d, d] as four [d, d] blocks of d input rows each, same order
    int64_t ffn_layer_stride;              // bytes from a layer's W1 (W2) to the next's
    const float* rel_bias;                 // [layers][heads, 4]
    uint32_t* flags;                       // [n] by position: 1 = rows published
    uint32_t* ctrl;                        // [1] abort word, [2] ticket counter
    uint64_t* prof;                        // nullable: 8 phase timers (10 ns ticks, summed over workgroups)
    int n_layers;
    float ln_eps; int epilogue; int project_kv;
    uint32_t spin_limit;
};
bool dg4_flow_supports(int dtype, int hidden, int ell_w);
int dg4_launch_pack_wa(int dtype, int hidden, const void* w, int ld, int col0, int n_cols, void* packed, hipStream_t s);
int dg4_launch_flow(int dtype, int hidden, const dg4_flow_args& a, hipStream_t s);

// ---- bulk projection on the matrix cores (dg4_sweep.hip): bf16, hidden 256 ----
struct dg4_bulk_args {
    const uint16_t* src;                   // [*, 256] input rows
    const int32_t* gather;                 // nullable: input row of output row r is gather[r]
    const void* w_packed; int n_cols;      // pack_w32 order; n_cols == 768
    uint16_t* out[2 * DG4_MAX_LAYERS + 3]; // column block j (256 columns) of row r at out[j] + r*out_stride
    int64_t out_stride;
    int64_t row_begin, row_end;
};
int dg4_launch_pack_w32(const void* w, int ld, void* packed, hipStream_t s);   // [256, 768] weights, row stride ld
int dg4_launch_bulk_proj(const dg4_bulk_args& a, hipStream_t s);

// Every kernel takes its argument block by value: plain data of pointer alignment, well inside the
// kernel-argument segment (4 KB), value-initialised by every caller before the fields are set.
#define DG4_CHECK_KERNEL_ARGS(S) \
    static_assert(std::is_trivially_copyable<S>::value && std::is_standard_layout<S>::value && alignof(S) == 8 && sizeof(S) <= 1024, #S)
DG4_CHECK_KERNEL_ARGS(dg4_attn_args);
DG4_CHECK_KERNEL_ARGS(dg4_gemm_args);
DG4_CHECK_KERNEL_ARGS(dg4_ffn_args);
DG4_CHECK_KERNEL_ARGS(dg4_sweep_args);
DG4_CHECK_KERNEL_ARGS(dg4_flow_args);
DG4_CHECK_KERNEL_ARGS(dg4_bulk_args);
#undef DG4_CHECK_KERNEL_ARGS
