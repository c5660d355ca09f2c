/*
 * CPU oracle for the sparse graph-attention layer over an And-Inverter Graph.
 *
 * TEST INFRASTRUCTURE ONLY. This file is the slow, plain, double-precision
 * statement of what the layer computes. Only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it; the GPU library shares no
 * code with it and never falls back to it.
 *
 * What follows the paper, and where:
 *   - logic level                      : Section 3.2, Eq. 1
 *   - cone_k(v) and its size bound     : Section 3.2 (partial order <=_k)
 *   - attention restricted to cone_k(v), realised as virtual edges
 *                                      : Section 3.5 "GAT-based Sparse Attention"
 *   - level-ordered sweep, every gate computed once, earlier gates frozen and
 *     read from the historical store   : Section 3.4, Algorithm 2, Fig. 2
 *   - a row with a single source has alpha = 1 : Section 3.7
 *
 * Readings taken where the paper is silent (it prints no attention formula
 * and the block diagram is a figure):
 *   R1  in-degree 0, 1 or 2 accepted; a duplicated (src,dst) pair, a self loop
 *       or an id out of range is an error.
 *   R2  the sweep schedule is Eq. 1 unless the caller supplies a levelling
 *       that is checked to be topological (PI = 0, every edge goes upward).
 *   R3  nodes inside a level are ordered by ascending id.
 *   R4  a neighbour row is stored by ascending id, the node itself included.
 *   R5  inverter flags enter as an additive per-head logit bias indexed by a
 *       relation code: 0 self, 1 direct fanin, 2 direct inverted fanin,
 *       3 virtual edge (shortest path of 2 or more hops). The shortest hop wins.
 *   R6  LEVEL-MAJOR nesting for several layers: a node runs through all layers
 *       before the next level starts; in every layer its sources are read at
 *       their FINAL embedding H_u, the node itself at its running state.
 *   R7  the block is attention + output projection + residual + LayerNorm
 *       without affine parameters (biased variance, eps inside the root);
 *       epilogue=0 returns the bare projection instead.
 *   R8  scores are scaled dot products <q,k>/sqrt(d_head).
 *   R9  softmax subtracts the row maximum; natural exponential.
 *   R10 no projection biases.
 *   R12 arithmetic is double throughout; the only rounding is of H when it is
 *       stored (to float or to bfloat16), because the storage format of the
 *       historical embeddings is part of the problem.
 *   R15 structural encoding (Section 3.5, Eq. 2) on a graph whose inverters are edge
 *       flags: a fanout node with in-degree 1 is a NOT/buffer gate; all inverted
 *       edges leaving v into AND gates stand for ONE inverter fed by v (structural
 *       hashing keeps one NOT per signal), and the ANDs behind it are fanouts of that
 *       inverter, not of v. So OutNOT(v) = #fanouts with in-degree 1 + [v has an
 *       inverted edge into an AND], OutAND(v) = #non-inverted edges into ANDs. Each
 *       Emb is a linear layer on a scalar, s*w + b; the encoding is added to the
 *       initial embedding.
 *   R16 Section 3.5 swaps the attention module for a GAT module and keeps the rest of the
 *       transformer layer as it is; read as the post-norm encoder block: after the attention sub-block h = LN(s + a Wo) comes the position-wise
 *       feed-forward sub-block s' = LN(h + max(h W1, 0) W2), W1 [d, 4d], W2 [4d, d],
 *       rectifier, no biases (R10), LayerNorm as in R7. Optional: a layer without
 *       W1 / W2 is the attention sub-block alone.
 *   R17 general partition and updating strategy (Section 3.3, Algorithm 1; Section 3.4,
 *       Algorithm 2) at inference. The gates of a level are visited by ascending id; a
 *       cone is named by its root, so an out-degree-0 gate that already roots a cone of
 *       its level is not added twice; a gate that after both loops lies in no cone roots
 *       one of its own in the list of its level, as the out-degree-0 gates do (the
 *       partition is stated to cover the whole circuit). Lists are taken by ascending
 *       level, mini-batches are consecutive runs of B cones of a list (the last one may
 *       be short). In a mini-batch the cones are merged into one graph: a gate lying in
 *       several of its cones is computed once, over the union of its per-cone
 *       neighbourhoods {u in cone_i : u <=_k v}. Inside a mini-batch gates go by
 *       ascending level and read their sources at the sources' final embeddings (R6),
 *       from the historical store if marked, else as computed earlier in the batch.
 *       Without marks (the ablation of Section 4.4) every gate of every mini-batch is
 *       recomputed from its initial features inside that mini-batch and the last
 *       result stands.
 *
 * Parity pins live in tests/ (brute-force dense masked attention, closed
 * forms, hand-worked graphs, invariances). The numeric values of embeddings
 * are NOT pinned by the paper, which prints none: "parity unpinned" by the
 * paper, pinned by mathematics only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_ERANGE = -2, ORC_EFANIN = -3, ORC_ECYCLE = -4,
       ORC_EHINT = -5, ORC_ENOMEM = -6 };

enum { ORC_STORE_F64 = 0, ORC_STORE_F32 = 1, ORC_STORE_BF16 = 2 };

/* threads the parallel loops over the nodes of one level will use */
int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ graph */

/* R1: validate the edge list. */
int orc_validate(int64_t n, int64_t e, const int32_t* src, const int32_t* dst, const uint8_t* inv)
{
    if (n < 0 || e < 0 || (e > 0 && (!src || !dst || !inv))) return ORC_EINVAL;
    int32_t* first = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    uint8_t* deg = (uint8_t*)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!first || !deg) { free(first); free(deg); return ORC_ENOMEM; }
    int rc = ORC_OK;
    for (int64_t i = 0; i < e && rc == ORC_OK; ++i) {
        int64_t u = src[i], v = dst[i];
        if (u < 0 || u >= n || v < 0 || v >= n) { rc = ORC_ERANGE; break; }
        if (inv[i] > 1) { rc = ORC_EINVAL; break; }
        if (u == v) { rc = ORC_ECYCLE; break; }
        if (deg[v] == 2) { rc = ORC_EFANIN; break; }
        if (deg[v] == 1 && first[v] == u) { rc = ORC_EFANIN; break; }
        if (deg[v] == 0) first[v] = (int32_t)u;
        ++deg[v];
    }
    free(first); free(deg);
    return rc;
}

/* Eq. 1 by Kahn's algorithm: a node is finished once all its fanins are. */
int orc_levels(int64_t n, int64_t e, const int32_t* src, const int32_t* dst, int32_t* level)
{
    int64_t* out_ptr = (int64_t*)calloc((size_t)n + 2, sizeof(int64_t));
    int32_t* out_dst = (int32_t*)malloc(sizeof(int32_t) * (size_t)(e > 0 ? e : 1));
    int32_t* pending = (int32_t*)calloc((size_t)(n > 0 ? n : 1), sizeof(int32_t));
    int32_t* queue = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    if (!out_ptr || !out_dst || !pending || !queue) {
        free(out_ptr); free(out_dst); free(pending); free(queue); return ORC_ENOMEM;
    }
    for (int64_t i = 0; i < e; ++i) { ++out_ptr[src[i] + 2]; ++pending[dst[i]]; }
    for (int64_t v = 0; v < n; ++v) out_ptr[v + 2] += out_ptr[v + 1];
    for (int64_t i = 0; i < e; ++i) out_dst[out_ptr[src[i] + 1]++] = dst[i];
    /* now out edges of u are out_dst[out_ptr[u] .. out_ptr[u+1]) */
    int64_t head = 0, tail = 0;
    for (int64_t v = 0; v < n; ++v) { level[v] = 0; if (pending[v] == 0) queue[tail++] = (int32_t)v; }
    while (head < tail) {
        int32_t u = queue[head++];
        for (int64_t i = out_ptr[u]; i < out_ptr[u + 1]; ++i) {
            int32_t w = out_dst[i];
            if (level[u] + 1 > level[w]) level[w] = level[u] + 1;
            if (--pending[w] == 0) queue[tail++] = w;
        }
    }
    free(out_ptr); free(out_dst); free(pending); free(queue);
    return tail == n ? ORC_OK : ORC_ECYCLE;
}

/* R2: a caller-supplied levelling must be topological. */
int orc_check_hint(int64_t n, int64_t e, const int32_t* src, const int32_t* dst, const int32_t* hint)
{
    uint8_t* has_fanin = (uint8_t*)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!has_fanin) return ORC_ENOMEM;
    int rc = ORC_OK;
    for (int64_t i = 0; i < e; ++i) {
        has_fanin[dst[i]] = 1;
        if (hint[dst[i]] <= hint[src[i]]) rc = ORC_EHINT;
    }
    for (int64_t v = 0; v < n; ++v) {
        if (hint[v] < 0) rc = ORC_EHINT;
        if (!has_fanin[v] && hint[v] != 0) rc = ORC_EHINT;
    }
    free(has_fanin);
    return rc;
}

/* R3: order = ids sorted by (level, id); level_ptr[l] = first position of level l,
 * l = 0..max_level+1 (so max_level+2 entries). */
void orc_order(int64_t n, const int32_t* level, int32_t max_level, int32_t* order, int64_t* level_ptr)
{
    for (int32_t l = 0; l <= max_level + 1; ++l) level_ptr[l] = 0;
    for (int64_t v = 0; v < n; ++v) ++level_ptr[level[v] + 1];
    for (int32_t l = 0; l <= max_level; ++l) level_ptr[l + 1] += level_ptr[l];
    int64_t* cursor = (int64_t*)malloc(sizeof(int64_t) * ((size_t)max_level + 2));
    memcpy(cursor, level_ptr, sizeof(int64_t) * ((size_t)max_level + 2));
    for (int64_t v = 0; v < n; ++v) order[cursor[level[v]]++] = (int32_t)v;
    free(cursor);
}

/*
 * cone_k(v): all u with a path u -> v of at most `hops` edges, v included
 * (Section 3.2). Breadth-first search backwards over fanin edges; the first
 * time a node is reached fixes its shortest hop, hence its relation code (R5).
 * nbr_idx / nbr_rel may be NULL to only count. Returns NNZ (or < 0 on error).
 */
int64_t orc_cone_csr(int64_t n, int64_t e, const int32_t* src, const int32_t* dst, const uint8_t* inv,
                     int32_t hops, int64_t* nbr_ptr, int32_t* nbr_idx, uint8_t* nbr_rel)
{
    if (hops < 0 || hops > 8) return ORC_EINVAL;
    /* fanin lists in edge order */
    int32_t* fin = (int32_t*)malloc(sizeof(int32_t) * 2 * (size_t)(n > 0 ? n : 1));
    uint8_t* finv = (uint8_t*)malloc(2 * (size_t)(n > 0 ? n : 1));
    uint8_t* deg = (uint8_t*)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!fin || !finv || !deg) { free(fin); free(finv); free(deg); return ORC_ENOMEM; }
    for (int64_t i = 0; i < e; ++i) {
        int32_t v = dst[i];
        fin[2 * (int64_t)v + deg[v]] = src[i];
        finv[2 * (int64_t)v + deg[v]] = inv[i];
        ++deg[v];
    }
    enum { CAP = 1 << 9 };                    /* 2^(8+1)-1 < CAP */
    int32_t found[CAP]; uint8_t code[CAP]; int32_t hop[CAP];
    int64_t nnz = 0;
    for (int64_t v = 0; v < n; ++v) {
        int cnt = 0;
        found[cnt] = (int32_t)v; code[cnt] = 0; hop[cnt] = 0; ++cnt;
        for (int head = 0; head < cnt; ++head) {          /* found[] doubles as the BFS queue */
            if (hop[head] == hops) continue;
            int32_t w = found[head];
            for (int k = 0; k < deg[w]; ++k) {
                int32_t u = fin[2 * (int64_t)w + k];
                int seen = 0;
                for (int j = 0; j < cnt; ++j) if (found[j] == u) { seen = 1; break; }
                if (seen) continue;
                found[cnt] = u; hop[cnt] = hop[head] + 1;
                code[cnt] = hop[cnt] == 1 ? (uint8_t)(1 + finv[2 * (int64_t)w + k]) : 3;
                ++cnt;
            }
        }
        nbr_ptr[v] = nnz;
        if (nbr_idx) {
            /* R4: ascending id (insertion sort of a tiny row) */
            for (int i = 1; i < cnt; ++i) {
                int32_t fi = found[i]; uint8_t ci = code[i]; int j = i - 1;
                while (j >= 0 && found[j] > fi) { found[j + 1] = found[j]; code[j + 1] = code[j]; --j; }
                found[j + 1] = fi; code[j + 1] = ci;
            }
            for (int i = 0; i < cnt; ++i) { nbr_idx[nnz + i] = found[i]; nbr_rel[nnz + i] = code[i]; }
        }
        nnz += cnt;
    }
    nbr_ptr[n] = nnz;
    free(fin); free(finv); free(deg);
    return nnz;
}

/* ------------------------------------------------------------- arithmetic */

/* nearest bfloat16 (8 significant bits), ties to even, straight from double. */
static double round_bf16(double x)
{
    if (x == 0.0 || !isfinite(x)) return x;
    int ex;
    double m = frexp(x, &ex);                 /* |m| in [0.5, 1) */
    return ldexp(rint(ldexp(m, 8)), ex - 8);  /* rint: current mode = nearest even */
}

static double round_store(double x, int store)
{
    if (store == ORC_STORE_BF16) return round_bf16(x);
    if (store == ORC_STORE_F32) return (double)(float)x;
    return x;
}

/* y[j] = sum_i s[i] * W[i, col0 + j], W row-major with `ld` columns. */
static void vec_mat(const double* s, int d, const float* W, int ld, int col0, int ncols, double* y)
{
    for (int j = 0; j < ncols; ++j) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i) acc += s[i] * (double)W[(int64_t)i * ld + col0 + j];
        y[j] = acc;
    }
}

/* Q = S Wq, K = S Wk, V = S Wv with W = [Wq | Wk | Wv] of shape [d, 3d]. */
void orc_qkv_proj(int64_t rows, int32_t d, const float* S, const float* W, double* Q, double* K, double* V)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double s[1024];
        for (int i = 0; i < d; ++i) s[i] = (double)S[r * d + i];
        vec_mat(s, d, W, 3 * d, 0, d, Q + r * d);
        vec_mat(s, d, W, 3 * d, d, d, K + r * d);
        vec_mat(s, d, W, 3 * d, 2 * d, d, V + r * d);
    }
}

/*
 * scores, softmax and aggregation of one destination (R5, R8, R9).
 * q[d]; k, v: cnt rows of d; rel[cnt]; bias[heads*4]. a[d] out.
 * alpha (nullable): cnt*heads, alpha[j*heads + h].
 */
static void attend(int d, int heads, int cnt, const double* q, const double* k, const double* v,
                   const uint8_t* rel, const float* bias, double* a, double* alpha)
{
    const int dh = d / heads;
    const double scale = 1.0 / sqrt((double)dh);
    double sc[1 << 9];
    for (int h = 0; h < heads; ++h) {
        double mx = -INFINITY;
        for (int j = 0; j < cnt; ++j) {
            double dot = 0.0;
            for (int c = 0; c < dh; ++c) dot += q[h * dh + c] * k[(int64_t)j * d + h * dh + c];
            sc[j] = dot * scale + (double)bias[h * 4 + rel[j]];
            if (sc[j] > mx) mx = sc[j];
        }
        double z = 0.0;
        for (int j = 0; j < cnt; ++j) { sc[j] = exp(sc[j] - mx); z += sc[j]; }
        for (int c = 0; c < dh; ++c) a[h * dh + c] = 0.0;
        for (int j = 0; j < cnt; ++j) {
            double al = sc[j] / z;
            if (alpha) alpha[j * heads + h] = al;
            for (int c = 0; c < dh; ++c) a[h * dh + c] += al * v[(int64_t)j * d + h * dh + c];
        }
    }
}

/* Kernel-level oracle: attention on given Q, K, V (rows indexed by node id). */
void orc_sparse_attn(int64_t n, int32_t d, int32_t heads, int64_t row_begin, int64_t row_end,
                     const float* Q, const float* K, const float* V, const float* bias,
                     const int64_t* nbr_ptr, const int32_t* nbr_idx, const uint8_t* nbr_rel,
                     double* A /* [n,d], rows outside the range untouched */,
                     double* alpha /* nullable [nnz, heads] */)
{
    (void)n;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t r = row_begin; r < row_end; ++r) {
        int cnt = (int)(nbr_ptr[r + 1] - nbr_ptr[r]);
        double* q = (double*)malloc(sizeof(double) * (size_t)d * (2 * (size_t)cnt + 1));
        double* k = q + d; double* v = k + (size_t)cnt * d;
        for (int i = 0; i < d; ++i) q[i] = (double)Q[r * d + i];
        for (int j = 0; j < cnt; ++j) {
            int64_t u = nbr_idx[nbr_ptr[r] + j];
            for (int i = 0; i < d; ++i) { k[(int64_t)j * d + i] = (double)K[u * d + i]; v[(int64_t)j * d + i] = (double)V[u * d + i]; }
        }
        attend(d, heads, cnt, q, k, v, nbr_rel + nbr_ptr[r], bias, A + r * d,
               alpha ? alpha + nbr_ptr[r] * heads : NULL);
        free(q);
    }
}

typedef struct {
    int32_t d, heads, n_layers, store, epilogue;
    double ln_eps;
    const float* x;         /* [n, d] */
    const float* wqkv;      /* [n_layers, d, 3d] */
    const float* wo;        /* [n_layers, d, d] */
    const float* bias;      /* [n_layers, heads, 4] */
    const float* w1;        /* [n_layers, d, 4d] or NULL: no feed-forward sub-block (R16) */
    const float* w2;        /* [n_layers, 4d, d] */
    const int64_t* nbr_ptr; const int32_t* nbr_idx; const uint8_t* nbr_rel;
} orc_layer;

/* t <- LayerNorm(t): no affine parameters, biased variance, eps inside the root (R7) */
static void layer_norm(double* t, int d, double eps)
{
    double mean = 0.0, var = 0.0;
    for (int i = 0; i < d; ++i) mean += t[i];
    mean /= d;
    for (int i = 0; i < d; ++i) var += (t[i] - mean) * (t[i] - mean);
    var /= d;
    double r = 1.0 / sqrt(var + eps);
    for (int i = 0; i < d; ++i) t[i] = (t[i] - mean) * r;
}

/* R16: s <- LN(s + max(s W1, 0) W2), W1 [d, 4d], W2 [4d, d]; u (4d) and o (d) are scratch */
static void ffn_block(double* s, int d, const float* W1, const float* W2, double eps, double* u, double* o)
{
    vec_mat(s, d, W1, 4 * d, 0, 4 * d, u);
    for (int i = 0; i < 4 * d; ++i) if (u[i] < 0.0) u[i] = 0.0;
    vec_mat(u, 4 * d, W2, d, 0, d, o);
    for (int i = 0; i < d; ++i) s[i] += o[i];
    layer_norm(s, d, eps);
}

/* Kernel-level oracle of the feed-forward sub-block on given rows S [rows, d]. */
int orc_ffn(int64_t rows, int32_t d, const float* S, const float* W1, const float* W2, double ln_eps,
            int32_t store, double* out)
{
    if (d <= 0 || d > 1024) return ORC_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double s[1024], o[1024], u[4096];
        for (int i = 0; i < d; ++i) s[i] = (double)S[r * d + i];
        ffn_block(s, d, W1, W2, ln_eps, u, o);
        for (int i = 0; i < d; ++i) out[r * d + i] = round_store(s[i], store);
    }
    return ORC_OK;
}

/*
 * All layers of one node v (R6, R7, R16). Source states come from Hd (double rows)
 * if non-NULL, else from Hf (float rows). kv_memo (nullable): per layer and
 * node the already projected [K | V] row of the node's final embedding; it is
 * a pure function of H_u, so using it changes no value.
 */
static void node_step_row(const orc_layer* L, int64_t v, const int32_t* row_idx, const uint8_t* row_rel, int cnt,
                          const double* Hd, const float* Hf, const double* kv_memo, int64_t n, double* out)
{
    const int d = L->d;
    double* buf = (double*)malloc(sizeof(double) * (size_t)d * (2 * (size_t)cnt + 9));
    double *s = buf, *q = s + d, *a = q + d, *o = a + d, *src = o + d;
    double *k = src + d, *vv = k + (size_t)cnt * d, *u = vv + (size_t)cnt * d;   /* u: 4d */
    for (int i = 0; i < d; ++i) s[i] = (double)L->x[v * d + i];
    for (int l = 0; l < L->n_layers; ++l) {
        const float* W = L->wqkv + (int64_t)l * d * 3 * d;
        vec_mat(s, d, W, 3 * d, 0, d, q);
        for (int j = 0; j < cnt; ++j) {
            int64_t u = row_idx[j];
            if (u == v) {
                vec_mat(s, d, W, 3 * d, d, d, k + (int64_t)j * d);
                vec_mat(s, d, W, 3 * d, 2 * d, d, vv + (int64_t)j * d);
            } else if (kv_memo) {
                const double* m = kv_memo + ((int64_t)l * n + u) * 2 * d;
                memcpy(k + (int64_t)j * d, m, sizeof(double) * d);
                memcpy(vv + (int64_t)j * d, m + d, sizeof(double) * d);
            } else {
                for (int i = 0; i < d; ++i) src[i] = Hd ? Hd[u * d + i] : (double)Hf[u * d + i];
                vec_mat(src, d, W, 3 * d, d, d, k + (int64_t)j * d);
                vec_mat(src, d, W, 3 * d, 2 * d, d, vv + (int64_t)j * d);
            }
        }
        attend(d, L->heads, cnt, q, k, vv, row_rel, L->bias + (int64_t)l * L->heads * 4, a, NULL);
        vec_mat(a, d, L->wo + (int64_t)l * d * d, d, 0, d, o);
        if (L->epilogue) {
            for (int i = 0; i < d; ++i) s[i] += o[i];
            layer_norm(s, d, L->ln_eps);
        } else {
            for (int i = 0; i < d; ++i) s[i] = o[i];
        }
        if (L->w1)
            ffn_block(s, d, L->w1 + (int64_t)l * d * 4 * d, L->w2 + (int64_t)l * 4 * d * d, L->ln_eps, u, o);
    }
    for (int i = 0; i < d; ++i) out[i] = round_store(s[i], L->store);
    free(buf);
}

/* the same with the node's row of the layer's neighbour table */
static void node_step(const orc_layer* L, int64_t v, const double* Hd, const float* Hf,
                      const double* kv_memo, int64_t n, double* out)
{
    const int64_t p0 = L->nbr_ptr[v];
    node_step_row(L, v, L->nbr_idx + p0, L->nbr_rel + p0, (int)(L->nbr_ptr[v + 1] - p0), Hd, Hf, kv_memo, n, out);
}

/*
 * The level sweep (Algorithm 2 with every level a root level): levels in
 * [level_begin, level_end) ascending; inside a level nodes are independent.
 * H must already hold the embeddings of all levels < level_begin.
 * memo != 0 caches the projected K/V of finished nodes (same values, less work).
 */
int orc_layer_fwd(int64_t n, int32_t d, int32_t heads, int32_t n_layers, int32_t store,
                  int32_t epilogue, double ln_eps, int32_t memo,
                  const float* x, const float* wqkv, const float* wo, const float* bias,
                  const float* w1 /* nullable */, const float* w2 /* nullable with w1 */,
                  const int32_t* order, const int64_t* level_ptr, int32_t level_begin, int32_t level_end,
                  const int64_t* nbr_ptr, const int32_t* nbr_idx, const uint8_t* nbr_rel,
                  double* H)
{
    if (d <= 0 || d > 1024 || heads <= 0 || d % heads || n_layers <= 0) return ORC_EINVAL;
    if ((w1 == NULL) != (w2 == NULL) || (w1 && !epilogue)) return ORC_EINVAL;
    orc_layer L = { d, heads, n_layers, store, epilogue, ln_eps, x, wqkv, wo, bias, w1, w2, nbr_ptr, nbr_idx, nbr_rel };
    double* kv = NULL;
    if (memo) {
        kv = (double*)malloc(sizeof(double) * (size_t)n_layers * (size_t)n * 2 * (size_t)d);
        if (!kv) return ORC_ENOMEM;
        /* nodes finished before level_begin */
#pragma omp parallel for schedule(static)
        for (int64_t p = 0; p < level_ptr[level_begin]; ++p) {
            int64_t u = order[p];
            for (int l = 0; l < n_layers; ++l)
                vec_mat(H + u * d, d, wqkv + (int64_t)l * d * 3 * d, 3 * d, d, 2 * d,
                        kv + ((int64_t)l * n + u) * 2 * d);
        }
    }
    for (int32_t lev = level_begin; lev < level_end; ++lev) {
#pragma omp parallel for schedule(dynamic, 16)
        for (int64_t p = level_ptr[lev]; p < level_ptr[lev + 1]; ++p) {
            int64_t v = order[p];
            node_step(&L, v, H, NULL, kv, n, H + v * d);
            if (kv)
                for (int l = 0; l < n_layers; ++l)
                    vec_mat(H + v * d, d, wqkv + (int64_t)l * d * 3 * d, 3 * d, d, 2 * d,
                            kv + ((int64_t)l * n + v) * 2 * d);
        }
    }
    free(kv);
    return ORC_OK;
}

/*
 * One step for listed nodes with the sources' final embeddings GIVEN (Hsrc,
 * float rows by node id): the single-node definition, used to check sampled
 * outputs of a large run and for teacher-forced comparison.
 */
int orc_layer_nodes(int64_t n, int32_t d, int32_t heads, int32_t n_layers, int32_t store,
                    int32_t epilogue, double ln_eps,
                    const float* x, const float* wqkv, const float* wo, const float* bias,
                    const float* w1 /* nullable */, const float* w2 /* nullable with w1 */,
                    const int64_t* nbr_ptr, const int32_t* nbr_idx, const uint8_t* nbr_rel,
                    const float* Hsrc, const int64_t* nodes, int64_t n_listed, double* out /* [n_listed, d] */)
{
    if (d <= 0 || d > 1024 || heads <= 0 || d % heads || n_layers <= 0) return ORC_EINVAL;
    if ((w1 == NULL) != (w2 == NULL) || (w1 && !epilogue)) return ORC_EINVAL;
    orc_layer L = { d, heads, n_layers, store, epilogue, ln_eps, x, wqkv, wo, bias, w1, w2, nbr_ptr, nbr_idx, nbr_rel };
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < n_listed; ++i)
        node_step(&L, nodes[i], NULL, Hsrc, NULL, n, out + i * d);
    return ORC_OK;
}

/* ------------------------------------------------------------------------------------------
 * Graph partition (Section 3.3, Algorithm 1) and updating strategy (Section 3.4, Algorithm 2),
 * reading R17. cone_k(v) is passed in as the rows of orc_cone_csr (ascending id).
 */
typedef struct {
    int64_t n_groups, n_cones, n_entries;
    int32_t* group_level;   /* [n_groups]     level l of the list cones^l, ascending          */
    int64_t* group_ptr;     /* [n_groups + 1] first cone of each list                         */
    int32_t* cone_root;     /* [n_cones]      root of each cone, lists in order of insertion  */
    int64_t* cone_ptr;      /* [n_cones + 1]  into cone_node                                  */
    int32_t* cone_node;     /* [n_entries]    the gates of each cone, ascending id            */
} orc_cones;

void orc_cones_free(orc_cones* c)
{
    if (!c) return;
    free(c->group_level); free(c->group_ptr); free(c->cone_root); free(c->cone_ptr); free(c->cone_node);
    free(c);
}

/* Algorithm 1. Returns NULL on bad arguments or lack of memory. */
orc_cones* orc_partition(int64_t n, int64_t e, const int32_t* src, const int32_t* level,
                         int32_t k, int32_t delta, const int64_t* nbr_ptr, const int32_t* nbr_idx)
{
    if (n < 0 || k < 1 || delta < 1 || delta >= k) return NULL;
    const size_t n1 = (size_t)(n > 0 ? n : 1);
    int32_t* app_root = (int32_t*)malloc(sizeof(int32_t) * n1);     /* roots in order of insertion */
    uint8_t* is_root = (uint8_t*)calloc(n1, 1);
    uint8_t* in_cone = (uint8_t*)calloc(n1, 1);
    uint8_t* has_out = (uint8_t*)calloc(n1, 1);
    orc_cones* c = (orc_cones*)calloc(1, sizeof(orc_cones));
    if (!app_root || !is_root || !in_cone || !has_out || !c) goto fail;
    int64_t n_app = 0;
    int32_t L = 0;
    for (int64_t v = 0; v < n; ++v) if (level[v] > L) L = level[v];
    for (int64_t i = 0; i < e; ++i) has_out[src[i]] = 1;
    /* the cones that end at levels k, k + delta, ... */
    for (int32_t l = k; l <= L; l += delta)
        for (int64_t v = 0; v < n; ++v)
            if (level[v] == l) {
                app_root[n_app++] = (int32_t)v; is_root[v] = 1;
                for (int64_t j = nbr_ptr[v]; j < nbr_ptr[v + 1]; ++j) in_cone[nbr_idx[j]] = 1;
            }
    /* the cones of the gates nothing reads */
    for (int64_t v = 0; v < n; ++v)
        if (!has_out[v] && !is_root[v]) {
            app_root[n_app++] = (int32_t)v; is_root[v] = 1;
            for (int64_t j = nbr_ptr[v]; j < nbr_ptr[v + 1]; ++j) in_cone[nbr_idx[j]] = 1;
        }
    /* R17: what is still in no cone (decided here, before any of these cones is added) */
    for (int64_t v = 0; v < n; ++v)
        if (!in_cone[v]) { app_root[n_app++] = (int32_t)v; is_root[v] = 1; }
    /* the lists by ascending level, each in order of insertion */
    int64_t* per_level = (int64_t*)calloc((size_t)L + 2, sizeof(int64_t));
    if (!per_level) goto fail;
    for (int64_t i = 0; i < n_app; ++i) ++per_level[level[app_root[i]] + 1];
    int64_t groups = 0;
    for (int32_t l = 0; l <= L; ++l) if (per_level[l + 1]) ++groups;
    c->n_groups = groups; c->n_cones = n_app;
    c->group_level = (int32_t*)malloc(sizeof(int32_t) * (size_t)(groups + 1));
    c->group_ptr = (int64_t*)malloc(sizeof(int64_t) * (size_t)(groups + 1));
    c->cone_root = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_app + 1));
    c->cone_ptr = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_app + 1));
    if (!c->group_level || !c->group_ptr || !c->cone_root || !c->cone_ptr) { free(per_level); goto fail; }
    {
        int64_t gi = 0, at = 0;
        for (int32_t l = 0; l <= L; ++l) {
            const int64_t cnt = per_level[l + 1];
            per_level[l + 1] = at;                     /* from here on: where level l's list starts */
            if (cnt) { c->group_level[gi] = l; c->group_ptr[gi] = at; ++gi; }
            at += cnt;
        }
        c->group_ptr[groups] = at;
    }
    for (int64_t i = 0; i < n_app; ++i) c->cone_root[per_level[level[app_root[i]] + 1]++] = app_root[i];
    free(per_level);
    {
        int64_t tot = 0;
        for (int64_t i = 0; i < n_app; ++i) { const int32_t r = c->cone_root[i]; c->cone_ptr[i] = tot; tot += nbr_ptr[r + 1] - nbr_ptr[r]; }
        c->cone_ptr[n_app] = tot; c->n_entries = tot;
        c->cone_node = (int32_t*)malloc(sizeof(int32_t) * (size_t)(tot + 1));
        if (!c->cone_node) goto fail;
        for (int64_t i = 0; i < n_app; ++i) {
            const int32_t r = c->cone_root[i];
            memcpy(c->cone_node + c->cone_ptr[i], nbr_idx + nbr_ptr[r], sizeof(int32_t) * (size_t)(nbr_ptr[r + 1] - nbr_ptr[r]));
        }
    }
    free(app_root); free(is_root); free(in_cone); free(has_out);
    return c;
fail:
    free(app_root); free(is_root); free(in_cone); free(has_out);
    orc_cones_free(c);
    return NULL;
}

void orc_cones_sizes(const orc_cones* c, int64_t* n_groups, int64_t* n_cones, int64_t* n_entries)
{
    *n_groups = c->n_groups; *n_cones = c->n_cones; *n_entries = c->n_entries;
}

void orc_cones_copy(const orc_cones* c, int32_t* group_level, int64_t* group_ptr, int32_t* cone_root,
                    int64_t* cone_ptr, int32_t* cone_node)
{
    memcpy(group_level, c->group_level, sizeof(int32_t) * (size_t)c->n_groups);
    memcpy(group_ptr, c->group_ptr, sizeof(int64_t) * (size_t)(c->n_groups + 1));
    memcpy(cone_root, c->cone_root, sizeof(int32_t) * (size_t)c->n_cones);
    memcpy(cone_ptr, c->cone_ptr, sizeof(int64_t) * (size_t)(c->n_cones + 1));
    memcpy(cone_node, c->cone_node, sizeof(int32_t) * (size_t)c->n_entries);
}

/* (qsort takes no context argument: the levels go through this file-scope pointer, so one call of
 * orc_partitioned_fwd at a time) */
static const int32_t* sort_level;
static int by_level_then_id(const void* a, const void* b)
{
    const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    if (sort_level[x] != sort_level[y]) return sort_level[x] < sort_level[y] ? -1 : 1;
    return x < y ? -1 : x > y;
}

/*
 * Algorithm 2 at inference: the lists by ascending level (inter-level updating is what the
 * marks left by earlier lists do), each list in mini-batches of `batch` cones (intra-level
 * updating). nbr_* are the rows of cone_k (the relation <=_k with its codes, R5).
 * mark = 0 is the ablation without marks. memo != 0 keeps the projected K | V of every gate's
 * current embedding (a pure function of that embedding: same values, less work). Outputs: H [n, d]; kept[j] (nullable) = 1 where
 * entry j of cone_k(v) was in the neighbourhood v was (last) computed with; stage_of[v]
 * (nullable) = running number of the mini-batch that (last) computed v; *n_computed
 * (nullable) = gate computations in total.
 */
int orc_partitioned_fwd(int64_t n, int32_t d, int32_t heads, int32_t n_layers, int32_t store,
                        int32_t epilogue, double ln_eps,
                        const float* x, const float* wqkv, const float* wo, const float* bias,
                        const float* w1 /* nullable */, const float* w2 /* nullable with w1 */,
                        const int32_t* level, const int64_t* nbr_ptr, const int32_t* nbr_idx, const uint8_t* nbr_rel,
                        int64_t n_groups, const int64_t* group_ptr, const int64_t* cone_ptr, const int32_t* cone_node,
                        int32_t batch, int32_t mark, int32_t memo,
                        double* H, uint8_t* kept, int32_t* stage_of, int64_t* n_computed)
{
    if (d <= 0 || d > 1024 || heads <= 0 || d % heads || n_layers <= 0 || batch < 1) return ORC_EINVAL;
    if ((w1 == NULL) != (w2 == NULL) || (w1 && !epilogue)) return ORC_EINVAL;
    orc_layer L = { d, heads, n_layers, store, epilogue, ln_eps, x, wqkv, wo, bias, w1, w2, nbr_ptr, nbr_idx, nbr_rel };
    const size_t n1 = (size_t)(n > 0 ? n : 1);
    const int64_t nnz = nbr_ptr[n];
    uint8_t* updated = (uint8_t*)calloc(n1, 1);                 /* the marks */
    uint8_t* keep = (uint8_t*)calloc((size_t)(nnz > 0 ? nnz : 1), 1);
    int64_t* seen_in = (int64_t*)malloc(sizeof(int64_t) * n1);   /* last mini-batch a gate was met in */
    int64_t* in_cone = (int64_t*)malloc(sizeof(int64_t) * n1);   /* last cone a gate was stamped for  */
    int32_t* todo = (int32_t*)malloc(sizeof(int32_t) * n1);
    int32_t* members = (int32_t*)malloc(sizeof(int32_t) * n1);
    double* kv = memo ? (double*)malloc(sizeof(double) * (size_t)n_layers * n1 * 2 * (size_t)d) : NULL;
    if (!updated || !keep || !seen_in || !in_cone || !todo || !members || (memo && !kv)) {
        free(updated); free(keep); free(seen_in); free(in_cone); free(todo); free(members); free(kv);
        return ORC_ENOMEM;
    }
    for (int64_t v = 0; v < n; ++v) { seen_in[v] = -1; in_cone[v] = -1; }
    int64_t stage = 0, computed = 0;
    for (int64_t g = 0; g < n_groups; ++g) {
        for (int64_t b0 = group_ptr[g]; b0 < group_ptr[g + 1]; b0 += batch, ++stage) {
            const int64_t b1 = b0 + batch < group_ptr[g + 1] ? b0 + batch : group_ptr[g + 1];
            int64_t n_todo = 0, n_members = 0;
            for (int64_t c = b0; c < b1; ++c) {
                for (int64_t i = cone_ptr[c]; i < cone_ptr[c + 1]; ++i) in_cone[cone_node[i]] = c;
                for (int64_t i = cone_ptr[c]; i < cone_ptr[c + 1]; ++i) {
                    const int32_t v = cone_node[i];
                    if (seen_in[v] != stage) {
                        seen_in[v] = stage; members[n_members++] = v;
                        if (!(mark && updated[v])) {
                            todo[n_todo++] = v;
                            memset(keep + nbr_ptr[v], 0, (size_t)(nbr_ptr[v + 1] - nbr_ptr[v]));
                        }
                    }
                    if (mark && updated[v]) continue;       /* retrieved from the store, its in-edges dropped */
                    /* the virtual edges of this cone into v: u <=_k v with u in the cone */
                    for (int64_t j = nbr_ptr[v]; j < nbr_ptr[v + 1]; ++j)
                        if (in_cone[nbr_idx[j]] == c) keep[j] = 1;
                }
            }
            sort_level = level;
            qsort(todo, (size_t)n_todo, sizeof(int32_t), by_level_then_id);
            for (int64_t a = 0; a < n_todo;) {
                int64_t z = a;
                while (z < n_todo && level[todo[z]] == level[todo[a]]) ++z;
#pragma omp parallel for schedule(dynamic, 8)
                for (int64_t t = a; t < z; ++t) {
                    const int32_t v = todo[t];
                    int32_t idx[1 << 9]; uint8_t rel[1 << 9];
                    int cnt = 0;
                    for (int64_t j = nbr_ptr[v]; j < nbr_ptr[v + 1]; ++j)
                        if (keep[j]) { idx[cnt] = nbr_idx[j]; rel[cnt] = nbr_rel[j]; ++cnt; }
                    node_step_row(&L, v, idx, rel, cnt, H, NULL, kv, n, H + (int64_t)v * d);
                }
                if (kv)                     /* after the level: no gate of it reads another */
#pragma omp parallel for schedule(static)
                    for (int64_t t = a; t < z; ++t)
                        for (int l = 0; l < n_layers; ++l)
                            vec_mat(H + (int64_t)todo[t] * d, d, wqkv + (int64_t)l * d * 3 * d, 3 * d, d, 2 * d,
                                    kv + ((int64_t)l * n + todo[t]) * 2 * d);
                a = z;
            }
            computed += n_todo;
            for (int64_t t = 0; t < n_todo; ++t) {
                const int32_t v = todo[t];
                if (stage_of) stage_of[v] = (int32_t)stage;
                if (kept) memcpy(kept + nbr_ptr[v], keep + nbr_ptr[v], (size_t)(nbr_ptr[v + 1] - nbr_ptr[v]));
            }
            for (int64_t t = 0; t < n_members; ++t) updated[members[t]] = 1;
        }
    }
    if (n_computed) *n_computed = computed;
    free(updated); free(keep); free(seen_in); free(in_cone); free(todo); free(members); free(kv);
    return ORC_OK;
}

/* ------------------------------------------------------------------------------------------
 * Structural encoding, Section 3.5 Eq. 2:
 *   SE(v) = Emb_l(level(v)) + Emb_and(OutAND(v)) + Emb_not(OutNOT(v)),  x'(v) = x(v) + SE(v)
 * with OutAND / OutNOT the numbers of AND / NOT gates among the direct fanouts of v (R15).
 */
void orc_out_degrees(int64_t n, int64_t e, const int32_t* src, const int32_t* dst, const uint8_t* inv,
                     int32_t* out_and, int32_t* out_not)
{
    int32_t* indeg = (int32_t*)calloc((size_t)(n > 0 ? n : 1), sizeof(int32_t));
    uint8_t* has_inverter = (uint8_t*)calloc((size_t)(n > 0 ? n : 1), 1);
    for (int64_t i = 0; i < e; ++i) indeg[dst[i]]++;
    for (int64_t v = 0; v < n; ++v) { out_and[v] = 0; out_not[v] = 0; }
    for (int64_t i = 0; i < e; ++i) {
        const int32_t v = src[i], u = dst[i];
        if (indeg[u] == 1) out_not[v]++;                 /* u is a NOT / buffer gate              */
        else if (inv[i]) has_inverter[v] = 1;            /* the one inverter behind v             */
        else out_and[v]++;                               /* u is an AND fed by v directly         */
    }
    for (int64_t v = 0; v < n; ++v) out_not[v] += has_inverter[v];
    free(indeg); free(has_inverter);
}

/* emb: [6][d] = w_l, b_l, w_and, b_and, w_not, b_not; out rounded as stored (store as above) */
void orc_struct_encode(int64_t n, int32_t d, const float* x, const int32_t* level,
                       const int32_t* out_and, const int32_t* out_not, const float* emb,
                       int32_t store, double* out)
{
    for (int64_t v = 0; v < n; ++v)
        for (int32_t c = 0; c < d; ++c) {
            const double se = ((double)level[v] * emb[0 * d + c] + emb[1 * d + c])
                            + ((double)out_and[v] * emb[2 * d + c] + emb[3 * d + c])
                            + ((double)out_not[v] * emb[4 * d + c] + emb[5 * d + c]);
            out[v * d + c] = round_store((double)x[v * d + c] + se, store);
        }
}
