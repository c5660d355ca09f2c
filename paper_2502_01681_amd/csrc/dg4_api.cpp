// extern "C" entry points: argument checks, workspace layout and the host side
// of the level sweep (paper Section 3.4, Algorithm 2). All arithmetic is in
// the device kernels; there is no CPU fallback.
#include <algorithm>
#include <cstdlib>
#include <cstring>

#include "dg4_internal.h"

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline size_t elt_size(int dtype) { return dtype == DG4_F32 ? 4 : 2; }

int check_cfg(const dg4_layer_cfg* c, bool need_layers)
{
    if (!c) return DG4_EINVAL;
    if (c->dtype != DG4_F32 && c->dtype != DG4_BF16) return DG4_EINVAL;
    if (c->flags & ~(uint32_t)(DG4_NO_EPILOGUE | DG4_PER_LEVEL | DG4_BOUNDED_KV | DG4_FFN | DG4_LEVEL_ORDER | DG4_PROFILE |
                               DG4_TIME_SWEEP | DG4_WEIGHTS_PACKED)) return DG4_EINVAL;
    if ((c->flags & DG4_FFN) && (c->flags & DG4_NO_EPILOGUE)) return DG4_EINVAL;
    if (c->hidden != 128 && c->hidden != 256) return DG4_EUNSUPPORTED;
    if (c->heads <= 0 || c->heads * 32 != c->hidden) return DG4_EUNSUPPORTED;
    if (c->hops < 1 || c->hops > DG4_MAX_HOPS) return DG4_EUNSUPPORTED;
    if (need_layers && (c->n_layers < 1 || c->n_layers > DG4_MAX_LAYERS)) return DG4_EUNSUPPORTED;
    if (!(c->ln_eps >= 0.f)) return DG4_EINVAL;
    return DG4_OK;
}

// Workspace of dg4_layer_fwd, in bytes from the (256-byte aligned) base.
struct LayerPlan {
    size_t wqkv[DG4_MAX_LAYERS], wo[DG4_MAX_LAYERS];
    size_t w1[DG4_MAX_LAYERS], w2[DG4_MAX_LAYERS];   // feed-forward weights, packed (DG4_FFN)
    size_t h1;           // [max_level_rows, d] state after the attention sub-block (DG4_FFN)
    size_t wkv_all;      // packed [d, n_layers*2d]: K|V columns of every layer
    size_t wkv_a;        // the same in the order of the persistent kernel for every shape
    size_t qkv_self;     // [n, 3d]  Q | K | V of x, level-sorted rows (layer 0)
    size_t kv;           // [n_layers, kv_rows, 2d]  K | V of the final embeddings, level-sorted
    size_t kv_rows;
    size_t hpos;         // [n, d]   final embeddings, level-sorted
    size_t abuf;         // [max_level_rows, d]
    size_t s0, s1;       // [max_level_rows, d] running state between layers
    size_t qkv_level;    // [max_level_rows, 3d] (layers >= 1)
    size_t wo_t, wkv_t;  // persistent sweep: weights in its A-operand order (layer 0)
    size_t ffn_t;        // persistent sweep: W1 | W2 in its streaming order (DG4_FFN)
    size_t park;         // persistent sweep: rows parked between the two tiles of a pair (DG4_FFN)
    size_t bias_all;     // [n_layers][heads, 4] float: the relation biases of every layer, contiguous
    size_t flags;        // [n] uint32 "rows published"
    size_t ctrl;         // abort word, ticket counter, phase timers
    size_t total;
    int64_t max_rows;
};

LayerPlan plan_layer(const dg4_layer_cfg* c, const dg4_graph* g)
{
    LayerPlan p{};
    const size_t es = elt_size(c->dtype), d = (size_t)c->hidden, n = (size_t)std::max<int64_t>(g->n, 1);
    const size_t L = (size_t)c->n_layers;
    int64_t mr = 1;
    for (size_t l = 0; l + 1 < g->level_ptr.size(); ++l) mr = std::max(mr, g->level_ptr[l + 1] - g->level_ptr[l]);
    if (!(c->flags & DG4_BOUNDED_KV))        // sweeps with the K|V store may run through the Eq. 1 levels
        for (size_t l = 0; l + 1 < g->eq1_level_ptr.size(); ++l) mr = std::max(mr, g->eq1_level_ptr[l + 1] - g->eq1_level_ptr[l]);
    p.max_rows = mr;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
    for (size_t l = 0; l < L; ++l) { p.wqkv[l] = take(d * 3 * d * es); p.wo[l] = take(d * d * es); }
    const bool ffn = (c->flags & DG4_FFN) != 0;
    for (size_t l = 0; l < L; ++l) { p.w1[l] = take(ffn ? d * 4 * d * es : 0); p.w2[l] = take(ffn ? 4 * d * d * es : 0); }
    p.wkv_all = take(d * 2 * d * L * es);
    p.wkv_a = take(d * 2 * d * L * es);
    p.qkv_self = take((c->flags & DG4_BOUNDED_KV) ? 0 : n * 3 * d * es);
    // K | V rows: of every finished gate, or (DG4_BOUNDED_KV) of one level's frontier only
    const bool bounded = (c->flags & DG4_BOUNDED_KV) != 0;
    p.kv_rows = bounded ? (size_t)std::max<int64_t>(g->front_max, 1) : n;
    p.kv = take(L * p.kv_rows * 2 * d * es);
    p.hpos = take(bounded ? 0 : n * d * es);
    p.abuf = take((size_t)mr * d * es);
    p.s0 = take((size_t)mr * d * es);
    p.s1 = take((size_t)mr * d * es);
    p.h1 = take(ffn ? (size_t)mr * d * es : 0);
    p.qkv_level = take(L > 1 || bounded ? (size_t)mr * 3 * d * es : 0);
    p.wo_t = take(d * d * es);
    p.wkv_t = take(d * 2 * d * es);
    p.ffn_t = take(ffn ? 2 * d * 4 * d * es : 0);
    p.park = take(ffn ? (size_t)DG4_MAX_SWEEP_GROUPS * DG4_TILE_ROWS * d * es : 0);
    p.bias_all = take(L * (size_t)c->heads * 4 * sizeof(float));
    p.flags = take(n * sizeof(uint32_t));
    p.ctrl = take(256);
    p.total = off;
    return p;
}

// polls of a flag before a persistent sweep gives up (cfg->spin_limit = 0: this default)
constexpr uint32_t DEFAULT_SPIN_LIMIT = 1u << 22;
// Optional timing of the persistent sweep kernel alone (DG4_TIME_SWEEP, a tracing aid): two events on
// the caller's stream around its launch, read back by dg4_sweep_elapsed_ms. One pair per process,
// guarded by a mutex; the figure is that of the most recent such call, whichever thread made it.
struct SweepEvents { std::mutex mu; hipEvent_t a = nullptr, b = nullptr; bool armed = false; };
SweepEvents& sweep_events() { static SweepEvents e; return e; }

#define HIPCHK(expr) do { if ((expr) != (int)hipSuccess) return DG4_EHIP; } while (0)

// rows are read and written as 16-byte pieces
template <typename... P> bool aligned16(P... ptrs) { return (((uintptr_t)ptrs | ...) & 15) == 0; }

}  // namespace

extern "C" const char* dg4_strerror(int status)
{
    switch (status) {
    case DG4_OK: return "ok";
    case DG4_EINVAL: return "invalid argument";
    case DG4_ERANGE: return "node id out of range";
    case DG4_EFANIN: return "in-degree above 2 or duplicated fanin edge";
    case DG4_ECYCLE: return "edge list is not a DAG";
    case DG4_EHINT: return "level hint is not a topological levelling";
    case DG4_EUNSUPPORTED: return "unsupported configuration";
    case DG4_ENOMEM: return "out of memory";
    case DG4_EWORKSPACE: return "workspace missing, misaligned or too small";
    case DG4_EHIP: return "HIP runtime error";
    case DG4_EABORTED: return "persistent sweep gave up on a dependency wait";
    default: return "unknown status";
    }
}

extern "C" int64_t dg4_proj_workspace_bytes(const dg4_layer_cfg* cfg)
{
    const int rc = check_cfg(cfg, false);
    if (rc != DG4_OK) return rc;
    return (int64_t)align256((size_t)cfg->hidden * 3 * cfg->hidden * elt_size(cfg->dtype));
}

extern "C" int64_t dg4_ffn_workspace_bytes(const dg4_layer_cfg* cfg)
{
    const int rc = check_cfg(cfg, false);
    if (rc != DG4_OK) return rc;
    return (int64_t)(2 * align256((size_t)cfg->hidden * 4 * cfg->hidden * elt_size(cfg->dtype)));
}

extern "C" int64_t dg4_layer_workspace_bytes(const dg4_layer_cfg* cfg, const dg4_graph* g)
{
    const int rc = check_cfg(cfg, true);
    if (rc != DG4_OK) return rc;
    if (!g) return DG4_EINVAL;
    if (g->hops != cfg->hops) return DG4_EINVAL;
    if (cfg->flags & DG4_BOUNDED_KV) {       // the size depends on the largest frontier: tables first
        dg4_graph* m = const_cast<dg4_graph*>(g);
        int rc2 = dg4_graph_ensure_device(m);
        if (rc2 == DG4_OK) rc2 = dg4_graph_ensure_frontier(m);
        if (rc2 != DG4_OK) return rc2;
    }
    return (int64_t)plan_layer(cfg, g).total;
}

// Argument checks of dg4_qkv_proj that do not concern the workspace (shared with dg4_qkv_proj_static).
int dg4_qkv_proj_check(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                       const void* Wqkv, const void* Q, const void* K, const void* V)
{
    const int rc = check_cfg(cfg, false);
    if (rc != DG4_OK) return rc;
    if (!S || !Wqkv || !Q || !K || !V || row_begin < 0 || row_end < row_begin) return DG4_EINVAL;
    if (!aligned16(S, Wqkv, Q, K, V)) return DG4_EINVAL;
    return DG4_OK;
}

// The launches of dg4_qkv_proj: `packed` (dg4_proj_workspace_bytes, 256-byte aligned) takes the weight
// in matrix-core operand order. Allocates nothing.
int dg4_qkv_proj_run(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                     const void* Wqkv, void* Q, void* K, void* V, void* packed, hipStream_t s)
{
    if (row_end == row_begin) return DG4_OK;
    const int d = cfg->hidden;
    if (cfg->dtype == DG4_BF16 && d == 256) {
        HIPCHK(dg4_launch_pack_w32(Wqkv, 3 * d, packed, s));
        dg4_bulk_args b{};
        b.src = (const uint16_t*)S;
        b.w_packed = packed; b.n_cols = 3 * d;
        b.out[0] = (uint16_t*)Q; b.out[1] = (uint16_t*)K; b.out[2] = (uint16_t*)V; b.out_stride = d;
        b.row_begin = row_begin; b.row_end = row_end;
        HIPCHK(dg4_launch_bulk_proj(b, s));
        return DG4_OK;
    }
    HIPCHK(dg4_launch_pack_w(cfg->dtype, Wqkv, 3 * d, 0, 3 * d, d, packed, s));
    dg4_gemm_args a{};
    a.a = S; a.a_stride = d;
    a.w_packed = packed; a.n_cols = 3 * d;
    a.out[0] = Q; a.out[1] = K; a.out[2] = V; a.out_stride = d;
    a.row_begin = row_begin; a.row_end = row_end;
    HIPCHK(dg4_launch_gemm(cfg->dtype, d, a, s));
    return DG4_OK;
}

extern "C" int dg4_qkv_proj(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                            const void* Wqkv, void* Q, void* K, void* V,
                            void* workspace, int64_t workspace_bytes, void* stream)
{
    const int rc = dg4_qkv_proj_check(cfg, S, row_begin, row_end, Wqkv, Q, K, V);
    if (rc != DG4_OK) return rc;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < dg4_proj_workspace_bytes(cfg)) return DG4_EWORKSPACE;
    return dg4_qkv_proj_run(cfg, S, row_begin, row_end, Wqkv, Q, K, V, workspace, (hipStream_t)stream);
}

extern "C" int dg4_ffn_fwd(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                           const void* W1, const void* W2, void* Out,
                           void* workspace, int64_t workspace_bytes, void* stream)
{
    int rc = check_cfg(cfg, false);
    if (rc != DG4_OK) return rc;
    if (!S || !W1 || !W2 || !Out || row_begin < 0 || row_end < row_begin) return DG4_EINVAL;
    if (!aligned16(S, W1, W2, Out)) return DG4_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < dg4_ffn_workspace_bytes(cfg)) return DG4_EWORKSPACE;
    if (row_end == row_begin) return DG4_OK;
    hipStream_t s = (hipStream_t)stream;
    const int d = cfg->hidden;
    char* w1p = (char*)workspace;
    char* w2p = w1p + align256((size_t)d * 4 * d * elt_size(cfg->dtype));
    if (cfg->dtype == DG4_BF16 && d == 256) {
        // this shape always takes the kernel for many rows (one kernel per shape: the result of a
        // row does not depend on the range it was asked for in)
        HIPCHK(dg4_launch_pack_ffn_bulk(W1, W2, w1p, s));
        dg4_ffn_args f{};
        f.h = S; f.h_stride = d;
        f.w1_packed = w1p;
        f.out = Out; f.out_stride = d;
        f.row_begin = row_begin; f.row_end = row_end;
        f.ln_eps = cfg->ln_eps;
        HIPCHK(dg4_launch_ffn_bulk(f, s));
        return DG4_OK;
    }
    HIPCHK(dg4_launch_pack_w(cfg->dtype, W1, 4 * d, 0, 4 * d, d, w1p, s));
    HIPCHK(dg4_launch_pack_w2(cfg->dtype, W2, d, w2p, s));
    dg4_ffn_args f{};
    f.h = S; f.h_stride = d;
    f.w1_packed = w1p; f.w2_packed = w2p;
    f.out = Out; f.out_stride = d;
    f.row_begin = row_begin; f.row_end = row_end;
    f.ln_eps = cfg->ln_eps;
    HIPCHK(dg4_launch_ffn(cfg->dtype, d, f, s));
    return DG4_OK;
}

extern "C" int dg4_struct_encode(const dg4_layer_cfg* cfg, dg4_graph* g, const void* X, const float* emb,
                                 void* Xout, void* stream)
{
    int rc = check_cfg(cfg, false);
    if (rc != DG4_OK) return rc;
    if (!g || !X || !emb || !Xout || !aligned16(X, emb, Xout)) return DG4_EINVAL;
    if (g->n == 0) return DG4_OK;
    rc = dg4_graph_ensure_struct(g);
    if (rc != DG4_OK) return rc;
    HIPCHK(dg4_launch_struct_encode(cfg->dtype, cfg->hidden, X, g->d_struct, emb, Xout, g->n, (hipStream_t)stream));
    return DG4_OK;
}

extern "C" int dg4_sparse_attn_fwd(const dg4_layer_cfg* cfg, dg4_graph* g, int64_t row_begin, int64_t row_end,
                                   const void* Q, const void* K, const void* V, const float* rel_bias,
                                   void* A, void* stream)
{
    int rc = check_cfg(cfg, false);
    if (rc != DG4_OK) return rc;
    if (!g || !Q || !K || !V || !rel_bias || !A || !aligned16(Q, K, V, A)) return DG4_EINVAL;
    if (g->hops != cfg->hops || row_begin < 0 || row_end < row_begin || row_end > g->n) return DG4_EINVAL;
    if (row_end == row_begin) return DG4_OK;
    rc = dg4_graph_ensure_device(g);
    if (rc != DG4_OK) return rc;
    const int d = cfg->hidden;
    dg4_attn_args a{};
    a.q = Q; a.q_stride = d;
    a.k_self = K; a.v_self = V; a.self_stride = d;
    a.k_src = K; a.v_src = V; a.src_stride = d;
    a.rel_bias = rel_bias;
    a.ell = g->d_ell_id; a.ell_w = g->ell_w;
    a.a = A; a.a_stride = d;
    a.row_begin = row_begin; a.row_end = row_end;
    HIPCHK(dg4_launch_attn(cfg->dtype, d, a, (hipStream_t)stream));
    return DG4_OK;
}

extern "C" int dg4_layer_fwd(const dg4_layer_cfg* cfg, dg4_graph* g, const void* X, const void* const* W,
                             int32_t level_begin, int32_t level_end, void* Hout,
                             void* workspace, int64_t workspace_bytes, void* stream)
{
    int rc = check_cfg(cfg, true);
    if (rc != DG4_OK) return rc;
    if (!g || !X || !W || !Hout || !aligned16(X, Hout)) return DG4_EINVAL;
    if (g->hops != cfg->hops) return DG4_EINVAL;
    const int32_t n_levels = g->max_level + 1;
    if (level_begin < 0 || level_end < level_begin || level_end > n_levels) return DG4_EINVAL;
    const int L = cfg->n_layers;
    const bool ffn = (cfg->flags & DG4_FFN) != 0;
    const int WS = ffn ? 5 : 3;                      // weight pointers per layer
    for (int i = 0; i < WS * L; ++i) if (!W[i]) return DG4_EINVAL;
    const bool bounded = (cfg->flags & DG4_BOUNDED_KV) != 0;
    if (bounded) {
        rc = dg4_graph_ensure_device(g);
        if (rc == DG4_OK) rc = dg4_graph_ensure_frontier(g);
        if (rc != DG4_OK) return rc;
    }
    const LayerPlan pl = plan_layer(cfg, g);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < (int64_t)pl.total) return DG4_EWORKSPACE;
    if (g->n == 0 || level_begin == level_end) return DG4_OK;
    rc = dg4_graph_ensure_device(g);
    if (rc != DG4_OK) return rc;

    hipStream_t s = (hipStream_t)stream;
    const int d = cfg->hidden, dt = cfg->dtype;
    const int64_t es = (int64_t)elt_size(dt);
    const bool epi = !(cfg->flags & DG4_NO_EPILOGUE);
    char* ws = (char*)workspace;
    auto at = [&](size_t off) { return (void*)(ws + off); };
    // base pointer of a per-level buffer such that row p (a position) lands at local row p - p0
    auto local = [&](size_t off, int64_t p0, int64_t stride) { return (void*)(ws + off - p0 * stride * es); };

    // Which path: the kernel specialised for bf16 / hidden 256 / one layer / cones of two hops (weights
    // resident in registers), the persistent dataflow kernel for the other shapes and any number of
    // layers, or level-by-level launches (DG4_PER_LEVEL, DG4_BOUNDED_KV, the feed-forward sub-block
    // on neighbour rows wider than 16 entries).
    const bool whole_range = level_begin == 0 && level_end == (int32_t)g->max_level + 1;
    const bool forced_levels = (cfg->flags & (DG4_PER_LEVEL | DG4_BOUNDED_KV)) != 0;
    const bool resident = dt == DG4_BF16 && d == 256 && L == 1 && cfg->hops <= 2 && !forced_levels && (!ffn || whole_range);
    const bool flow = !resident && !forced_levels && dg4_flow_supports(dt, d, g->ell_w) && (!ffn || g->ell_w <= 16);
    // a caller that has not changed the weights since its last call with this configuration, graph
    // and workspace vouches for the packed copies that call left behind
    const bool pack = !(cfg->flags & DG4_WEIGHTS_PACKED);
    const uint32_t spin_limit = cfg->spin_limit ? cfg->spin_limit : DEFAULT_SPIN_LIMIT;

    if (pack) {
        for (int l = 0; l < L; ++l) {
            if (flow) {
                // layer 0's Q | K | V weight serves the bulk projection of x (packed further down for bf16)
                if (l > 0) HIPCHK(dg4_launch_pack_wa(dt, d, W[WS * l], 3 * d, 0, 3 * d, at(pl.wqkv[l]), s));
                else if (dt != DG4_BF16) HIPCHK(dg4_launch_pack_w(dt, W[0], 3 * d, 0, 3 * d, d, at(pl.wqkv[0]), s));
                HIPCHK(dg4_launch_pack_wa(dt, d, W[WS * l + 1], d, 0, d, at(pl.wo[l]), s));
                HIPCHK(dg4_launch_pack_wa(dt, d, W[WS * l], 3 * d, d, 2 * d, ws + pl.wkv_a + (size_t)l * 2 * d * d * es, s));
                if (ffn) {      // W1 whole; W2 as four blocks of d input rows
                    HIPCHK(dg4_launch_pack_wa(dt, d, W[WS * l + 3], 4 * d, 0, 4 * d, at(pl.w1[l]), s));
                    for (int c4 = 0; c4 < 4; ++c4)
                        HIPCHK(dg4_launch_pack_wa(dt, d, (const char*)W[WS * l + 4] + (size_t)c4 * d * d * es, d, 0, d,
                                                  ws + pl.w2[l] + (size_t)c4 * d * d * es, s));
                }
            } else if (!resident) {
                HIPCHK(dg4_launch_pack_w(dt, W[WS * l], 3 * d, 0, 3 * d, d, at(pl.wqkv[l]), s));
                HIPCHK(dg4_launch_pack_w(dt, W[WS * l + 1], d, 0, d, d, at(pl.wo[l]), s));
            }
            // K | V columns of layer l go to column tiles [l*2d/32, (l+1)*2d/32) of wkv_all
            if ((!resident && !flow) || (resident && level_begin > 0))
                HIPCHK(dg4_launch_pack_w(dt, W[WS * l], 3 * d, d, 2 * d, d, ws + pl.wkv_all + (size_t)l * 2 * d * d * es, s));
            if (ffn && !resident && !flow) {
                HIPCHK(dg4_launch_pack_w(dt, W[WS * l + 3], 4 * d, 0, 4 * d, d, at(pl.w1[l]), s));
                HIPCHK(dg4_launch_pack_w2(dt, W[WS * l + 4], d, at(pl.w2[l]), s));
            }
        }
    }
    const int64_t P0 = g->level_ptr[level_begin], P1 = g->level_ptr[level_end];

    auto kv_project = [&](const void* rows, int64_t stride, const int32_t* gather, int64_t r0, int64_t r1) -> int {
        dg4_gemm_args a{};
        a.a = rows; a.a_stride = stride; a.a_gather = gather;
        a.w_packed = at(pl.wkv_all); a.n_cols = 2 * d * L;
        for (int l = 0; l < L; ++l) {
            char* base = ws + pl.kv + (size_t)l * pl.kv_rows * 2 * d * es;
            a.out[2 * l] = base; a.out[2 * l + 1] = base + (size_t)d * es;
        }
        a.out_stride = 2 * d;
        a.row_begin = r0; a.row_end = r1;
        return dg4_launch_gemm(dt, d, a, s);
    };

    // K/V of gates finished before this call (resume): from the caller's H (the persistent kernel for
    // every shape does that itself, with its own arithmetic)
    if (P0 > 0 && !bounded && !flow) HIPCHK(kv_project(Hout, d, g->d_order, 0, P0));

    // optional timing of the persistent kernel alone (a call that runs none leaves nothing to read back)
    const bool timed = (cfg->flags & DG4_TIME_SWEEP) != 0 && (resident || flow);
    if ((cfg->flags & DG4_TIME_SWEEP) && !timed) {
        SweepEvents& ev = sweep_events();
        std::lock_guard<std::mutex> lock(ev.mu);
        ev.armed = false;
    }
    auto bracket = [&](auto&& launch) -> int {
        if (!timed) return launch();
        SweepEvents& ev = sweep_events();
        std::lock_guard<std::mutex> lock(ev.mu);
        if (!ev.a && (hipEventCreate(&ev.a) != hipSuccess || hipEventCreate(&ev.b) != hipSuccess)) return (int)hipErrorUnknown;
        if (hipEventRecord(ev.a, s) != hipSuccess) return (int)hipErrorUnknown;
        const int rc2 = launch();
        if (rc2 != (int)hipSuccess) return rc2;
        if (hipEventRecord(ev.b, s) != hipSuccess) return (int)hipErrorUnknown;
        ev.armed = true;
        return (int)hipSuccess;
    };

    // One persistent dataflow kernel for the whole range of levels (with the feed-forward sub-block:
    // whole-graph sweeps only, partial ones run level by level)
    if (resident) {
        // A sweep over all levels runs in the dependency-driven tile order, a partial one (resume)
        // or one with DG4_LEVEL_ORDER level by level; rows of the internal buffers are positions in
        // the order in use.
        const bool whole = whole_range && (ffn || !(cfg->flags & DG4_LEVEL_ORDER));
        if (ffn) {
            rc = dg4_graph_ensure_pairs(g);
            if (rc != DG4_OK) return rc;
        }
        const int32_t* order_in_use = ffn ? g->d_pair_order : whole ? g->d_flow_order : g->d_order;
        {   // Q | K | V of x for every gate of the swept levels, rows in processing order
            if (pack) HIPCHK(dg4_launch_pack_w32(W[0], 3 * d, at(pl.wqkv[0]), s));
            dg4_bulk_args b{};
            b.src = (const uint16_t*)X; b.gather = order_in_use;
            b.w_packed = at(pl.wqkv[0]); b.n_cols = 3 * d;
            uint16_t* base = (uint16_t*)at(pl.qkv_self);
            b.out[0] = base; b.out[1] = base + d; b.out[2] = base + 2 * d; b.out_stride = 3 * d;
            b.row_begin = P0; b.row_end = P1;
            HIPCHK(dg4_launch_bulk_proj(b, s));
        }
        if (pack) {
            HIPCHK(dg4_launch_pack_wt(W[1], d, 0, 4, 4, at(pl.wo_t), s));
            HIPCHK(dg4_launch_pack_wt(W[0], 3 * d, d, 8, 4, at(pl.wkv_t), s));
        }
        dg4_sweep_args a{};
        a.tiles = ffn ? g->d_pair_tiles : whole ? g->d_flow_tiles : g->d_tiles;
        a.tile_begin = whole ? 0 : g->level_tile_ptr[level_begin];
        a.n_tiles = ffn ? g->n_pair_tiles : whole ? g->n_flow_tiles : g->level_tile_ptr[level_end] - a.tile_begin;
        a.ell = ffn ? g->d_pair_ell : whole ? g->d_flow_ell : g->d_ell_pos; a.ell_w = g->ell_w;
        a.order = order_in_use;
        a.x = (const uint16_t*)X;
        a.qkv_self = (const uint16_t*)at(pl.qkv_self);
        a.kv = (uint16_t*)at(pl.kv);
        a.h_out = (uint16_t*)Hout;
        a.wo_packed = at(pl.wo_t); a.wkv_packed = at(pl.wkv_t);
        a.rel_bias = (const float*)W[2];
        if (ffn) {
            if (pack) HIPCHK(dg4_launch_pack_ffn(W[3], W[4], at(pl.ffn_t), s));
            a.ffn_packed = at(pl.ffn_t);
            a.park = (uint16_t*)at(pl.park);
        }
        a.flags = (uint32_t*)at(pl.flags); a.ctrl = (uint32_t*)at(pl.ctrl);
        a.ln_eps = cfg->ln_eps; a.epilogue = epi ? 1 : 0; a.eager_publish = whole ? 0 : 1;
        a.spin_limit = spin_limit;
        a.prof = (cfg->flags & DG4_PROFILE) ? (uint64_t*)((char*)at(pl.ctrl) + 64) : nullptr;
        HIPCHK(dg4_launch_sweep_init(a.flags, a.ctrl, g->n, P0, s));
        HIPCHK(bracket([&]() { return dg4_launch_sweep(a, s); }));
        return DG4_OK;
    }

    if (flow) {
        // tiles of up to 32 mutually independent gates: the pairs of the dependency-driven order for a
        // sweep over all levels, runs inside a level otherwise
        // (rows wider than 16 entries: always level by level, tiles of a few gates)
        const bool wide = g->ell_w > 16;
        const bool whole = whole_range && !(cfg->flags & DG4_LEVEL_ORDER) && !wide;
        if (whole) {
            rc = dg4_graph_ensure_pairs(g);
            if (rc != DG4_OK) return rc;
        }
        if (wide) {
            rc = dg4_graph_ensure_wide_tiles(g);
            if (rc != DG4_OK) return rc;
        }
        const int32_t* order_in_use = whole ? g->d_pair_order : g->d_order;
        if (dt == DG4_BF16) {       // (hidden 256: the bulk projection kernel and its weight order)
            if (pack) HIPCHK(dg4_launch_pack_w32(W[0], 3 * d, at(pl.wqkv[0]), s));
            dg4_bulk_args b{};
            b.src = (const uint16_t*)X; b.gather = order_in_use;
            b.w_packed = at(pl.wqkv[0]); b.n_cols = 3 * d;
            uint16_t* base = (uint16_t*)at(pl.qkv_self);
            b.out[0] = base; b.out[1] = base + d; b.out[2] = base + 2 * d; b.out_stride = 3 * d;
            b.row_begin = P0; b.row_end = P1;
            HIPCHK(dg4_launch_bulk_proj(b, s));
        } else {
            dg4_gemm_args a{};
            a.a = X; a.a_stride = d; a.a_gather = order_in_use;
            a.w_packed = at(pl.wqkv[0]); a.n_cols = 3 * d;
            char* base = ws + pl.qkv_self;
            a.out[0] = base; a.out[1] = base + (size_t)d * es; a.out[2] = base + (size_t)2 * d * es;
            a.out_stride = 3 * d;
            a.row_begin = P0; a.row_end = P1;
            HIPCHK(dg4_launch_gemm(dt, d, a, s));
        }
        if (pack)
            for (int l = 0; l < L; ++l)
                if (hipMemcpyAsync(ws + pl.bias_all + (size_t)l * cfg->heads * 4 * sizeof(float), W[WS * l + 2],
                                   (size_t)cfg->heads * 4 * sizeof(float), hipMemcpyDeviceToDevice, s) != hipSuccess) return DG4_EHIP;
        dg4_flow_args a{};
        if (whole) {
            // Tiles of 32 gates (two of the table's tiles of 16, which never depend on each other) share a
            // pass over the weights; on a deep, narrow circuit, where a level is a handful of tiles and
            // most compute units idle, tiles of 16 halve the matrix-core time on the dependency chain.
            const int64_t depth = g->eq1_level_ptr.empty() ? (int64_t)g->max_level + 1 : (int64_t)g->eq1_level_ptr.size() - 1;
            const bool narrow = g->n / std::max<int64_t>(depth, 1) < 4096;
            a.tiles = g->d_pair_tiles; a.pairs = narrow ? 0 : 1; a.tile_begin = 0;
            a.n_tiles = narrow ? g->n_pair_tiles : g->n_pair_tiles / 2;
            a.tile_cap = narrow ? 16 : 32;
            // (there the chain from level to level is what counts: with several layers a reader starts on K | V
            // of the first layer while its sources still project the later ones)
            a.layer_flags = narrow && L > 1 ? 1 : 0;
            a.ell = g->d_pair_ell;
        } else if (wide) {
            a.tiles = g->d_tilesw; a.pairs = 0; a.tile_rows = g->wide_tile_rows; a.tile_cap = 16;
            a.tile_begin = g->level_tilew_ptr[level_begin];
            a.n_tiles = g->level_tilew_ptr[level_end] - a.tile_begin;
            a.ell = g->d_ell_pos;
        } else {
            a.tiles = g->d_tiles32; a.pairs = 0; a.tile_begin = g->level_tile32_ptr[level_begin]; a.tile_cap = 32;
            a.n_tiles = g->level_tile32_ptr[level_end] - a.tile_begin;
            a.ell = g->d_ell_pos;
        }
        a.ell_w = g->ell_w;
        a.pre_rows = P0; a.n_pre = (P0 + a.tile_cap - 1) / a.tile_cap;
        a.order = order_in_use;
        a.x = X; a.qkv_self = at(pl.qkv_self);
        a.kv = at(pl.kv); a.kv_layer_stride = (int64_t)pl.kv_rows * 2 * d;
        a.h_out = Hout;
        a.wqkv_packed = at(pl.wqkv[0]); a.wo_packed = at(pl.wo[0]);
        a.w_layer_stride = L > 1 ? (int64_t)(pl.wqkv[1] - pl.wqkv[0]) : 0;
        a.wkv_packed = at(pl.wkv_a);
        if (ffn) {
            a.ffn = 1; a.w1_packed = at(pl.w1[0]); a.w2_packed = at(pl.w2[0]);
            a.ffn_layer_stride = L > 1 ? (int64_t)(pl.w1[1] - pl.w1[0]) : 0;
        }
        a.rel_bias = (const float*)at(pl.bias_all);
        a.flags = (uint32_t*)at(pl.flags); a.ctrl = (uint32_t*)at(pl.ctrl);
        a.n_layers = L; a.ln_eps = cfg->ln_eps; a.epilogue = epi ? 1 : 0; a.project_kv = 1;
        a.spin_limit = spin_limit;
        a.prof = (cfg->flags & DG4_PROFILE) ? (uint64_t*)((char*)at(pl.ctrl) + 64) : nullptr;
        HIPCHK(dg4_launch_sweep_init(a.flags, a.ctrl, g->n, 0, s));
        HIPCHK(bracket([&]() { return dg4_launch_flow(dt, d, a, s); }));
        return DG4_OK;
    }
    HIPCHK(dg4_launch_sweep_init((uint32_t*)at(pl.flags), (uint32_t*)at(pl.ctrl), 0, 0, s));   // the status words only

    // A sweep over ALL levels of a graph whose levelling (a caller's hint) is deeper than Eq. 1 goes
    // through the Eq. 1 levels instead: as many rounds of launches as the circuit is deep. Same
    // embeddings (every source of a gate lies on a lower Eq. 1 level too); rows of the internal
    // buffers are then positions in that order. DG4_LEVEL_ORDER keeps the caller's levels.
    const bool compact = whole_range && !bounded && !g->eq1_level_ptr.empty() && !(cfg->flags & DG4_LEVEL_ORDER);
    if (compact) {
        rc = dg4_graph_ensure_eq1(g);
        if (rc != DG4_OK) return rc;
    }
    const std::vector<int64_t>& lptr = compact ? g->eq1_level_ptr : g->level_ptr;
    const int32_t* d_order = compact ? g->d_order_eq1 : g->d_order;
    const uint32_t* d_ell_pos = compact ? g->d_ell_eq1 : g->d_ell_pos;
    const int32_t lev_first = compact ? 0 : level_begin;
    const int32_t lev_end = compact ? (int32_t)lptr.size() - 1 : level_end;
    const int32_t lev_count = compact ? (int32_t)lptr.size() - 1 : n_levels;
    // one layer without feed-forward sub-block: the output projection's launch also projects K | V
    const bool fuse_kv = L == 1 && !ffn && !bounded && epi && dg4_gemm_fuses_kv(dt, d);

    // layer 0 projections of x for every gate of the swept levels, in one pass (level by level
    // further down if nothing of the size of the graph may be kept)
    if (!bounded) {
        dg4_gemm_args a{};
        a.a = X; a.a_stride = d; a.a_gather = d_order;
        a.w_packed = at(pl.wqkv[0]); a.n_cols = 3 * d;
        char* base = ws + pl.qkv_self;
        a.out[0] = base; a.out[1] = base + (size_t)d * es; a.out[2] = base + (size_t)2 * d * es;
        a.out_stride = 3 * d;
        a.row_begin = P0; a.row_end = P1;
        HIPCHK(dg4_launch_gemm(dt, d, a, s));
    }

    for (int32_t lev = lev_first; lev < lev_end; ++lev) {
        const int64_t p0 = lptr[lev], p1 = lptr[lev + 1];
        if (p1 == p0) continue;
        if (bounded) {
            // K | V (every layer) of this level's distinct sources, from their final embeddings
            const int64_t f0 = g->front_ptr[lev], f1 = g->front_ptr[lev + 1];
            if (f1 > f0) HIPCHK(kv_project(Hout, d, g->d_front_id + f0, 0, f1 - f0));
        }
        if (bounded) {
            dg4_gemm_args a{};
            a.a = X; a.a_stride = d; a.a_gather = g->d_order;
            a.w_packed = at(pl.wqkv[0]); a.n_cols = 3 * d;
            char* base = (char*)local(pl.qkv_level, p0, 3 * d);
            a.out[0] = base; a.out[1] = base + (size_t)d * es; a.out[2] = base + (size_t)2 * d * es;
            a.out_stride = 3 * d;
            a.row_begin = p0; a.row_end = p1;
            HIPCHK(dg4_launch_gemm(dt, d, a, s));
        }
        for (int l = 0; l < L; ++l) {
            const bool last = l == L - 1;
            dg4_attn_args t{};
            if (l == 0 && !bounded) {
                char* base = ws + pl.qkv_self;
                t.q = base; t.k_self = base + (size_t)d * es; t.v_self = base + (size_t)2 * d * es;
            } else {
                char* base = (char*)local(pl.qkv_level, p0, 3 * d);
                t.q = base; t.k_self = base + (size_t)d * es; t.v_self = base + (size_t)2 * d * es;
            }
            t.q_stride = 3 * d; t.self_stride = 3 * d;
            char* kvb = ws + pl.kv + (size_t)l * pl.kv_rows * 2 * d * es;
            t.k_src = kvb; t.v_src = kvb + (size_t)d * es; t.src_stride = 2 * d;
            t.rel_bias = (const float*)W[WS * l + 2];
            t.ell = bounded ? g->d_ell_front : d_ell_pos; t.ell_w = g->ell_w;
            t.a = local(pl.abuf, p0, d); t.a_stride = d;
            t.row_begin = p0; t.row_end = p1;
            // narrow rows, a level of few gates (bound by the latency of its launches): the attention
            // runs inside the output projection's launch. The same arithmetic either way, so the
            // choice by the size of the level does not show in the result.
            const bool fuse_att = epi && g->ell_w <= 16 && p1 - p0 <= 4096 && dg4_gemm_fuses_kv(dt, d);
            if (!fuse_att) HIPCHK(dg4_launch_attn(dt, d, t, s));

            // s_{l+1} = LN(s_l + a Wo_l), then (DG4_FFN) s_{l+1} <- LN(s_{l+1} + relu(s_{l+1} W1_l) W2_l);
            // the last layer's result is H
            dg4_gemm_args o{};
            o.a = local(pl.abuf, p0, d); o.a_stride = d;
            o.w_packed = at(pl.wo[l]); o.n_cols = d;
            o.row_begin = p0; o.row_end = p1;
            o.epilogue = epi ? 1 : 0; o.ln_eps = cfg->ln_eps;
            if (l == 0) { o.resid = X; o.resid_stride = d; o.resid_gather = d_order; }
            else { o.resid = local((l & 1) ? pl.s1 : pl.s0, p0, d); o.resid_stride = d; }
            void* next = local(((l + 1) & 1) ? pl.s1 : pl.s0, p0, d);
            if (ffn) {
                o.out[0] = local(pl.h1, p0, d); o.out_stride = d;
            } else if (last) {
                o.out[0] = Hout; o.out_stride = d; o.out_scatter = d_order;
                if (!bounded) { o.out2 = at(pl.hpos); o.out2_stride = d; }
                if (fuse_kv && lev + 1 < lev_count) {        // K | V of the level's gates in the same launch
                    o.kv_w_packed = at(pl.wkv_all); o.kv_out = ws + pl.kv; o.kv_stride = 2 * d;
                }
            } else {
                o.out[0] = next; o.out_stride = d;
            }
            if (fuse_att) HIPCHK(dg4_launch_attn_gemm(dt, d, t, o, s));
            else HIPCHK(dg4_launch_gemm(dt, d, o, s));
            if (ffn) {
                dg4_ffn_args f{};
                f.h = local(pl.h1, p0, d); f.h_stride = d;
                f.w1_packed = at(pl.w1[l]); f.w2_packed = at(pl.w2[l]);
                f.row_begin = p0; f.row_end = p1; f.ln_eps = cfg->ln_eps;
                if (last) {
                    f.out = Hout; f.out_stride = d; f.out_scatter = d_order;
                    if (!bounded) { f.out2 = at(pl.hpos); f.out2_stride = d; }
                } else {
                    f.out = next; f.out_stride = d;
                }
                HIPCHK(dg4_launch_ffn(dt, d, f, s));
            }

            if (!last) {
                dg4_gemm_args a{};
                a.a = local(((l + 1) & 1) ? pl.s1 : pl.s0, p0, d); a.a_stride = d;
                a.w_packed = at(pl.wqkv[l + 1]); a.n_cols = 3 * d;
                char* base = (char*)local(pl.qkv_level, p0, 3 * d);
                a.out[0] = base; a.out[1] = base + (size_t)d * es; a.out[2] = base + (size_t)2 * d * es;
                a.out_stride = 3 * d;
                a.row_begin = p0; a.row_end = p1;
                HIPCHK(dg4_launch_gemm(dt, d, a, s));
            }
        }
        // publish K/V of the level's final embeddings for every layer
        if (lev + 1 < lev_count && !bounded && !fuse_kv) HIPCHK(kv_project(at(pl.hpos), d, nullptr, p0, p1));
    }
    return DG4_OK;
}

extern "C" int dg4_layer_status(const dg4_layer_cfg* cfg, const dg4_graph* g, const void* workspace)
{
    const int rc = check_cfg(cfg, true);
    if (rc != DG4_OK) return rc;
    if (!g || !workspace) return DG4_EINVAL;
    const LayerPlan pl = plan_layer(cfg, g);
    uint32_t ctrl[4];
    if (hipMemcpy(ctrl, (const char*)workspace + pl.ctrl, sizeof(ctrl), hipMemcpyDeviceToHost) != hipSuccess) return DG4_EHIP;
    return ctrl[1] ? DG4_EABORTED : DG4_OK;
}

extern "C" int dg4_layer_profile(const dg4_layer_cfg* cfg, const dg4_graph* g, const void* workspace,
                                 uint64_t* ticks8, uint32_t* aborted)
{
    const int rc = check_cfg(cfg, true);
    if (rc != DG4_OK) return rc;
    if (!g || !workspace || !ticks8 || !aborted) return DG4_EINVAL;
    const LayerPlan pl = plan_layer(cfg, g);
    uint32_t ctrl[64];
    if (hipMemcpy(ctrl, (const char*)workspace + pl.ctrl, sizeof(ctrl), hipMemcpyDeviceToHost) != hipSuccess) return DG4_EHIP;
    memcpy(ticks8, ctrl + 16, 8 * sizeof(uint64_t));
    *aborted = ctrl[1];
    return DG4_OK;
}

extern "C" int dg4_sweep_elapsed_ms(float* ms)
{
    SweepEvents& ev = sweep_events();
    if (!ms) return DG4_EINVAL;
    std::lock_guard<std::mutex> lock(ev.mu);
    if (!ev.armed) return DG4_EINVAL;
    if (hipEventSynchronize(ev.b) != hipSuccess) return DG4_EHIP;
    if (hipEventElapsedTime(ms, ev.a, ev.b) != hipSuccess) return DG4_EHIP;
    return DG4_OK;
}
