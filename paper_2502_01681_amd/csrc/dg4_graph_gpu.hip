// Graph analysis of paper Section 3.2 on the device, behind dg4_build_levels_device: validation,
// fanin table, logic levels (Eq. 1) by rounds over the fanin table, the (level, id) order by a
// stable radix sort, cone_k rows with relation codes by a per-gate backward search, and the fanout
// counts of Eq. 2. Integer work throughout: every table equals the host builder's bit for bit
// (nothing here depends on the order in which atomics land: the fanin slot a source takes is not
// observable in any output).
#include <hip/hip_runtime.h>
#include <hipcub/hipcub.hpp>
#include <stdint.h>

#include <algorithm>
#include <memory>
#include <new>
#include <vector>

#include "dg4_internal.h"

namespace {

constexpr int MAXW = 15;            // 2^(3+1) - 1: the largest cone for hops <= 3

// status word: the most negative status any thread reports wins (deterministic for a list with
// one kind of defect; for several kinds the host call reports the first in edge order instead)
__device__ __forceinline__ void report(int* status, int code) { atomicMin(status, code); }

__global__ void fanin_kernel(int64_t n, int64_t e, const int32_t* es, const int32_t* ed, const uint8_t* ei,
                             int32_t* fin, uint8_t* finv, int32_t* deg, int* status)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= e) return;
    const int64_t u = es[i], v = ed[i];
    if (u < 0 || u >= n || v < 0 || v >= n) { report(status, DG4_ERANGE); return; }
    if (ei[i] > 1) { report(status, DG4_EINVAL); return; }
    if (u == v) { report(status, DG4_ECYCLE); return; }
    const int slot = atomicAdd(&deg[v], 1);
    if (slot >= 2) { report(status, DG4_EFANIN); return; }
    fin[2 * v + slot] = (int32_t)u;
    finv[2 * v + slot] = ei[i];
}

// duplicated fanin pair; primary inputs start at level 0 and are done
__global__ void fanin_check_kernel(int64_t n, const int32_t* fin, const int32_t* deg, int32_t* level, uint8_t* done, int* status)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    if (deg[v] == 2 && fin[2 * v] == fin[2 * v + 1]) report(status, DG4_EFANIN);
    level[v] = 0;
    done[v] = deg[v] == 0;
}

// One round of Eq. 1: a gate whose fanins were all done BEFORE this round gets max + 1. Two flag
// arrays alternate so that a round reads only the previous round's state (level[] of a fanin is
// final once its flag is set). progress[0] counts the gates finished so far.
__global__ void level_round_kernel(int64_t n, const int32_t* fin, const int32_t* deg, const uint8_t* done_in,
                                   uint8_t* done_out, int32_t* level, unsigned long long* progress)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    if (done_in[v]) { done_out[v] = 1; return; }
    const int d = deg[v];
    int32_t best = -1;
    bool ready = true;
    for (int k = 0; k < d; ++k) {
        const int32_t u = fin[2 * v + k];
        if (done_in[u]) best = max(best, level[u]); else ready = false;
    }
    if (ready) { level[v] = best + 1; atomicAdd(progress, 1ull); }
    done_out[v] = ready;
}

__global__ void count_done_kernel(int64_t n, const uint8_t* done, unsigned long long* progress)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n && done[v]) atomicAdd(progress, 1ull);
}

// a caller's levelling: non-negative, 0 exactly on primary inputs' side of the rule, strictly
// increasing along every edge (which also rules out cycles)
__global__ void hint_check_kernel(int64_t n, const int32_t* fin, const int32_t* deg, const int32_t* hint, int32_t* level, int* status)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    const int32_t h = hint[v];
    bool ok = h >= 0 && !(deg[v] == 0 && h != 0);
    for (int k = 0; k < deg[v]; ++k) ok = ok && hint[fin[2 * v + k]] < h;
    if (!ok) report(status, DG4_EHINT);
    level[v] = h;
}

__global__ void iota_max_kernel(int64_t n, const int32_t* level, int32_t* ids, int32_t* max_level)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int32_t m = 0;
    if (v < n) { ids[v] = (int32_t)v; m = level[v]; }
    for (int off = 32; off > 0; off >>= 1) m = max(m, __shfl_xor(m, off));     // one atomic per wave
    if ((threadIdx.x & 63) == 0) atomicMax(max_level, m);
}

// level_ptr[l] = first position whose level is >= l, l = 0 .. max_level + 1 (binary search in the sorted keys)
__global__ void level_ptr_kernel(int64_t n, const int32_t* sorted_level, int32_t n_ptr, int64_t* level_ptr)
{
    const int32_t l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= n_ptr) return;
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (sorted_level[mid] < l) lo = mid + 1; else hi = mid;
    }
    level_ptr[l] = lo;
}

// cone_k(v) by a backward breadth-first search over the fanin table: the first visit fixes the
// smallest hop count, hence the relation code (0 self, 1 / 2 direct fanin plain / inverted,
// 3 reached by two or more edges); the row is then sorted by id. Fixed-width rows; counts in cnt.
__global__ void cone_kernel(int64_t n, int hops, const int32_t* fin, const uint8_t* finv, const int32_t* deg,
                            int32_t* row_id, uint8_t* row_rel, int64_t* cnt)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    int32_t id[MAXW];
    uint8_t rel[MAXW], hop[MAXW];
    int c = 0;
    id[0] = (int32_t)v; rel[0] = 0; hop[0] = 0; c = 1;
    for (int head = 0; head < c; ++head) {
        if (hop[head] == hops) continue;
        const int32_t w = id[head];
        const int d = deg[w];
        for (int k = 0; k < d; ++k) {
            const int32_t u = fin[2 * (int64_t)w + k];
            bool seen = false;
            for (int j = 0; j < c; ++j) seen = seen || id[j] == u;
            if (seen) continue;
            id[c] = u; hop[c] = (uint8_t)(hop[head] + 1);
            rel[c] = hop[c] == 1 ? (uint8_t)(1 + finv[2 * (int64_t)w + k]) : (uint8_t)3;
            ++c;
        }
    }
    for (int i = 1; i < c; ++i) {                       // insertion sort by id
        const int32_t ti = id[i]; const uint8_t tr = rel[i];
        int j = i - 1;
        while (j >= 0 && id[j] > ti) { id[j + 1] = id[j]; rel[j + 1] = rel[j]; --j; }
        id[j + 1] = ti; rel[j + 1] = tr;
    }
    for (int i = 0; i < c; ++i) { row_id[v * MAXW + i] = id[i]; row_rel[v * MAXW + i] = rel[i]; }
    cnt[v] = c;
}

// Cones deeper than three hops, one hop at a time: cone_j(v) = {v} u cone_{j-1}(f0) u cone_{j-1}(f1) over
// the fanins f0, f1 of v, as a merge of id-sorted rows (a gate with no fanin keeps {v}). One thread
// per gate walks the two rows and its own id in step; FILL = false counts the distinct ids, FILL =
// true writes them (ascending) and, if rel is given, their relation codes: 0 the gate itself, 1 / 2 a
// direct fanin (plain / inverted: the shortest path decides, Section 3.5), 3 anything further.
// prev_ptr == nullptr stands for the rows of zero hops ({u} for every u).
template <bool FILL>
__global__ void cone_merge_kernel(int64_t n, const int32_t* fin, const uint8_t* finv, const int32_t* deg,
                                  const int64_t* prev_ptr, const int32_t* prev_idx,
                                  int64_t* cnt, const int64_t* ptr, int32_t* idx, uint8_t* rel)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    const int d = deg[v];
    const int32_t f0 = d > 0 ? fin[2 * v] : -1, f1 = d > 1 ? fin[2 * v + 1] : -1;
    int64_t a = 0, a1 = 0, b = 0, b1 = 0;          // [a, a1) and [b, b1): the rows of f0 and f1
    int32_t self0 = f0, self1 = f1;                // (zero hops: the row of u is u itself)
    if (prev_ptr) {
        if (f0 >= 0) { a = prev_ptr[f0]; a1 = prev_ptr[f0 + 1]; }
        if (f1 >= 0) { b = prev_ptr[f1]; b1 = prev_ptr[f1 + 1]; }
    } else {
        a1 = f0 >= 0 ? 1 : 0; b1 = f1 >= 0 ? 1 : 0;
    }
    auto at_a = [&](int64_t i) { return prev_ptr ? prev_idx[i] : self0; };
    auto at_b = [&](int64_t i) { return prev_ptr ? prev_idx[i] : self1; };
    bool self_left = true;
    int64_t out = FILL ? ptr[v] : 0, count = 0;
    const int32_t none = 0x7FFFFFFF;
    int32_t xa = a < a1 ? at_a(a) : none, xb = b < b1 ? at_b(b) : none;
    for (;;) {
        const int32_t xs = self_left ? (int32_t)v : none;
        int32_t m = xa < xb ? xa : xb;
        m = xs < m ? xs : m;
        if (m == none) break;
        if (FILL) {
            idx[out] = m;
            if (rel) rel[out] = m == (int32_t)v ? 0 : m == f0 ? (uint8_t)(1 + finv[2 * v]) : m == f1 ? (uint8_t)(1 + finv[2 * v + 1]) : (uint8_t)3;
            ++out;
        }
        ++count;
        if (xa == m) { ++a; xa = a < a1 ? at_a(a) : none; }
        if (xb == m) { ++b; xb = b < b1 ? at_b(b) : none; }
        if (xs == m) self_left = false;
    }
    if (!FILL) cnt[v] = count;
}

__global__ void compact_kernel(int64_t n, const int32_t* row_id, const uint8_t* row_rel, const int64_t* nbr_ptr,
                               int32_t* nbr_idx, uint8_t* nbr_rel)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    const int64_t p0 = nbr_ptr[v];
    const int c = (int)(nbr_ptr[v + 1] - p0);
    for (int i = 0; i < c; ++i) { nbr_idx[p0 + i] = row_id[v * MAXW + i]; nbr_rel[p0 + i] = row_rel[v * MAXW + i]; }
}

// Fanout counts of Eq. 2 from the fanin table (integer atomics: the sums do not depend on order)
__global__ void fanout_kernel(int64_t n, const int32_t* fin, const uint8_t* finv, const int32_t* deg,
                              int32_t* out_and, int32_t* out_not, uint8_t* inverter)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    const int d = deg[v];
    if (d == 1) { atomicAdd(&out_not[fin[2 * v]], 1); return; }        // v is a NOT / buffer gate
    for (int k = 0; k < d; ++k) {
        const int32_t u = fin[2 * v + k];
        if (finv[2 * v + k]) inverter[u] = 1; else atomicAdd(&out_and[u], 1);
    }
}
__global__ void add_inverter_kernel(int64_t n, int32_t* out_not, const uint8_t* inverter)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n) out_not[v] += inverter[v];
}

// ---- partition and updating strategy (Algorithms 1 and 2 with marks) on the device.
// Kinds of cone roots, as in the host analysis: 0 a gate on a stride level (level >= k and (level - k)
// a multiple of the stride), 1 a gate nobody reads, 2 a gate that no cone of the first two kinds
// holds (it roots its own cone); PART_NONE: not a root.
constexpr uint8_t PART_NONE = 255;

__global__ void part_read_kernel(int64_t n, const int32_t* fin, const int32_t* deg, uint8_t* is_read)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    for (int i = 0; i < deg[v]; ++i) is_read[fin[2 * v + i]] = 1;       // (every writer stores the same byte)
}

__global__ void part_kind_kernel(int64_t n, int32_t k, int32_t stride, const int32_t* level, const uint8_t* is_read, uint8_t* kind)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    const int32_t l = level[v];
    kind[v] = l >= k && (l - k) % stride == 0 ? (uint8_t)0 : !is_read[v] ? (uint8_t)1 : PART_NONE;
}

// one wave per gate: the members of the cones rooted so far are covered
__global__ void part_cover_kernel(int64_t n, const uint8_t* kind, const int64_t* nbr_ptr, const int32_t* nbr_idx, uint8_t* covered)
{
    const int64_t v = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (v >= n || kind[v] == PART_NONE) return;
    for (int64_t j = nbr_ptr[v] + lane; j < nbr_ptr[v + 1]; j += 64) covered[nbr_idx[j]] = 1;
}

// sort key of position q of the (level, id) order: roots by (level, kind), everything else behind them
__global__ void part_key_kernel(int64_t n, const int32_t* order, const int32_t* level, uint8_t* kind, const uint8_t* covered,
                                uint32_t none_key, uint32_t* key, unsigned long long* n_roots)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n) return;
    const int32_t v = order[q];
    uint8_t kd = kind[v];
    if (kd == PART_NONE && !covered[v]) { kd = 2; kind[v] = 2; }
    key[q] = kd == PART_NONE ? none_key : ((uint32_t)level[v] << 2) | kd;
    if (kd != PART_NONE) atomicAdd(n_roots, 1ull);
}

__global__ void part_fill_stage_kernel(int64_t n, int32_t* stage)
{
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n) stage[v] = INT32_MAX;
}

// one wave per cone: a gate is computed by the first mini-batch that holds it
__global__ void part_stage_kernel(int64_t n_cones, const int32_t* cone_root, const int32_t* cone_stage,
                                  const int64_t* nbr_ptr, const int32_t* nbr_idx, int32_t* stage)
{
    const int64_t c = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (c >= n_cones) return;
    const int32_t r = cone_root[c];
    const int32_t st = cone_stage[c];
    for (int64_t j = nbr_ptr[r] + lane; j < nbr_ptr[r + 1]; j += 64) atomicMin(&stage[nbr_idx[j]], st);
}

// one wave per cone, a lane per member v computed in the cone's mini-batch: the entries of row(v) that
// also lie in row(root) are kept (two rows of ascending ids, merged; every writer stores the same byte)
__global__ void part_keep_kernel(int64_t n_cones, const int32_t* cone_root, const int32_t* cone_stage, const int32_t* stage,
                                 const int64_t* nbr_ptr, const int32_t* nbr_idx, uint8_t* keep)
{
    const int64_t c = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (c >= n_cones) return;
    const int32_t r = cone_root[c];
    const int32_t st = cone_stage[c];
    const int64_t r0 = nbr_ptr[r], r1 = nbr_ptr[r + 1];
    for (int64_t j = r0 + lane; j < r1; j += 64) {
        const int32_t v = nbr_idx[j];
        if (stage[v] != st) continue;
        int64_t a = nbr_ptr[v], b = r0;
        const int64_t a1 = nbr_ptr[v + 1];
        while (a < a1 && b < r1) {
            const int32_t x = nbr_idx[a], y = nbr_idx[b];
            if (x == y) { keep[a] = 1; ++a; ++b; }
            else if (x < y) ++a;
            else ++b;
        }
    }
}

// one wave per gate: kept entries counted, then (FILL) written in order behind new_ptr[v]
template <bool FILL>
__global__ void part_compact_kernel(int64_t n, const int64_t* nbr_ptr, const int32_t* nbr_idx, const uint8_t* nbr_rel, const uint8_t* keep,
                                    int64_t* cnt, const int64_t* new_ptr, int32_t* new_idx, uint8_t* new_rel)
{
    const int64_t v = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (v >= n) return;
    int64_t out = FILL ? new_ptr[v] : 0;
    for (int64_t j0 = nbr_ptr[v]; j0 < nbr_ptr[v + 1]; j0 += 64) {
        const int64_t j = j0 + lane;
        const bool k = j < nbr_ptr[v + 1] && keep[j] != 0;
        const unsigned long long m = __ballot(k);
        if (FILL && k) {
            const int64_t o = out + __popcll(m & ((1ull << lane) - 1ull));
            new_idx[o] = nbr_idx[j]; new_rel[o] = nbr_rel[j];
        }
        out += __popcll(m);
    }
    if (!FILL && lane == 0) cnt[v] = out;
}

// Device memory of one call: carved out of at most two allocations (the tables sized by the node
// count, then those sized by the number of neighbour entries), released when the call returns.
struct Arena {
    std::vector<void*> blocks;
    char* cur = nullptr;
    size_t left = 0;
    ~Arena() { for (void* p : blocks) (void)hipFree(p); }
    bool reserve(size_t bytes)
    {
        void* p = nullptr;
        if (hipMalloc(&p, bytes + 256) != hipSuccess) return false;
        blocks.push_back(p);
        cur = (char*)p; left = bytes + 256;
        return true;
    }
    template <typename T> T* get(size_t count, bool zero, hipStream_t s)
    {
        const size_t bytes = (std::max<size_t>(count, 1) * sizeof(T) + 255) & ~(size_t)255;
        if (bytes > left && !reserve(bytes)) return nullptr;
        T* p = (T*)cur;
        cur += bytes; left -= bytes;
        if (zero && hipMemsetAsync(p, 0, bytes, s) != hipSuccess) return nullptr;
        return p;
    }
};

inline unsigned blocks_for(int64_t items) { return (unsigned)((items + 255) / 256); }

#define GPU_CHECK(expr) do { if ((expr) != hipSuccess) return DG4_EHIP; } while (0)
#define GPU_ALLOC(var, T, count, zero) T* var = arena.get<T>((count), (zero), s); if (!var) return DG4_ENOMEM

// stride == 0: plain cone rows; else the rows of the partitioned update with marks
int build_device(int64_t n, int64_t e, const int32_t* es, const int32_t* ed, const uint8_t* ei, int32_t hops,
                 const int32_t* level_hint, int32_t stride, int32_t batch, void* stream, dg4_graph** out)
{
    if (!out || n < 0 || e < 0 || (e > 0 && (!es || !ed || !ei))) return DG4_EINVAL;
    if (hops < 1 || hops > DG4_MAX_HOPS) return DG4_EUNSUPPORTED;
    if (n >= (int64_t)0x3FFFFFFF) return DG4_EUNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    try {
        std::unique_ptr<dg4_graph> g(new dg4_graph());
        g->n = n; g->e = e; g->hops = hops;
        if (n == 0) {
            g->level_ptr.assign(2, 0); g->nbr_ptr.assign(1, 0);
            if (stride > 0) { g->cone_group_ptr.assign(1, 0); g->stride = stride; g->batch_cones = batch; }
            *out = g.release();
            return DG4_OK;
        }
        Arena arena;
        // everything sized by the node count in one allocation (about 140 bytes a node, plus the
        // sort's and the scan's own scratch, which are small)
        if (!arena.reserve((size_t)n * 160 + (16u << 20))) return DG4_ENOMEM;
        GPU_ALLOC(fin, int32_t, 2 * (size_t)n, false);
        GPU_ALLOC(finv, uint8_t, 2 * (size_t)n, true);
        GPU_ALLOC(deg, int32_t, (size_t)n, true);
        GPU_ALLOC(level, int32_t, (size_t)n, false);
        GPU_ALLOC(done_a, uint8_t, (size_t)n, false);
        GPU_ALLOC(done_b, uint8_t, (size_t)n, false);
        GPU_ALLOC(status, int, 1, true);
        GPU_ALLOC(progress, unsigned long long, 1, true);
        GPU_ALLOC(max_level, int32_t, 1, true);
        const unsigned nb = blocks_for(n);

        if (e > 0) hipLaunchKernelGGL(fanin_kernel, dim3(blocks_for(e)), dim3(256), 0, s, n, e, es, ed, ei, fin, finv, deg, status);
        hipLaunchKernelGGL(fanin_check_kernel, dim3(nb), dim3(256), 0, s, n, fin, deg, level, done_a, status);
        int st = 0;
        GPU_CHECK(hipMemcpyAsync(&st, status, sizeof(int), hipMemcpyDeviceToHost, s));
        GPU_CHECK(hipStreamSynchronize(s));
        if (st != DG4_OK) return st;

        if (level_hint) {
            hipLaunchKernelGGL(hint_check_kernel, dim3(nb), dim3(256), 0, s, n, fin, deg, level_hint, level, status);
            GPU_CHECK(hipMemcpyAsync(&st, status, sizeof(int), hipMemcpyDeviceToHost, s));
            GPU_CHECK(hipStreamSynchronize(s));
            if (st != DG4_OK) return st;
        } else {
            // rounds of Eq. 1, a batch at a time; no progress in a batch with gates left = a cycle
            hipLaunchKernelGGL(count_done_kernel, dim3(nb), dim3(256), 0, s, n, done_a, progress);
            unsigned long long finished = 0, before = ~0ull;
            uint8_t* cur = done_a; uint8_t* nxt = done_b;
            for (;;) {
                GPU_CHECK(hipMemcpyAsync(&finished, progress, sizeof(finished), hipMemcpyDeviceToHost, s));
                GPU_CHECK(hipStreamSynchronize(s));
                if (finished == (unsigned long long)n) break;
                if (finished == before) return DG4_ECYCLE;
                before = finished;
                for (int r = 0; r < 32; ++r) {
                    hipLaunchKernelGGL(level_round_kernel, dim3(nb), dim3(256), 0, s, n, fin, deg, cur, nxt, level, progress);
                    std::swap(cur, nxt);
                }
            }
        }

        // (level, id) order: stable sort of the ids by level
        GPU_ALLOC(ids, int32_t, (size_t)n, false);
        GPU_ALLOC(sorted_level, int32_t, (size_t)n, false);
        GPU_ALLOC(order, int32_t, (size_t)n, false);
        hipLaunchKernelGGL(iota_max_kernel, dim3(nb), dim3(256), 0, s, n, level, ids, max_level);
        int32_t h_max = 0;
        GPU_CHECK(hipMemcpyAsync(&h_max, max_level, sizeof(int32_t), hipMemcpyDeviceToHost, s));
        GPU_CHECK(hipStreamSynchronize(s));
        g->max_level = h_max;
        int bits = 1;
        while (bits < 31 && (h_max >> bits) != 0) ++bits;
        size_t sort_bytes = 0;
        GPU_CHECK(hipcub::DeviceRadixSort::SortPairs(nullptr, sort_bytes, level, sorted_level, ids, order, (int)n, 0, bits, s));
        GPU_ALLOC(sort_tmp, unsigned char, sort_bytes, false);
        GPU_CHECK(hipcub::DeviceRadixSort::SortPairs(sort_tmp, sort_bytes, level, sorted_level, ids, order, (int)n, 0, bits, s));
        const int32_t n_ptr = h_max + 2;
        GPU_ALLOC(level_ptr, int64_t, (size_t)n_ptr, false);
        hipLaunchKernelGGL(level_ptr_kernel, dim3(blocks_for(n_ptr)), dim3(256), 0, s, n, sorted_level, n_ptr, level_ptr);

        // cones
        GPU_ALLOC(cnt, int64_t, (size_t)n + 1, true);
        GPU_ALLOC(nbr_ptr, int64_t, (size_t)n + 1, false);
        size_t scan_bytes = 0;
        GPU_CHECK(hipcub::DeviceScan::ExclusiveSum(nullptr, scan_bytes, cnt, nbr_ptr, (int)(n + 1), s));
        GPU_ALLOC(scan_tmp, unsigned char, scan_bytes, false);
        int64_t nnz = 0;
        int32_t* nbr_idx = nullptr;
        uint8_t* nbr_rel = nullptr;
        if (hops <= 3) {
            GPU_ALLOC(row_id, int32_t, (size_t)n * MAXW, false);
            GPU_ALLOC(row_rel, uint8_t, (size_t)n * MAXW, false);
            hipLaunchKernelGGL(cone_kernel, dim3(nb), dim3(256), 0, s, n, (int)hops, fin, finv, deg, row_id, row_rel, cnt);
            GPU_CHECK(hipcub::DeviceScan::ExclusiveSum(scan_tmp, scan_bytes, cnt, nbr_ptr, (int)(n + 1), s));
            GPU_CHECK(hipMemcpyAsync(&nnz, nbr_ptr + n, sizeof(int64_t), hipMemcpyDeviceToHost, s));
            GPU_CHECK(hipStreamSynchronize(s));
            if (!arena.reserve((size_t)nnz * 5 + 1024)) return DG4_ENOMEM;
            nbr_idx = arena.get<int32_t>((size_t)nnz, false, s);
            nbr_rel = arena.get<uint8_t>((size_t)nnz, false, s);
            if (!nbr_idx || !nbr_rel) return DG4_ENOMEM;
            hipLaunchKernelGGL(compact_kernel, dim3(nb), dim3(256), 0, s, n, row_id, row_rel, nbr_ptr, nbr_idx, nbr_rel);
        } else {
            // one hop at a time, rows of hop j from those of hop j - 1 (count, scan, fill); the row
            // pointers of two consecutive hops alternate between two buffers
            GPU_ALLOC(ptr_b, int64_t, (size_t)n + 1, false);
            int64_t* ptr_cur = nbr_ptr;
            int64_t* ptr_prev = nullptr;
            int32_t* idx_prev = nullptr;
            for (int32_t j = 1; j <= hops; ++j) {
                hipLaunchKernelGGL(cone_merge_kernel<false>, dim3(nb), dim3(256), 0, s, n, fin, finv, deg,
                                   (const int64_t*)ptr_prev, (const int32_t*)idx_prev, cnt, (const int64_t*)nullptr, (int32_t*)nullptr, (uint8_t*)nullptr);
                GPU_CHECK(hipcub::DeviceScan::ExclusiveSum(scan_tmp, scan_bytes, cnt, ptr_cur, (int)(n + 1), s));
                GPU_CHECK(hipMemcpyAsync(&nnz, ptr_cur + n, sizeof(int64_t), hipMemcpyDeviceToHost, s));
                GPU_CHECK(hipStreamSynchronize(s));
                const bool final_hop = j == hops;
                if (!arena.reserve((size_t)nnz * (final_hop ? 5 : 4) + 1024)) return DG4_ENOMEM;
                int32_t* idx_cur = arena.get<int32_t>((size_t)nnz, false, s);
                uint8_t* rel_cur = final_hop ? arena.get<uint8_t>((size_t)nnz, false, s) : nullptr;
                if (!idx_cur || (final_hop && !rel_cur)) return DG4_ENOMEM;
                hipLaunchKernelGGL(cone_merge_kernel<true>, dim3(nb), dim3(256), 0, s, n, fin, finv, deg,
                                   (const int64_t*)ptr_prev, (const int32_t*)idx_prev, (int64_t*)nullptr, (const int64_t*)ptr_cur, idx_cur, rel_cur);
                nbr_idx = idx_cur; nbr_rel = rel_cur;
                ptr_prev = ptr_cur; idx_prev = idx_cur;
                ptr_cur = ptr_cur == nbr_ptr ? ptr_b : nbr_ptr;
            }
            if (ptr_prev != nbr_ptr)             // the last hop's pointers, where the copies below expect them
                GPU_CHECK(hipMemcpyAsync(nbr_ptr, ptr_prev, ((size_t)n + 1) * sizeof(int64_t), hipMemcpyDeviceToDevice, s));
        }
        // ---- partition and updating strategy: roots, mini-batch numbers, rows restricted to the cones
        // a gate shares with the mini-batch that computes it (the host analysis, step by step)
        int32_t* stage = nullptr;
        if (stride > 0) {
            GPU_ALLOC(is_read, uint8_t, (size_t)n, true);
            GPU_ALLOC(kind, uint8_t, (size_t)n, false);
            GPU_ALLOC(covered, uint8_t, (size_t)n, true);
            GPU_ALLOC(pkey, uint32_t, (size_t)n, false);
            GPU_ALLOC(pkey_sorted, uint32_t, (size_t)n, false);
            GPU_ALLOC(roots_sorted, int32_t, (size_t)n, false);
            GPU_ALLOC(n_roots_d, unsigned long long, 1, true);
            const unsigned nb_wave = blocks_for(n * 64);
            hipLaunchKernelGGL(part_read_kernel, dim3(nb), dim3(256), 0, s, n, fin, deg, is_read);
            hipLaunchKernelGGL(part_kind_kernel, dim3(nb), dim3(256), 0, s, n, hops, stride, level, is_read, kind);
            hipLaunchKernelGGL(part_cover_kernel, dim3(nb_wave), dim3(256), 0, s, n, kind, nbr_ptr, nbr_idx, covered);
            const uint32_t none_key = ((uint32_t)h_max + 1u) << 2;
            hipLaunchKernelGGL(part_key_kernel, dim3(nb), dim3(256), 0, s, n, order, level, kind, covered, none_key, pkey, n_roots_d);
            int key_bits = 1;
            while (key_bits < 32 && (none_key >> key_bits) != 0) ++key_bits;
            size_t psort_bytes = 0;
            GPU_CHECK(hipcub::DeviceRadixSort::SortPairs(nullptr, psort_bytes, pkey, pkey_sorted, order, roots_sorted, (int)n, 0, key_bits, s));
            GPU_ALLOC(psort_tmp, unsigned char, psort_bytes, false);
            GPU_CHECK(hipcub::DeviceRadixSort::SortPairs(psort_tmp, psort_bytes, pkey, pkey_sorted, order, roots_sorted, (int)n, 0, key_bits, s));
            unsigned long long n_roots = 0;
            GPU_CHECK(hipMemcpyAsync(&n_roots, n_roots_d, sizeof(n_roots), hipMemcpyDeviceToHost, s));
            GPU_CHECK(hipStreamSynchronize(s));
            // the lists (one per level that has roots) and the running number of every cone's mini-batch
            std::vector<uint32_t> keys((size_t)n_roots);
            g->cone_root.resize((size_t)n_roots);
            GPU_CHECK(hipMemcpyAsync(keys.data(), pkey_sorted, (size_t)n_roots * 4, hipMemcpyDeviceToHost, s));
            GPU_CHECK(hipMemcpyAsync(g->cone_root.data(), roots_sorted, (size_t)n_roots * 4, hipMemcpyDeviceToHost, s));
            GPU_CHECK(hipStreamSynchronize(s));
            std::vector<int32_t> cone_stage((size_t)n_roots);
            int32_t next_stage = 0;
            for (size_t c = 0; c < (size_t)n_roots;) {
                const uint32_t l = keys[c] >> 2;
                size_t c1 = c;
                while (c1 < (size_t)n_roots && (keys[c1] >> 2) == l) ++c1;
                g->cone_group_level.push_back((int32_t)l);
                g->cone_group_ptr.push_back((int64_t)c);
                for (size_t i = c; i < c1; ++i) cone_stage[i] = next_stage + (int32_t)((i - c) / (size_t)batch);
                next_stage += (int32_t)((c1 - c + (size_t)batch - 1) / (size_t)batch);
                c = c1;
            }
            g->cone_group_ptr.push_back((int64_t)n_roots);
            g->stride = stride; g->batch_cones = batch;
            GPU_ALLOC(cone_stage_d, int32_t, (size_t)n_roots, false);
            GPU_CHECK(hipMemcpyAsync(cone_stage_d, cone_stage.data(), (size_t)n_roots * 4, hipMemcpyHostToDevice, s));
            stage = arena.get<int32_t>((size_t)n, false, s);
            if (!stage) return DG4_ENOMEM;
            hipLaunchKernelGGL(part_fill_stage_kernel, dim3(nb), dim3(256), 0, s, n, stage);
            const unsigned cb_wave = blocks_for((int64_t)n_roots * 64);
            if (n_roots)
                hipLaunchKernelGGL(part_stage_kernel, dim3(cb_wave), dim3(256), 0, s, (int64_t)n_roots, roots_sorted, cone_stage_d, nbr_ptr, nbr_idx, stage);
            if (!arena.reserve((size_t)nnz + 1024)) return DG4_ENOMEM;
            uint8_t* keep = arena.get<uint8_t>((size_t)nnz, true, s);
            if (!keep) return DG4_ENOMEM;
            if (n_roots)
                hipLaunchKernelGGL(part_keep_kernel, dim3(cb_wave), dim3(256), 0, s, (int64_t)n_roots, roots_sorted, cone_stage_d, stage, nbr_ptr, nbr_idx, keep);
            GPU_ALLOC(part_ptr, int64_t, (size_t)n + 1, false);
            hipLaunchKernelGGL(part_compact_kernel<false>, dim3(nb_wave), dim3(256), 0, s, n, nbr_ptr, nbr_idx, nbr_rel, keep,
                               cnt, (const int64_t*)nullptr, (int32_t*)nullptr, (uint8_t*)nullptr);
            GPU_CHECK(hipcub::DeviceScan::ExclusiveSum(scan_tmp, scan_bytes, cnt, part_ptr, (int)(n + 1), s));
            int64_t nnz2 = 0;
            GPU_CHECK(hipMemcpyAsync(&nnz2, part_ptr + n, sizeof(int64_t), hipMemcpyDeviceToHost, s));
            GPU_CHECK(hipStreamSynchronize(s));        // (the stream's copy of cone_stage has been consumed too)
            if (!arena.reserve((size_t)nnz2 * 5 + 1024)) return DG4_ENOMEM;
            int32_t* idx2 = arena.get<int32_t>((size_t)nnz2, false, s);
            uint8_t* rel2 = arena.get<uint8_t>((size_t)nnz2, false, s);
            if (!idx2 || !rel2) return DG4_ENOMEM;
            hipLaunchKernelGGL(part_compact_kernel<true>, dim3(nb_wave), dim3(256), 0, s, n, nbr_ptr, nbr_idx, nbr_rel, keep,
                               (int64_t*)nullptr, (const int64_t*)part_ptr, idx2, rel2);
            GPU_CHECK(hipMemcpyAsync(nbr_ptr, part_ptr, ((size_t)n + 1) * sizeof(int64_t), hipMemcpyDeviceToDevice, s));
            nbr_idx = idx2; nbr_rel = rel2; nnz = nnz2;
        }
        g->nnz = nnz;

        // fanout counts of the structural encoding
        GPU_ALLOC(out_and, int32_t, (size_t)n, true);
        GPU_ALLOC(out_not, int32_t, (size_t)n, true);
        GPU_ALLOC(inverter, uint8_t, (size_t)n, true);
        hipLaunchKernelGGL(fanout_kernel, dim3(nb), dim3(256), 0, s, n, fin, finv, deg, out_and, out_not, inverter);
        hipLaunchKernelGGL(add_inverter_kernel, dim3(nb), dim3(256), 0, s, n, out_not, inverter);
        GPU_CHECK(hipGetLastError());

        // host copies: the graph object hands them out and derives its device tables from them
        g->level.resize((size_t)n); g->order.resize((size_t)n); g->pos.resize((size_t)n);
        g->level_ptr.resize((size_t)n_ptr); g->nbr_ptr.resize((size_t)n + 1);
        g->nbr_idx.resize((size_t)nnz); g->nbr_rel.resize((size_t)nnz);
        g->out_and.resize((size_t)n); g->out_not.resize((size_t)n);
        GPU_CHECK(hipMemcpyAsync(g->level.data(), level, (size_t)n * 4, hipMemcpyDeviceToHost, s));
        GPU_CHECK(hipMemcpyAsync(g->order.data(), order, (size_t)n * 4, hipMemcpyDeviceToHost, s));
        GPU_CHECK(hipMemcpyAsync(g->level_ptr.data(), level_ptr, (size_t)n_ptr * 8, hipMemcpyDeviceToHost, s));
        GPU_CHECK(hipMemcpyAsync(g->nbr_ptr.data(), nbr_ptr, ((size_t)n + 1) * 8, hipMemcpyDeviceToHost, s));
        GPU_CHECK(hipMemcpyAsync(g->nbr_idx.data(), nbr_idx, (size_t)nnz * 4, hipMemcpyDeviceToHost, s));
        GPU_CHECK(hipMemcpyAsync(g->nbr_rel.data(), nbr_rel, (size_t)nnz, hipMemcpyDeviceToHost, s));
        GPU_CHECK(hipMemcpyAsync(g->out_and.data(), out_and, (size_t)n * 4, hipMemcpyDeviceToHost, s));
        GPU_CHECK(hipMemcpyAsync(g->out_not.data(), out_not, (size_t)n * 4, hipMemcpyDeviceToHost, s));
        if (stage) {
            g->stage.resize((size_t)n);
            GPU_CHECK(hipMemcpyAsync(g->stage.data(), stage, (size_t)n * 4, hipMemcpyDeviceToHost, s));
        }
        GPU_CHECK(hipStreamSynchronize(s));
        for (int64_t p = 0; p < n; ++p) g->pos[(size_t)g->order[(size_t)p]] = (int32_t)p;
        *out = g.release();
        return DG4_OK;
    } catch (const std::bad_alloc&) {
        return DG4_ENOMEM;
    } catch (...) {
        return DG4_EINVAL;
    }
}

}  // namespace

extern "C" int dg4_build_levels_device(int64_t n, int64_t e, const int32_t* es, const int32_t* ed,
                                       const uint8_t* ei, int32_t hops, const int32_t* level_hint,
                                       void* stream, dg4_graph** out)
{
    return build_device(n, e, es, ed, ei, hops, level_hint, 0, 0, stream, out);
}

extern "C" int dg4_build_partitioned_device(int64_t n, int64_t e, const int32_t* es, const int32_t* ed,
                                            const uint8_t* ei, int32_t hops, const int32_t* level_hint,
                                            int32_t stride, int32_t batch_cones, void* stream, dg4_graph** out)
{
    if (hops < 1 || hops > DG4_MAX_HOPS) return DG4_EUNSUPPORTED;
    if (stride < 1 || stride >= hops || batch_cones < 1) return DG4_EINVAL;
    return build_device(n, e, es, ed, ei, hops, level_hint, stride, batch_cones, stream, out);
}
