// Graph analysis of paper Section 3.2 on the device, behind dg4_build_levels_device: validation,
// fanin table, logic levels (Eq. 1) by rounds over the fanin table, the (level, id) order by a
// stable radix sort (this file's own, like its prefix sum), cone_k rows with relation codes by a per-gate backward search, and the fanout
// counts of Eq. 2. Integer work throughout: every table equals the host builder's bit for bit
// (nothing here depends on the order in which atomics land: the fanin slot a source takes is not
// observable in any output).
#include <hip/hip_runtime.h>
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

// ---- two primitives of this file's own: an exclusive prefix sum of 64-bit counts, and a stable
// sort of (32-bit key, 32-bit value) pairs by the key's low bits, least significant digit first.
// Both are deterministic: no result depends on the order in which workgroups run.
constexpr int SCAN_ITEMS = 8, SCAN_CHUNK = 256 * SCAN_ITEMS;      // consecutive items per thread, per workgroup
constexpr int RADIX_BITS = 8, RADIX = 1 << RADIX_BITS;
constexpr int SORT_ROUNDS = 16, SORT_CHUNK = 256 * SORT_ROUNDS;   // items per workgroup, 256 at a time

// exclusive prefix of v over the 256 threads of a workgroup (in thread order) and the workgroup's total
__device__ __forceinline__ int64_t block_exclusive(int64_t v, int64_t* total)
{
    __shared__ int64_t wave_sum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int64_t up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
    }
    __syncthreads();                              // (the array may still be read from an earlier call)
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int64_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) { if (w < wave) before += wave_sum[w]; all += wave_sum[w]; }
    *total = all;
    return before + incl - v;
}

__global__ __launch_bounds__(256) void scan_sums_kernel(const int64_t* in, int64_t n, int64_t* sums)
{
    const int64_t i0 = (int64_t)blockIdx.x * SCAN_CHUNK + (int64_t)threadIdx.x * SCAN_ITEMS;
    int64_t v = 0;
    for (int k = 0; k < SCAN_ITEMS; ++k) if (i0 + k < n) v += in[i0 + k];
    int64_t total;
    (void)block_exclusive(v, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// the chunk sums become chunk offsets, in place: one workgroup walks them 256 at a time
__global__ __launch_bounds__(256) void scan_top_kernel(int64_t* sums, int64_t chunks)
{
    int64_t carry = 0;
    for (int64_t c0 = 0; c0 < chunks; c0 += 256) {
        const int64_t c = c0 + threadIdx.x;
        const int64_t v = c < chunks ? sums[c] : 0;
        int64_t total;
        const int64_t ex = block_exclusive(v, &total);
        if (c < chunks) sums[c] = carry + ex;
        carry += total;
    }
}

__global__ __launch_bounds__(256) void scan_apply_kernel(const int64_t* in, int64_t n, const int64_t* sums, int64_t* out)
{
    const int64_t i0 = (int64_t)blockIdx.x * SCAN_CHUNK + (int64_t)threadIdx.x * SCAN_ITEMS;
    int64_t item[SCAN_ITEMS];
    int64_t v = 0;
    for (int k = 0; k < SCAN_ITEMS; ++k) { item[k] = i0 + k < n ? in[i0 + k] : 0; v += item[k]; }
    int64_t total;
    int64_t run = sums[blockIdx.x] + block_exclusive(v, &total);
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (i0 + k < n) out[i0 + k] = run;
        run += item[k];
    }
}

inline size_t scan_chunks(int64_t n) { return (size_t)((n + SCAN_CHUNK - 1) / SCAN_CHUNK); }
// out[i] = in[0] + ... + in[i-1]; sums: scan_chunks(n) words of scratch; in and out may be the same array
inline void exclusive_sum(const int64_t* in, int64_t* out, int64_t n, int64_t* sums, hipStream_t s)
{
    if (n <= 0) return;
    const unsigned chunks = (unsigned)scan_chunks(n);
    hipLaunchKernelGGL(scan_sums_kernel, dim3(chunks), dim3(256), 0, s, in, n, sums);
    hipLaunchKernelGGL(scan_top_kernel, dim3(1), dim3(256), 0, s, sums, (int64_t)chunks);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(chunks), dim3(256), 0, s, in, n, (const int64_t*)sums, out);
}

// One digit of the sort. Workgroup b owns items b * SORT_CHUNK ..; hist[digit * chunks + b] counts its
// items per digit, so that the exclusive sum over the whole table is, for every (digit, workgroup), where
// that workgroup's first item with that digit goes: all smaller digits first, then the same digit in
// earlier workgroups.
__global__ __launch_bounds__(256) void sort_count_kernel(const uint32_t* keys, int64_t n, int shift, int64_t chunks, int64_t* hist)
{
    __shared__ unsigned cnt[RADIX];
    cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t i0 = (int64_t)blockIdx.x * SORT_CHUNK;
    for (int r = 0; r < SORT_ROUNDS; ++r) {
        const int64_t i = i0 + r * 256 + threadIdx.x;
        if (i < n) atomicAdd(&cnt[(keys[i] >> shift) & (RADIX - 1)], 1u);
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * chunks + blockIdx.x] = cnt[threadIdx.x];
}

// Items leave in their order within the workgroup: 256 at a time, an item's place among the equal
// digits of its round is the number of such items in lower waves plus those in lower lanes of its own.
__global__ __launch_bounds__(256) void sort_move_kernel(const uint32_t* keys, const int32_t* vals, int64_t n, int shift, int64_t chunks,
                                                        const int64_t* offs, uint32_t* keys_out, int32_t* vals_out)
{
    __shared__ int64_t next[RADIX];               // where the workgroup's next item of a digit goes
    __shared__ unsigned in_wave[4][RADIX];        // this round's items per wave and digit
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    next[threadIdx.x] = offs[(int64_t)threadIdx.x * chunks + blockIdx.x];
#pragma unroll
    for (int w = 0; w < 4; ++w) in_wave[w][threadIdx.x] = 0;
    __syncthreads();
    const int64_t i0 = (int64_t)blockIdx.x * SORT_CHUNK;
    for (int r = 0; r < SORT_ROUNDS; ++r) {
        const int64_t i = i0 + r * 256 + threadIdx.x;
        const bool valid = i < n;
        const uint32_t key = valid ? keys[i] : 0u;
        const int32_t val = valid ? vals[i] : 0;
        const uint32_t d = (key >> shift) & (RADIX - 1);
        unsigned long long peers = __ballot(valid);           // the lanes of this wave with the same digit
#pragma unroll
        for (int b = 0; b < RADIX_BITS; ++b) {
            const bool set = ((d >> b) & 1u) != 0;
            const unsigned long long m = __ballot(set);
            peers &= set ? m : ~m;
        }
        const unsigned long long lower = peers & ((1ull << lane) - 1ull);
        if (valid && lower == 0) in_wave[wave][d] = (unsigned)__popcll(peers);
        __syncthreads();
        if (valid) {
            int64_t pos = next[d] + __popcll(lower);
            for (int w = 0; w < wave; ++w) pos += in_wave[w][d];
            keys_out[pos] = key; vals_out[pos] = val;
        }
        __syncthreads();
        unsigned moved = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) { moved += in_wave[w][threadIdx.x]; in_wave[w][threadIdx.x] = 0; }
        next[threadIdx.x] += moved;
        __syncthreads();
    }
}

inline size_t sort_chunks(int64_t n) { return (size_t)((n + SORT_CHUNK - 1) / SORT_CHUNK); }
inline size_t sort_hist_words(int64_t n) { return sort_chunks(n) * RADIX; }
// (keys_out, vals_out) = (keys, vals) in ascending order of the keys' low `bits` bits, equal keys in their
// input order; the inputs are left as they are. tmp_keys / tmp_vals: n words each (used for more than one
// digit); hist: sort_hist_words(n) words; sums: scan_chunks(sort_hist_words(n)) words.
inline void sort_pairs(const uint32_t* keys, const int32_t* vals, uint32_t* keys_out, int32_t* vals_out, int64_t n, int bits,
                       uint32_t* tmp_keys, int32_t* tmp_vals, int64_t* hist, int64_t* sums, hipStream_t s)
{
    if (n <= 0) return;
    const int passes = (bits + RADIX_BITS - 1) / RADIX_BITS;
    const int64_t chunks = (int64_t)sort_chunks(n);
    const uint32_t* src_k = keys;
    const int32_t* src_v = vals;
    for (int k = 0; k < passes; ++k) {
        const bool to_out = ((passes - 1 - k) & 1) == 0;      // the last digit lands in the output arrays
        uint32_t* dst_k = to_out ? keys_out : tmp_keys;
        int32_t* dst_v = to_out ? vals_out : tmp_vals;
        hipLaunchKernelGGL(sort_count_kernel, dim3((unsigned)chunks), dim3(256), 0, s, src_k, n, k * RADIX_BITS, chunks, hist);
        exclusive_sum(hist, hist, chunks * RADIX, sums, s);
        hipLaunchKernelGGL(sort_move_kernel, dim3((unsigned)chunks), dim3(256), 0, s, src_k, src_v, n, k * RADIX_BITS, chunks,
                           (const int64_t*)hist, dst_k, dst_v);
        src_k = dst_k; src_v = dst_v;
    }
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
        GPU_ALLOC(sort_keys, uint32_t, (size_t)n, false);
        GPU_ALLOC(sort_vals, int32_t, (size_t)n, false);
        GPU_ALLOC(sort_hist, int64_t, sort_hist_words(n), false);
        GPU_ALLOC(scan_sums, int64_t, scan_chunks(std::max<int64_t>(n + 1, (int64_t)sort_hist_words(n))), false);
        sort_pairs((const uint32_t*)level, ids, (uint32_t*)sorted_level, order, n, bits, sort_keys, sort_vals, sort_hist, scan_sums, s);
        const int32_t n_ptr = h_max + 2;
        GPU_ALLOC(level_ptr, int64_t, (size_t)n_ptr, false);
        hipLaunchKernelGGL(level_ptr_kernel, dim3(blocks_for(n_ptr)), dim3(256), 0, s, n, sorted_level, n_ptr, level_ptr);

        // cones
        GPU_ALLOC(cnt, int64_t, (size_t)n + 1, true);
        GPU_ALLOC(nbr_ptr, int64_t, (size_t)n + 1, false);
        int64_t nnz = 0;
        int32_t* nbr_idx = nullptr;
        uint8_t* nbr_rel = nullptr;
        if (hops <= 3) {
            GPU_ALLOC(row_id, int32_t, (size_t)n * MAXW, false);
            GPU_ALLOC(row_rel, uint8_t, (size_t)n * MAXW, false);
            hipLaunchKernelGGL(cone_kernel, dim3(nb), dim3(256), 0, s, n, (int)hops, fin, finv, deg, row_id, row_rel, cnt);
            exclusive_sum(cnt, nbr_ptr, n + 1, scan_sums, s);
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
                exclusive_sum(cnt, ptr_cur, n + 1, scan_sums, s);
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
            sort_pairs(pkey, order, pkey_sorted, roots_sorted, n, key_bits, sort_keys, sort_vals, sort_hist, scan_sums, s);
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
            exclusive_sum(cnt, part_ptr, n + 1, scan_sums, s);
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
