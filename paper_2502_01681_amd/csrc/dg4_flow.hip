// The level sweep as one persistent dataflow kernel, for every shape: fp32 with hidden 128 or bf16 with
// hidden 256 (rows of 512 bytes either way), cones of up to three hops (neighbour rows of 8 or 16
// entries) or deeper ones (rows of any width, several lane groups per gate), 1 to 16 stacked layers,
// with or without the feed-forward sub-block.
//
// The updating strategy (paper Section 3.4, Algorithm 2) requires that a gate reads the FINAL
// embeddings of its cone sources and is itself computed once; with several layers a gate runs all
// of them before anything that reads it (level-major). Work is cut into tiles of at most 32 gates
// without dependencies among them, in an order in which every source of a gate sits in an earlier
// tile. Workgroups take tiles from a ticket counter, so a tile is only ever claimed by a workgroup
// that is running, and it waits only for lower-numbered tiles: the wait always ends, however many
// workgroups the device keeps resident. A bounded spin count turns any violation into an abort word
// instead of a hang.
//
// Per tile (eight waves): wait for the "published" flags of the sources of its gates; then per layer
// the attention over the cone rows (16 lanes per gate split the feature dimension; sources are read
// through a structured buffer over the layer's K | V store, so that an entry that is no source costs
// neither a branch nor a request and a lane has 32 row halves in flight; the gate's own rows and its
// neighbour row sit in LDS), the output projection on the matrix cores, residual + LayerNorm, and the
// Q | K | V projection of the new state for the next layer, into LDS; after the last layer the
// embeddings go out and K | V of every layer are projected from them into the store of finished gates. Projections run on blocks of
// 16 gates with the WEIGHT as the A operand of a 16x16 product and the gates as B: a lane ends up
// with 16 contiguous bytes of ONE gate's row, so residual, LayerNorm and the stores need no
// transposition, and a tile of at most 16 gates costs half the matrix-core time of a full one (what
// counts on deep, narrow circuits, where a level is one or two tiles). The packed weights stream
// from the L2 cache through a ring of fragments in registers that is refilled one group of columns
// ahead, across phase boundaries: the first fragments of the next product travel during the
// LayerNorm, those of the next tile's first product during the last stores. A gate's arithmetic does
// not depend on which tile or block it falls into: any schedule gives the same bits.
//
// Visibility between compute units: a K | V row is written exactly once per sweep, with agent-scope
// (write-through) stores, and its flag is raised, again at agent scope, only after the writing
// threads have waited for those stores to complete (s_waitcnt, then a workgroup barrier). The flag
// of a gate counts the layers whose rows are in the store: it goes up once, to the number of layers,
// or (deep, narrow circuits) layer by layer while the later layers are still being projected.
// A reader polls the flag with agent-scope loads, which are served past its own L1 and L2, and
// reads a row only after it has seen the flag cover that row's layer. No row is ever read before it is written, not
// even speculatively, so no cache on the reader's side can hold an older copy of its lines.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dg4_device.h"
#include "dg4_internal.h"
#include "dg4_rowops.h"

namespace {

constexpr int FT = 32;                    // gates per tile (two blocks of 16)
constexpr int FLOW_THREADS = 512;
#ifndef FLOW_RING_DEPTH
#define FLOW_RING_DEPTH 8
#endif

// One fragment of packed weight (16 bytes per lane: 16 output columns x 32 bytes of the input
// dimension) against a block of 16 gates: c[i] of lane (n = lane % 16, g = lane / 16) is gate n,
// output column 4*g + i of the fragment's 16.
template <typename T> struct Blk;
template <> struct Blk<bf16_t> {
    __device__ static __forceinline__ void run(const uint4& w, const uint4& r, f32x4& c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, r), c, 0, 0, 0);
    }
};
template <> struct Blk<float> {
    __device__ static __forceinline__ void run(const uint4& w, const uint4& r, f32x4& c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(w.x), __uint_as_float(r.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(w.y), __uint_as_float(r.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(w.z), __uint_as_float(r.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(w.w), __uint_as_float(r.w), c, 0, 0, 0);
    }
};

// 16 bytes <-> the lane's contiguous columns (4 floats or 8 bfloat16)
template <typename T> struct Piece;
template <> struct Piece<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void unpack(const uint4& v, float* f)
    {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    __device__ static __forceinline__ uint4 pack(const float* f)
    {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};
template <> struct Piece<bf16_t> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void unpack(const uint4& v, float* f)
    {
        const uint32_t w[4] = { v.x, v.y, v.z, v.w };
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = bf16_lo(w[i]); f[2 * i + 1] = bf16_hi(w[i]); }
    }
    __device__ static __forceinline__ uint4 pack(const float* f)
    {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
    }
};

// Weights in the order the kernel streams them, 16-byte units. Columns come in GROUPS of gt tiles of
// 16 (one group = what one wave computes at a time: 16*gt consecutive columns), each tile in 8 steps
// of 32 bytes of the input dimension. Unit (((group*gt + nt)*8 + s)*64 + lane), lane = 16*kq + m,
// holds input rows k = s*4E + kq*E .. +E-1 (E = 16 / sizeof(T)) of column
//   col0 + group*16*gt + (m/4)*4*gt + nt*4 + m%4,
// so that accumulator register i of lane (n, g) of tile nt is column group*16*gt + g*4*gt + nt*4 + i:
// the lane owns 4*gt consecutive columns (16 bytes) of gate n.
template <typename T>
__global__ void pack_wa_kernel(const T* w, int ld, int col0, int n_cols, int gt, T* packed)
{
    constexpr int E = 16 / (int)sizeof(T);
    const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t units = (int64_t)(n_cols / 16) * 8 * 64;
    if (unit >= units) return;
    const int lane = (int)(unit & 63);
    const int s = (int)((unit >> 6) & 7);
    const int tile = (int)(unit >> 9);
    const int nt = tile % gt, group = tile / gt;
    const int m = lane & 15, kq = lane >> 4;
    const int col = col0 + group * 16 * gt + (m >> 2) * 4 * gt + nt * 4 + (m & 3);
    const int k0 = s * 4 * E + kq * E;
#pragma unroll
    for (int j = 0; j < E; ++j) packed[unit * E + j] = w[(int64_t)(k0 + j) * ld + col];
}

// 16 bytes written through to device memory (agent scope) in ONE instruction: the four lanes that
// hold neighbouring columns of a gate then fill whole 64-byte pieces of its row (two 8-byte stores
// per lane left every memory sector half written twice: 2.3 times the bytes on the way to HBM).
// Not tracked by the compiler's wait counting: the kernel waits with vmcnt(0) before it raises flags.
// (The two idle cycles keep the next vector instruction from overwriting the data registers while the
// store still reads them: a hazard the compiler covers for its own wide stores, not inside assembly.)
typedef uint32_t flow_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store16_agent(void* dst, const uint4& v)
{
    const flow_u32x4 t = { v.x, v.y, v.z, v.w };
    __asm__ volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(dst), "v"(t) : "memory");
}

// Global memory -> LDS without passing through registers: every lane moves 16 bytes from its own global
// address to LDS address lds_base + 16 * lane (lds_base wave-uniform). The transfers count in vmcnt like
// loads, but the compiler does not see them: the reader waits with vmcnt(0) itself.
__device__ __forceinline__ void flow_dma16(const void* src, uint32_t lds_base)
{
    __asm__ volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                     : : "v"(src), "s"((uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base)) : "memory", "m0");
}

// x summed over the four 16-lane rows of a wave (lanes with equal lane % 16), in every lane
__device__ __forceinline__ float sum_lane_rows(float x)
{
    const uint32_t u = __float_as_uint(x);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);      // rows (0,1) and (2,3) exchanged
    const uint32_t v = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);      // halves exchanged
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

template <typename T, int AW, bool TIMERS, bool TWO>
__global__ __launch_bounds__(FLOW_THREADS) void flow_kernel(dg4_flow_args p)
{
    constexpr int D = 512 / (int)sizeof(T);       // 128 (fp32) or 256 (bf16): a row is 512 bytes
    constexpr int E = 16 / (int)sizeof(T);
    constexpr int EPL = Elem<T>::EPL, LPR = D / EPL;
    static_assert(LPR == 16 && AW <= LPR, "16 lanes per gate in the attention, one per neighbour entry while waiting");
    // AW == 0: neighbour rows of any width (a multiple of four entries; cones deeper than three hops).
    // Tiles then hold p.tile_rows <= 16 gates and 32 / tile_rows lane groups share a gate's row.
    constexpr bool WIDE = AW == 0;
    constexpr int AWN = WIDE ? 1 : AW;
    constexpr int GT = D / 16 / 8;                // 16-column tiles per group (1 or 2): a wave's share of D columns
    constexpr int CW = 4 * GT;                    // consecutive columns a lane owns (16 bytes)
    static_assert(CW == Piece<T>::N, "a lane's columns are one 16-byte piece");
    constexpr int RING = 8 * GT;                  // fragments of one group
    constexpr int YS = D + E;                     // row stride in LDS (16 bytes of padding)
    constexpr int QS = 3 * D + E;
    constexpr int CPR = D / E;                    // 16-byte pieces per row (32)
    constexpr int PPT = FT * CPR / FLOW_THREADS;  // pieces of the tile's rows per thread (2)
    constexpr int GROUP_UNITS = RING * 64;        // 16-byte units per group in the packed stream

    extern __shared__ __attribute__((aligned(16))) unsigned char flow_smem[];
    constexpr size_t ROW_BUF = (size_t)FT * YS * sizeof(T);
    T* buf0 = (T*)flow_smem;
    T* buf1 = (T*)(flow_smem + ROW_BUF);
    float (*part)[8][FT] = (float (*)[8][FT])(flow_smem + 2 * ROW_BUF);             // [2][wave][row]
    // two tile descriptors {kind, first position, rows, -} (this tile's and the next one's), then the abort word
    int* ctl = (int*)(flow_smem + 2 * ROW_BUF + 2 * 8 * FT * sizeof(float));
    // the packed neighbour rows of this tile's gates and of the next tile's, [2][FT][AW] (read by the 16
    // lanes of a gate's group at the start of every attention: kept in LDS, not in registers)
    constexpr size_t ENT_BYTES = WIDE ? 0 : 2 * (size_t)FT * AWN * sizeof(uint32_t);
    uint32_t (*entbuf)[FT][AWN] = (uint32_t (*)[FT][AWN])(flow_smem + 2 * ROW_BUF + 2 * 8 * FT * sizeof(float) + 64);
    // Q | K | V of the tile's gates at their running state, [FT][QS]: layer 0's come in from the projection
    // of x at the top of a tile, the next layer's are projected here (rows of any width read layer 0's
    // from global memory and have the buffer only in sweeps of several layers)
    T* qkvbuf = (T*)(flow_smem + 2 * ROW_BUF + 2 * 8 * FT * sizeof(float) + 64 + ENT_BYTES);
    const size_t qkv_bytes = (!WIDE || p.n_layers > 1) ? (size_t)FT * QS * sizeof(T) : 0;
    const uint32_t qkv_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)flow_smem +
                             (uint32_t)(2 * ROW_BUF + 2 * 8 * FT * sizeof(float) + 64 + ENT_BYTES);
    // Rows of 16 entries: the attention keeps 128 registers of row halves in flight, so nothing else may
    // stay in registers across it: the weight ring is then filled after the attention, not before it.
    constexpr bool OVER = AW == 8 && TWO;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;       // projection role: gate n of a block, columns wave*16*GT + g*CW .. +CW-1 of a group
    const int cbase = wave * 16 * GT + g * CW;
    const int arow = tid >> 4, sub = tid & 15;    // attention role: gate `arow` of the tile, 32 bytes `sub` of its rows
    const int L = p.n_layers;

    // optional phase timers (thread 0, constant-rate clock, 10 ns ticks, summed over workgroups):
    // ticket, wait, attention, output projection + LayerNorm, next layer's Q|K|V, rows out + K|V, publish
    uint64_t prof[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    uint64_t tick = 0;
    if (TIMERS && tid == 0) tick = wall_clock64();
    auto lap = [&](int phase) __attribute__((always_inline)) {
        if (TIMERS && tid == 0) { const uint64_t now = wall_clock64(); prof[phase] += now - tick; tick = now; }
    };

    // The ring: the next eight fragments of the packed weight stream this wave multiplies, refilled
    // eight fragments ahead as they are used up, across the end of a group into the group that follows.
    // (TWO = false: every tile of the launch is a single block of at most 16 gates, as on narrow circuits and for
    // rows of any width; the registers of the second block's operands then go to a ring twice as deep)
    constexpr int RD_WANT = TWO ? FLOW_RING_DEPTH : 2 * FLOW_RING_DEPTH;
    constexpr int RD = RD_WANT < RING ? RD_WANT : RING;                      // fragments in flight per wave
    uint4 ring[RD];
    const uint4* ring_src;                        // the group whose first fragments the ring holds
    auto group_ptr = [&](const void* packed, int group) __attribute__((always_inline)) {
        return (const uint4*)packed + (int64_t)group * GROUP_UNITS + lane;
    };
    auto fill_ring = [&](const uint4* src) __attribute__((always_inline)) {
        ring_src = src;
#pragma unroll
        for (int f = 0; f < RD; ++f) ring[f] = src[f * 64];
    };
    // acc[block][tile] = (the group in the ring) x b; `next`: the group that follows it
    // (`refill` false: nothing follows that may be requested yet, the ring is left empty)
    auto run_group = [&](const uint4 (&b)[2][8], bool two, const uint4* next, f32x4 (&acc)[2][GT], bool add = false,
                         bool refill = true) __attribute__((always_inline)) {
        const uint4* cur = ring_src;
        if (!add) {
#pragma unroll
            for (int nt = 0; nt < GT; ++nt) {
                acc[0][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
                acc[1][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
            }
        }
#pragma unroll
        for (int f = 0; f < RING; ++f) {
            const int nt = f / 8, s = f % 8;
            const uint4 frag = ring[f % RD];
            Blk<T>::run(frag, b[0][s], acc[0][nt]);
            if (two) Blk<T>::run(frag, b[1][s], acc[1][nt]);
            if (f + RD < RING) ring[f % RD] = cur[(f + RD) * 64];
            else if (refill) ring[f % RD] = next[(f + RD - RING) * 64];
        }
        ring_src = next;
    };
    // the B operands: this lane's 16 bytes per step of the rows of both blocks (the second block's
    // are read, and never used, when the tile has no second block)
    auto load_rows = [&](const T* buf, uint4 (&b)[2][8], int stride = (512 + 16) / (int)sizeof(T)) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            b[0][s] = *(const uint4*)((const unsigned char*)buf + (size_t)n * (stride * sizeof(T)) + s * 64 + g * 16);
            b[1][s] = *(const uint4*)((const unsigned char*)buf + (size_t)(16 + n) * (stride * sizeof(T)) + s * 64 + g * 16);
        }
    };
    // LayerNorm over each gate's row (no affine, biased variance), two passes: the lane's columns, the
    // wave's 16*GT columns across its four lane rows, the eight waves through LDS; then the rows go,
    // rounded to T, to dst. Barriers inside: every wave has read what it needed of dst before.
    auto normalise_to = [&](float (&tv)[2][CW], bool two, bool norm, T* dst) __attribute__((always_inline)) {
        __syncthreads();                          // every wave holds its operands: dst may be written
        if (norm) {
            float mean[2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                float s1 = 0.f;
#pragma unroll
                for (int i = 0; i < CW; ++i) s1 += tv[nb][i];
                s1 = sum_lane_rows(s1);
                if (g == 0) part[0][wave][16 * nb + n] = s1;
            }
            __syncthreads();
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                float a1 = 0.f;
#pragma unroll
                for (int w2 = 0; w2 < 8; ++w2) a1 += part[0][w2][16 * nb + n];
                mean[nb] = a1 * (1.0f / D);
                float s2 = 0.f;
#pragma unroll
                for (int i = 0; i < CW; ++i) { const float d2 = tv[nb][i] - mean[nb]; s2 = fmaf(d2, d2, s2); }
                s2 = sum_lane_rows(s2);
                if (g == 0) part[1][wave][16 * nb + n] = s2;
            }
            __syncthreads();
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                float a2 = 0.f;
#pragma unroll
                for (int w2 = 0; w2 < 8; ++w2) a2 += part[1][w2][16 * nb + n];
                const float rstd = rsqrtf(a2 * (1.0f / D) + p.ln_eps);
#pragma unroll
                for (int i = 0; i < CW; ++i) tv[nb][i] = (tv[nb][i] - mean[nb]) * rstd;
            }
        }
        *(uint4*)&dst[n * YS + cbase] = Piece<T>::pack(tv[0]);
        if (two) *(uint4*)&dst[(16 + n) * YS + cbase] = Piece<T>::pack(tv[1]);
        __syncthreads();                          // dst complete
    };
    // the lane's CW values of group-local columns from an accumulator
    auto cols_of = [&](const f32x4 (&a)[GT], float* t) __attribute__((always_inline)) {
#pragma unroll
        for (int nt = 0; nt < GT; ++nt)
#pragma unroll
            for (int i = 0; i < 4; ++i) t[nt * 4 + i] = a[nt][i];
    };

    // Tickets, by thread 0. Tickets below n_pre stand for the gates finished before this call (a
    // resumed sweep), 32 positions each (16 in launches whose tiles hold one block): nothing is computed for them but K | V of every layer, from
    // the caller's embeddings, with the arithmetic of a gate computed here. The ticket of the next
    // tile is drawn at the top of a tile and its descriptor lands in LDS in the middle of it.
    const int64_t total = p.n_pre + p.n_tiles;
    auto describe = [&](int64_t t, int slot) __attribute__((always_inline)) {      // kind: 0 no tile left, 1 tile, 2 finished gates, 3 empty
        int kind = 0, p0 = 0, rows = 0;
        if (t < p.n_pre) {
            constexpr int PRE = TWO ? FT : 16;      // positions per ticket: what a tile of this launch can hold
            kind = 2; p0 = (int)(t * PRE); rows = (int)(p.pre_rows - p0 < PRE ? p.pre_rows - p0 : PRE);
        } else if (t < total) {
            if (p.pairs) {
                const uint2 ta = p.tiles[p.tile_begin + 2 * (t - p.n_pre)], tb = p.tiles[p.tile_begin + 2 * (t - p.n_pre) + 1];
                p0 = (int)ta.x; rows = (int)(ta.y + tb.y);
            } else {
                const uint2 ta = p.tiles[p.tile_begin + (t - p.n_pre)];
                p0 = (int)ta.x; rows = (int)ta.y;
            }
            kind = rows > 0 ? 1 : 3;
        }
        ctl[4 * slot] = kind; ctl[4 * slot + 1] = p0; ctl[4 * slot + 2] = rows;
    };
    if (tid == 0) {
        ctl[8] = 0;
        describe((int64_t)__hip_atomic_fetch_add(&p.ctrl[2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), 0);
    }
    if (OVER) fill_ring(group_ptr(p.wo_packed, wave));    // layer 0's output projection, this wave's columns
    bool have_next = false;                       // entbuf[it & 1] holds the rows of this tile already (workgroup-uniform)
    for (int it = 0;; ++it) {
        __syncthreads();                          // the descriptor; the previous tile is done with every buffer
        const int kind = ctl[4 * (it & 1)];
        if (kind == 0 || ctl[8]) break;
        const int64_t p0 = ctl[4 * (it & 1) + 1];
        const int rows = ctl[4 * (it & 1) + 2];
        const bool pre = kind == 2;
        // the next tile's ticket travels during this tile
        int64_t t_next = 0;
        if (tid == 0) t_next = (int64_t)__hip_atomic_fetch_add(&p.ctrl[2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (kind != 1) {
            if (tid == 0) describe(t_next, (it + 1) & 1);
            have_next = false;
            if (kind == 3) continue;              // an empty tile of the table
        }
        const bool two = TWO && rows > 16;        // a second block of 16 gates
        const int live = two ? FT : 16;           // rows that are computed (past `rows`: the last gate again, never stored)
        auto pos_of = [&](int r) { return p0 + (r < rows ? r : rows - 1); };
        lap(0);

        T* resid = buf0;                          // the running state s_l
        T* ybuf = buf1;                           // attention output, then the normalised rows

        // s_0 = X rows of the tile's gates, as 16-byte pieces
#pragma unroll
        for (int q = 0; q < PPT; ++q) {
            const int piece = tid + FLOW_THREADS * q, row = piece / CPR, c = piece % CPR;
            if (row < live) {
                const int64_t id = p.order[pos_of(row)];
                if (pre) *(uint4*)&ybuf[row * YS + c * E] = *((const uint4*)((const T*)p.h_out + id * D) + c);
                else *(uint4*)&resid[row * YS + c * E] = *((const uint4*)((const T*)p.x + id * D) + c);
            }
        }

        // ---- the sources of the tile's gates must be published
        const bool attends = arow < live && !pre; // (whole waves: 4 gates per wave)
        const int64_t apos = pos_of(arow);
        if constexpr (!WIDE) {
            // Q | K | V of layer 0 for this wave's four gates, straight into LDS (96 pieces of 16 bytes a row)
            if (!pre) {
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int r = 4 * wave + gq;
                    if (r >= live) break;
                    const unsigned char* src = (const unsigned char*)((const T*)p.qkv_self + pos_of(r) * (3 * D)) + lane * 16;
                    const uint32_t dst = qkv_lds + (uint32_t)(r * QS * sizeof(T));
                    flow_dma16(src, dst);
                    if (lane < 32) flow_dma16(src + 1024, dst + 1024u);
                }
            }
        }
        auto give_up = [&](uint32_t spins) __attribute__((always_inline)) -> bool {
            if (spins > p.spin_limit ||
                ((spins & 63u) == 0 && __hip_atomic_load(&p.ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                // the tile is computed from whatever is there (every access stays in bounds),
                // nothing of it is published, and the workgroup leaves after it
                if (lane == 0) {
                    __hip_atomic_store(&p.ctrl[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ctl[8] = 1;
                }
                return true;
            }
            return false;
        };
        // A flag counts the layers whose K | V of its gate are in the store (all of them at once, or one
        // by one: see the end of the tile). The lanes of a wave wait until every source they watch shows
        // at least `need`; the result is the smallest count seen, at most the number of layers: what the
        // wave need not ask about again.
        auto await = [&](uint32_t e, int need) __attribute__((always_inline)) -> int {
            const bool watch = e != DG4_ELL_PAD && (e >> 30) != 0;
            const uint32_t* f = p.flags + (watch ? (e & 0x3FFFFFFFu) : 0u);
            uint32_t spins = 0, seen;
            for (;;) {
                seen = watch ? __hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0xFFFFFFFFu;
                if (__ballot(seen < (uint32_t)need) == 0) break;
                __builtin_amdgcn_s_sleep(1);
                if (give_up(++spins)) break;
            }
            // (the flag loads above are the only ordering needed, see the head of the file; the fence
            // keeps the compiler from moving row loads above them)
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            int known = need;
            while (known < L && __ballot(seen < (uint32_t)(known + 1)) == 0) ++known;
            return known;
        };
        int have = L;                             // (this wave's sources; only rows of at most 16 entries are followed layer by layer)
        if constexpr (WIDE) {
            // 512 / tile_rows lanes per gate, each watching every (512 / tile_rows)-th entry of its row
            const int LR = FLOW_THREADS / p.tile_rows;
            const int wrow = tid / LR, wl = tid % LR;
            const bool act = !pre && wrow < rows;
            const uint32_t* erow = p.ell + (p0 + (act ? wrow : 0)) * (int64_t)p.ell_w;
            uint32_t spins = 0;
            for (;;) {
                bool ok = true;
                if (act)
                    for (int i = wl; i < p.ell_w; i += LR) {
                        const uint32_t e = erow[i];
                        if (e != DG4_ELL_PAD && (e >> 30) != 0 &&
                            __hip_atomic_load(p.flags + (e & 0x3FFFFFFFu), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) ok = false;
                    }
                if (__ballot(!ok) == 0) break;
                __builtin_amdgcn_s_sleep(1);
                if (give_up(++spins)) break;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __syncthreads();                      // a gate's entries were watched by several waves
        } else if (attends) {
            // lane `sub` of a gate's lane group watches entry `sub` of its row (the row came in during
            // the previous tile, or is fetched now; the 16 lanes of a gate sit in one wave)
            if (!have_next && sub < AWN) entbuf[it & 1][arow][sub] = p.ell[apos * AWN + sub];
            const uint32_t e = sub < AWN ? entbuf[it & 1][arow][sub] : DG4_ELL_PAD;
            have = await(e, 1);
        }
        if (TIMERS) __syncthreads();
        lap(1);

        uint4 b[2][8];
        f32x4 acc[2][GT];
        if (pre) {
            fill_ring(group_ptr(p.wkv_packed, wave));     // (the ring held the first product of a tile that is computed)
            __syncthreads();
            load_rows(ybuf, b);
        }
        for (int l = 0; l < (pre ? 0 : L); ++l) {
            const bool last = l == L - 1;
            // ---- attention of layer l: the gate's own Q, K, V from the projection of x (layer 0) or
            // from LDS (its running state, projected at the end of the previous layer); sources from
            // the store of finished gates, layer l
            if constexpr (WIDE) {
                // S = 32 / tile_rows lane groups share a gate: group `part` walks the chunks of eight
                // entries part, part + S, ... with a running maximum, denominator and weighted sum
                // (the softmax is unchanged by the rescaling); the S partial results are merged
                // through LDS by the first group, always in the same order.
                const int S = FLOW_THREADS / 16 / p.tile_rows;
                const int grp = tid >> 4, r = grp / S, part = grp % S;
                const bool act = r < rows;
                const int64_t eoff = (int64_t)sub * EPL;
                float m = -INFINITY, z = 0.f;
                float av[EPL];
#pragma unroll
                for (int i = 0; i < EPL; ++i) av[i] = 0.f;
                if (act) {
                    // sources through the structured buffer of layer l's K | V store: an entry that is no
                    // source (the gate itself, padding) asks for the row past its end and gets zeros
                    // without a request, so the sixteen requests of a chunk go out back to back
                    const uint32_t kv_rows = (uint32_t)(p.kv_layer_stride / (2 * D));
                    const dg4_i32x4 kvb = row_buffer((const T*)p.kv + (int64_t)l * p.kv_layer_stride, 2 * D * sizeof(T), kv_rows);
                    const T* qrow = l == 0 ? (const T*)p.qkv_self + (p0 + r) * (3 * D) : qkvbuf + r * QS;
                    const uint4 qa = ((const uint4*)(qrow + eoff))[0], qb = ((const uint4*)(qrow + eoff))[1];
                    const float* bp = p.rel_bias + l * (D / 32) * 4 + (int)(eoff >> 5) * 4;
                    const float bias[4] = { bp[0], bp[1], bp[2], bp[3] };
                    const float scale = 0.17677669529663687f;     // 1/sqrt(32)
                    const uint32_t* erow = p.ell + (p0 + r) * (int64_t)p.ell_w;
                    for (int c0 = part * 8; c0 < p.ell_w; c0 += S * 8) {
                        uint32_t en[8];
                        {
                            const uint4 e0 = *(const uint4*)(erow + c0);
                            const uint4 e1 = c0 + 4 < p.ell_w ? *(const uint4*)(erow + c0 + 4)
                                                              : make_uint4(DG4_ELL_PAD, DG4_ELL_PAD, DG4_ELL_PAD, DG4_ELL_PAD);
                            en[0] = e0.x; en[1] = e0.y; en[2] = e0.z; en[3] = e0.w; en[4] = e1.x; en[5] = e1.y; en[6] = e1.z; en[7] = e1.w;
                        }
                        if (en[0] == DG4_ELL_PAD) break;          // rows are padded at the end only
                        uint4 ka[8], kb[8], va[8], vb[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const bool src = en[j] != DG4_ELL_PAD && (en[j] >> 30) != 0;
                            const uint32_t row = src ? (en[j] & 0x3FFFFFFFu) : kv_rows;
                            ka[j] = row_load16(kvb, row, (uint32_t)sub * 32u);
                            kb[j] = row_load16(kvb, row, (uint32_t)sub * 32u + 16u);
                        }
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const bool src = en[j] != DG4_ELL_PAD && (en[j] >> 30) != 0;
                            const uint32_t row = src ? (en[j] & 0x3FFFFFFFu) : kv_rows;
                            va[j] = row_load16(kvb, row, (uint32_t)(D * sizeof(T)) + (uint32_t)sub * 32u);
                            vb[j] = row_load16(kvb, row, (uint32_t)(D * sizeof(T)) + (uint32_t)sub * 32u + 16u);
                        }
                        float sc[8];
                        float cm = m;
                        bool self_here = false;                   // the chunk holds the gate's own entry (same for its 16 lanes)
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const float dot = Elem<T>::head_sum(Elem<T>::dot(qa, qb, ka[j], kb[j]));
                            const uint32_t rel = en[j] >> 30;
                            const float bb = rel == 1 ? bias[1] : rel == 2 ? bias[2] : bias[3];
                            const bool src = en[j] != DG4_ELL_PAD && rel != 0;
                            self_here = self_here || rel == 0;
                            sc[j] = src ? fmaf(dot, scale, bb) : -INFINITY;
                            cm = fmaxf(cm, sc[j]);
                        }
                        float s_self = -INFINITY;
                        float vs[EPL];
                        if (self_here) {                          // its K and V come from the gate's own projection
                            const uint4* kp = (const uint4*)(qrow + D + eoff);
                            const uint4* vp = (const uint4*)(qrow + 2 * D + eoff);
                            s_self = fmaf(Elem<T>::head_sum(Elem<T>::dot(qa, qb, kp[0], kp[1])), scale, bias[0]);
                            Elem<T>::unpack(vp[0], vp[1], vs);
                            cm = fmaxf(cm, s_self);
                        }
                        // (a chunk holds at least one entry, a source or the gate itself: cm is finite)
                        const float corr = __expf(m - cm);        // 0 if these are the first terms (m = -inf)
                        z *= corr;
#pragma unroll
                        for (int i = 0; i < EPL; ++i) av[i] *= corr;
                        if (self_here) {
                            const float ps = __expf(s_self - cm);
                            z += ps;
#pragma unroll
                            for (int i = 0; i < EPL; ++i) av[i] = fmaf(ps, vs[i], av[i]);
                        }
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            float v[EPL];
                            Elem<T>::unpack(va[j], vb[j], v);
                            const float pj = __expf(sc[j] - cm);  // 0 for what is no source
                            z += pj;
#pragma unroll
                            for (int i = 0; i < EPL; ++i) av[i] = fmaf(pj, v[i], av[i]);
                        }
                        m = cm;
                    }
                }
                float* mrg = (float*)((unsigned char*)qkvbuf + qkv_bytes);        // [EPL + 2][512]
                mrg[EPL * FLOW_THREADS + tid] = m;
                mrg[(EPL + 1) * FLOW_THREADS + tid] = z;
#pragma unroll
                for (int i = 0; i < EPL; ++i) mrg[i * FLOW_THREADS + tid] = av[i];
                __syncthreads();
                if (act && part == 0) {
                    // (this group holds the row's first chunk, so its maximum is finite)
                    float mm = m;
                    for (int s2 = 1; s2 < S; ++s2) mm = fmaxf(mm, mrg[EPL * FLOW_THREADS + tid + 16 * s2]);
                    const float c0f = __expf(m - mm);
                    z *= c0f;
#pragma unroll
                    for (int i = 0; i < EPL; ++i) av[i] *= c0f;
                    for (int s2 = 1; s2 < S; ++s2) {
                        const int t2 = tid + 16 * s2;
                        const float cs = __expf(mrg[EPL * FLOW_THREADS + t2] - mm);   // 0 for a part that saw no entry
                        z = fmaf(mrg[(EPL + 1) * FLOW_THREADS + t2], cs, z);
#pragma unroll
                        for (int i = 0; i < EPL; ++i) av[i] = fmaf(mrg[i * FLOW_THREADS + t2], cs, av[i]);
                    }
                    const float rz = 1.0f / z;
#pragma unroll
                    for (int i = 0; i < EPL; ++i) av[i] *= rz;
                    uint4 oa, ob;
                    Elem<T>::pack(av, oa, ob);
                    uint4* op = (uint4*)&ybuf[r * YS + sub * EPL];
                    op[0] = oa; op[1] = ob;
                }
            } else if (attends) {
                // the sources' K | V of this layer (published layer by layer on deep, narrow circuits)
                if (have < l + 1) have = await(sub < AWN ? entbuf[it & 1][arow][sub] : DG4_ELL_PAD, l + 1);
                const T* kvl = (const T*)p.kv + (int64_t)l * p.kv_layer_stride;
                const T* qrow = qkvbuf + arow * QS;
                if (l == 0) {                     // this wave's transfers of the gates' own rows have landed
                    __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
                    __asm__ volatile("" ::: "memory");
                }
                float av[EPL];
                uint32_t ent[AWN];
                {
                    const uint4* ep = (const uint4*)&entbuf[it & 1][arow][0];
#pragma unroll
                    for (int i = 0; i < AWN / 4; ++i) {
                        const uint4 t4 = ep[i];
                        ent[4 * i] = t4.x; ent[4 * i + 1] = t4.y; ent[4 * i + 2] = t4.z; ent[4 * i + 3] = t4.w;
                    }
                }
                const uint32_t kv_rows = (uint32_t)(p.kv_layer_stride / (2 * D));
                // (rows of eight entries: one trip to memory either way, and the plain two-pass form has the
                // shorter chain of arithmetic, which is what deep, narrow circuits wait for)
                if constexpr (AWN == 8)
                    attend_core<T, D, AWN, AWN, true>(ent, qrow, qrow + D, qrow + 2 * D, kvl, kvl + D, 2 * D,
                                                      p.rel_bias + l * (D / 32) * 4, sub, av);
                else
                attend_chunked<T, D, AWN>(ent, qrow, qrow + D, qrow + 2 * D, row_buffer(kvl, 2 * D * sizeof(T), kv_rows), kv_rows,
                                          p.rel_bias + l * (D / 32) * 4, sub, av);
                uint4 oa, ob;
                Elem<T>::pack(av, oa, ob);
                uint4* op = (uint4*)&ybuf[arow * YS + sub * EPL];
                op[0] = oa; op[1] = ob;
            }
            __syncthreads();
            lap(2);
            // ---- s_{l+1} = LN(s_l + a Wo_l): this lane ends with columns cbase .. cbase+CW-1 of gates n and 16+n
            if (!OVER) fill_ring(group_ptr((const char*)p.wo_packed + (int64_t)l * p.w_layer_stride, wave));
            load_rows(ybuf, b);
            // (the ring then takes the first group of the product that follows the LayerNorm)
            const void* after = last ? p.wkv_packed : (const void*)((const char*)p.wqkv_packed + (int64_t)(l + 1) * p.w_layer_stride);
            const void* w1l = (const char*)p.w1_packed + (int64_t)l * p.ffn_layer_stride;
            const void* w2l = (const char*)p.w2_packed + (int64_t)l * p.ffn_layer_stride;
            run_group(b, two, p.ffn ? group_ptr(w1l, wave) : group_ptr(after, wave), acc);
            if (l == 0 && tid == 0) describe(t_next, (it + 1) & 1);       // (the ticket has had the attention to arrive)
            float tv[2][CW];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                cols_of(acc[nb], tv[nb]);
                if (p.epilogue && (nb == 0 || two)) {
                    float r[CW];
                    Piece<T>::unpack(*(const uint4*)&resid[(16 * nb + n) * YS + cbase], r);
#pragma unroll
                    for (int i = 0; i < CW; ++i) tv[nb][i] += r[i];
                }
            }
            normalise_to(tv, two, p.epilogue != 0, ybuf);         // ybuf = LN(s_l + a Wo_l), rounded to T (and the next tile's descriptor is in LDS)
            if (p.ffn) {
                // ---- the feed-forward sub-block (Section 3.5 keeps the transformer structure around the
                // attention): s_{l+1} = LN(h + max(h W1, 0) W2), h = ybuf. The 4D activations of the
                // tile go to LDS rounded to T (slab `sl` of D hidden units: this wave's columns of it),
                // the second product runs over them in four steps of D, accumulating.
                constexpr int US = 4 * D + E;
                T* ubuf = (T*)((unsigned char*)qkvbuf + qkv_bytes);
                load_rows(ybuf, b);
#pragma unroll 1
                for (int sl = 0; sl < 4; ++sl) {
                    run_group(b, two, sl < 3 ? group_ptr(w1l, 8 * (sl + 1) + wave) : group_ptr(w2l, wave), acc);
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb) {
                        if (nb == 1 && !two) continue;
                        float v[CW];
                        cols_of(acc[nb], v);
#pragma unroll
                        for (int i = 0; i < CW; ++i) v[i] = fmaxf(v[i], 0.f);
                        *(uint4*)&ubuf[(16 * nb + n) * US + sl * D + cbase] = Piece<T>::pack(v);
                    }
                }
                __syncthreads();                  // the activations of every wave
#pragma unroll 1
                for (int c4 = 0; c4 < 4; ++c4) {
                    load_rows(ubuf + c4 * D, b, US);
                    run_group(b, two, c4 < 3 ? group_ptr(w2l, 8 * (c4 + 1) + wave) : group_ptr(after, wave), acc, c4 > 0);
                }
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) {
                    cols_of(acc[nb], tv[nb]);
                    if (nb == 0 || two) {
                        float r[CW];
                        Piece<T>::unpack(*(const uint4*)&ybuf[(16 * nb + n) * YS + cbase], r);
#pragma unroll
                        for (int i = 0; i < CW; ++i) tv[nb][i] += r[i];
                    }
                }
                normalise_to(tv, two, true, ybuf);
                lap(7);
            }
            lap(3);
            load_rows(ybuf, b);
            if (l == 0 && !WIDE) {
                // the neighbour row this lane group will need at the top of the next tile
                const int nslot = 4 * ((it + 1) & 1);
                have_next = ctl[nslot] == 1;
                if (have_next) {
                    const int nrows = ctl[nslot + 2];
                    if (arow < (nrows > 16 ? FT : 16) && sub < AWN) {
                        const int64_t npos = (int64_t)ctl[nslot + 1] + (arow < nrows ? arow : nrows - 1);
                        entbuf[(it + 1) & 1][arow][sub] = p.ell[npos * AWN + sub];
                    }
                }
            }

            if (!last) {
                // ---- Q | K | V of the new state for the next layer, into LDS: groups wave, 8 + wave, 16 + wave
                // of the 3D columns are this wave's columns of Q, of K and of V
                const void* wq = (const char*)p.wqkv_packed + (int64_t)(l + 1) * p.w_layer_stride;
                const void* wo_next = (const char*)p.wo_packed + (int64_t)(l + 1) * p.w_layer_stride;
#pragma unroll
                for (int part3 = 0; part3 < 3; ++part3) {
                    run_group(b, two, part3 < 2 ? group_ptr(wq, 8 * (part3 + 1) + wave) : group_ptr(wo_next, wave), acc, false,
                              OVER || part3 < 2);
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb) {
                        if (nb == 1 && !two) continue;
                        float v[CW];
                        cols_of(acc[nb], v);
                        *(uint4*)&qkvbuf[(16 * nb + n) * QS + part3 * D + cbase] = Piece<T>::pack(v);
                    }
                }
                // the new state is the next layer's residual; the old one's space takes the next attention output
                T* tmp = resid; resid = ybuf; ybuf = tmp;
                __syncthreads();
                lap(4);
                continue;
            }
        }
        // ---- the embeddings of the tile's gates go out, by node id
#pragma unroll
        for (int q = 0; q < PPT; ++q) {
            const int piece = tid + FLOW_THREADS * q, row = piece / CPR, c = piece % CPR;
            if (row >= rows || pre) continue;
            *((uint4*)((T*)p.h_out + (int64_t)p.order[p0 + row] * D) + c) = *(const uint4*)&ybuf[row * YS + c * E];
        }
        // ---- K | V of every layer from the final embeddings: per layer, groups wave (K) and 8 + wave (V)
        // of its 2D columns; written through to device memory (agent scope), 16 bytes per lane
        for (int j = 0; j < 2 * L; ++j) {
            const int nj = j + 1;
            const uint4* next = nj < 2 * L ? group_ptr(p.wkv_packed, (nj >> 1) * 16 + (nj & 1) * 8 + wave)
                                           : group_ptr(p.wo_packed, wave);      // the next tile's first product
            run_group(b, two, next, acc, false, OVER || nj < 2 * L);
            T* base = (T*)p.kv + (int64_t)(j >> 1) * p.kv_layer_stride + (j & 1) * D + cbase;
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const int row = 16 * nb + n;
                if (row >= rows) continue;
                float v[CW];
                cols_of(acc[nb], v);
                store16_agent(base + (p0 + row) * (2 * D), Piece<T>::pack(v));
            }
            // Layer by layer (deep, narrow circuits with several layers: a reader can run its first layers while
            // this tile still projects K | V for the later ones): once K of layer j/2 has been issued, V of the
            // layer before is a whole group behind. Loads and stores of a wave complete in order, and since
            // those V stores the wave has issued this group's RING fragment loads and at least one store: with
            // at most RING operations outstanding they are written through.
            if (p.layer_flags && (j & 1) == 0 && j >= 2) {
                __builtin_amdgcn_s_waitcnt(RING == 16 ? 0x4F70 : 0x0F78);        // vmcnt(16) / vmcnt(8)
                __asm__ volatile("" ::: "memory");
                __syncthreads();
                if (!ctl[8] && tid < rows)
                    __hip_atomic_store(&p.flags[p0 + tid], (uint32_t)(j >> 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        lap(5);
        // ---- publish: every thread's row stores have completed (the ring's loads with them) before the flags go up
        __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
        __asm__ volatile("" ::: "memory");
        __syncthreads();
        if (ctl[8]) break;                        // an aborted tile publishes nothing
        if (tid < rows) __hip_atomic_store(&p.flags[p0 + tid], (uint32_t)L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lap(6);
    }
    if (TIMERS && tid == 0)
        for (int i = 0; i < 8; ++i) atomicAdd((unsigned long long*)&p.prof[i], (unsigned long long)prof[i]);
}

template <typename T>
int launch_flow_t(const dg4_flow_args& a, hipStream_t s)
{
    constexpr int D = 512 / (int)sizeof(T), E = 16 / (int)sizeof(T);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return hipErrorInvalidDevice;
    const bool wide = a.ell_w > 16;
    const size_t smem = 2 * (size_t)FT * (D + E) * sizeof(T) + 2 * 8 * FT * sizeof(float) + 64 +
                        (wide ? 0 : 2 * (size_t)FT * a.ell_w * sizeof(uint32_t)) +
                        (a.n_layers > 1 || !wide ? (size_t)FT * (3 * D + E) * sizeof(T) : 0) +
                        (wide ? (size_t)(Elem<T>::EPL + 2) * FLOW_THREADS * sizeof(float) : 0) +
                        (a.ffn ? (size_t)FT * (4 * D + E) * sizeof(T) : 0);
    if (a.ffn && (wide || !a.w1_packed || !a.w2_packed)) return hipErrorInvalidValue;
    void (*kern)(dg4_flow_args) = nullptr;
    // tiles of 32 gates: whole sweeps that take the pair table two tiles at a time, and sweeps over a range of levels
    if (a.tile_cap != 16 && a.tile_cap != 32) return hipErrorInvalidValue;
    const bool two = a.tile_cap == 32;
    if (wide && two) return hipErrorInvalidValue;
    if (a.ell_w == 8) kern = two ? (a.prof ? flow_kernel<T, 8, true, true> : flow_kernel<T, 8, false, true>)
                                 : (a.prof ? flow_kernel<T, 8, true, false> : flow_kernel<T, 8, false, false>);
    else if (a.ell_w == 16) kern = two ? (a.prof ? flow_kernel<T, 16, true, true> : flow_kernel<T, 16, false, true>)
                                       : (a.prof ? flow_kernel<T, 16, true, false> : flow_kernel<T, 16, false, false>);
    else if (wide && a.ell_w % 4 == 0 && !a.pairs && (a.tile_rows == 2 || a.tile_rows == 4 || a.tile_rows == 8 || a.tile_rows == 16))
        kern = a.prof ? flow_kernel<T, 0, true, false> : flow_kernel<T, 0, false, false>;
    if (!kern) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    // one workgroup of eight waves per compute unit (tiles are handed out by tickets, so fewer
    // resident ones would only cost speed)
    // (with fewer XCDs at work the whole grid is still launched: the idle workgroups leave at once)
    const int64_t grid = std::min<int64_t>((int64_t)cus, a.n_tiles + a.n_pre);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(FLOW_THREADS), smem, s, a);
    return hipGetLastError();
}

}  // namespace

bool dg4_flow_supports(int dtype, int hidden, int ell_w)
{
    return ((dtype == DG4_F32 && hidden == 128) || (dtype == DG4_BF16 && hidden == 256)) &&
           (ell_w == 8 || ell_w == 16 || (ell_w > 16 && ell_w % 4 == 0));
}

// `packed` takes columns [col0, col0 + n_cols) of the row-major weight w (row stride ld, hidden rows)
// in the streaming order of the kernel above; n_cols a multiple of 16 * (hidden / 128)
int dg4_launch_pack_wa(int dtype, int hidden, const void* w, int ld, int col0, int n_cols, void* packed, hipStream_t s)
{
    const int gt = hidden / 16 / 8;
    if (gt < 1 || n_cols % (16 * gt)) return hipErrorInvalidValue;
    const int64_t units = (int64_t)(n_cols / 16) * 8 * 64;
    const unsigned grid = (unsigned)((units + 255) / 256);
    if (dtype == DG4_F32)
        hipLaunchKernelGGL(pack_wa_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)w, ld, col0, n_cols, gt, (float*)packed);
    else
        hipLaunchKernelGGL(pack_wa_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, (const uint16_t*)w, ld, col0, n_cols, gt, (uint16_t*)packed);
    return hipGetLastError();
}

int dg4_launch_flow(int dtype, int hidden, const dg4_flow_args& a, hipStream_t s)
{
    if (a.n_tiles <= 0) return hipSuccess;
    if (!dg4_flow_supports(dtype, hidden, a.ell_w) || a.n_layers < 1 || a.n_pre * a.tile_cap < a.pre_rows) return hipErrorInvalidValue;
    return dtype == DG4_F32 ? launch_flow_t<float>(a, s) : launch_flow_t<bf16_t>(a, s);
}
