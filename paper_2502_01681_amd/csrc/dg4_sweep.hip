// The level sweep as ONE persistent dataflow kernel (bf16, hidden 256, one layer, cones of at most two hops).
//
// The updating strategy (paper Section 3.4, Algorithm 2) orders the work level
// by level; what it requires is that a gate reads the FINAL embeddings of its
// cone sources and is itself computed once. Work is cut into tiles of at most 16
// gates, in an order in which every source of a gate sits in an earlier tile:
// level by level, or (whole-graph sweeps) list-scheduled over the dependencies.
// One workgroup per compute unit; workgroups draw tiles from a ticket counter,
// three tiles ahead of the one they work on (the descriptors of the next two
// travel while a tile is computed). A tile waits only on the "published" flags
// of ITS sources, so many levels are in flight at once while every gate still
// sees exactly the values the level-by-level sweep would give it. A tile waits
// only for lower-numbered tiles; those were drawn earlier, by workgroups that
// are running and that take their own tiles in ascending order, so the wait
// always ends, whether or not every workgroup of the launch is resident. A
// bounded spin count turns any violation into an abort flag instead of a hang.
//
// With the weights resident in registers (Wo in vector registers, Wk|Wv in the
// accumulation registers) there is ONE wave per SIMD: nothing hides latency for
// free, and every instruction costs four cycles of issue. Hence the shape of
// the code: rows travel from global memory straight into LDS (no registers, no
// waits in between), the next tile's sources are requested while this tile's
// attention runs, and the per-row bookkeeping is vectorised across lanes.
//
// Per tile: attention over the cone rows (lanes split the feature dimension,
// scores and softmax in registers), output projection on the matrix cores with
// the tile as the B operand (so a lane ends up owning CONTIGUOUS output columns
// of one gate), residual + LayerNorm in registers, K|V projection of the new
// embeddings, publication of the rows and, once they are written through, of
// the flags.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "dg4_device.h"
#include "dg4_internal.h"

namespace {

typedef __bf16 bf16x8s __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int TILE = DG4_TILE_ROWS;   // 16
constexpr int D = 256;
constexpr int LDS_STRIDE = D + 8;     // bf16 elements per LDS row (16 bytes of padding)
constexpr int KV_STRIDE = 2 * D + 8;
// LDS map (bytes): three row buffers (sKV overlays the first two; the second, spare one also
// holds the flag snapshots and the address scatter of the attention phase), LayerNorm partial
// sums, for this tile and the next two the packed neighbour rows followed by the node ids (one
// contiguous block per tile, filled by a single gather), the abort word, timers, the bias table,
// one Wo fragment per wave, then the landing zone: per gate 8 KB = six source slots of K|V (1 KB
// each), the gate's own K|V as a seventh slot, its own Q row (512 B) and its residual row (512 B).
constexpr int SMEM_TILE = 3 * TILE * LDS_STRIDE * 2;                // sA, sX (spare), sH
static_assert(TILE * KV_STRIDE * 2 <= 2 * TILE * LDS_STRIDE * 2, "sKV must fit over sA and sX");
constexpr int SMEM_LOOK = TILE * LDS_STRIDE * 2;                    // two flag snapshots and the address scatter (1 KB each) in the spare row buffer
constexpr int SMEM_RED = SMEM_TILE;
constexpr int SMEM_DESC = SMEM_RED + TILE * 4 * 2 * 4;              // [3 tiles][ent 16 x 8 words | ids 16 words]
constexpr int DESC_BYTES = TILE * 8 * 4 + TILE * 4;                 // 576
constexpr int SMEM_ABORT = SMEM_DESC + 3 * DESC_BYTES;
constexpr int SMEM_PROF = SMEM_ABORT + 16;
constexpr int SMEM_BIAS = SMEM_PROF + 64;                          // rel_bias [8 heads][4]
constexpr int SMEM_WOF = SMEM_BIAS + 128;                           // one Wo fragment per wave (4 x 1 KB)
constexpr int SMEM_LAND = SMEM_WOF + 4096;
constexpr int LAND_GATE = 8192, LAND_SELF = 6144, LAND_Q = 7168, LAND_X = 7680;
constexpr int SMEM_BYTES = SMEM_LAND + TILE * LAND_GATE;
static_assert(SMEM_BYTES + 512 <= 160 * 1024, "LDS budget");
static_assert(SMEM_LAND % 16 == 0 && SMEM_DESC % 16 == 0 && DESC_BYTES % 16 == 0, "alignment");

typedef __bf16 bf16x2s __attribute__((ext_vector_type(2)));
// sum += a.lo*b.lo + a.hi*b.hi on packed bf16 pairs, fp32 accumulation
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float sum)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2s, a), __builtin_bit_cast(bf16x2s, b), sum, false);
}

__device__ __forceinline__ f32x4 mfma16(const uint4& a, const uint4& b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8s, a), __builtin_bit_cast(bf16x8s, b), c, 0, 0, 0);
}

// Global memory -> LDS without passing through registers: every lane moves 16 bytes from its own
// global address to LDS address lds_base + 16*lane (lds_base wave-uniform). Issued as assembly
// so that the waits stay under this file's control: the compiler would otherwise drain every
// outstanding transfer before ANY later LDS read, whatever its address. The transfers count in
// vmcnt like loads and complete in issue order; a reader waits with s_waitcnt (plus a barrier if
// another wave issued the transfer).
// (the scalar operands go through readfirstlane: the compiler does not do that by itself for a
// value it keeps in a vector register, and folds it away for one it knows to be uniform)
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ const void* uniform_ptr(const void* q)
{
    const uint64_t a = (uint64_t)(uintptr_t)q;
    return (const void*)(uintptr_t)((uint64_t)uniform32((uint32_t)a) | ((uint64_t)uniform32((uint32_t)(a >> 32)) << 32));
}
__device__ __forceinline__ void dma16(const void* src, uint32_t lds_base)
{
    __asm__ volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(uniform32(lds_base)) : "memory", "m0");
}
// same with a wave-uniform 64-bit base and a per-lane 32-bit byte offset
__device__ __forceinline__ void dma16_row(const void* base, uint32_t lane_off, uint32_t lds_base)
{
    __asm__ volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_off), "s"(uniform_ptr(base)), "s"(uniform32(lds_base)) : "memory", "m0");
}
// one 32-bit word per lane, read at device scope (served by the L2, never by this unit's L1)
__device__ __forceinline__ void dma4_fresh(const void* base, uint32_t lane_off, uint32_t lds_base)
{
    __asm__ volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1 sc1" : : "v"(lane_off), "s"(uniform_ptr(base)), "s"(uniform32(lds_base)) : "memory", "m0");
}

// Packed order for weights used as the A operand of a 16x16x32 MFMA, in
// 16-byte units: unit (((wave*NTW + nt)*8 + ks)*64 + lane) holds rows
// k = ks*32 + 8*(lane/16) .. +7 of output column
//   col0 + wave*NTW*16 + (m/4)*NTW*4 + nt*4 + m%4,   m = lane%16.
// With the tile as B operand, accumulator register i of lane (n = lane%16,
// g = lane/16) of tile nt is then gate n, column wave*NTW*16 + g*NTW*4 + nt*4 + i:
// every lane owns NTW*4 contiguous columns of one gate.
__global__ void pack_wt_kernel(const uint16_t* w, int ld, int col0, int ntw, int waves, uint16_t* packed)
{
    const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t units = (int64_t)waves * ntw * 8 * 64;
    if (unit >= units) return;
    const int lane = (int)(unit & 63);
    const int ks = (int)((unit >> 6) & 7);
    const int t = (int)(unit >> 9);              // wave*ntw + nt
    const int nt = t % ntw, wave = t / ntw;
    const int m = lane & 15, g = lane >> 4;
    const int col = col0 + wave * ntw * 16 + (m >> 2) * ntw * 4 + nt * 4 + (m & 3);
    const int k0 = ks * 32 + 8 * g;
#pragma unroll
    for (int j = 0; j < 8; ++j) packed[unit * 8 + j] = w[(int64_t)(k0 + j) * ld + col];
}

// 16 bytes per lane from the lane's own global address, read at device scope (rows this compute
// unit wrote earlier in the kernel: never served from a line its L1 may still hold)
__device__ __forceinline__ void dma16_fresh(const void* src, uint32_t lds_base)
{
    __asm__ volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off sc1" : : "v"(src), "s"(uniform32(lds_base)) : "memory", "m0");
}

// The feed-forward weights in the order the sweep streams them (16-byte units). A tile's
// sub-block runs in FFN_PASSES passes of 256 hidden units; in a pass wave w first forms the
// activations of its 64 hidden units (A operand: a 16 x 32 piece of W1 transposed, hidden unit
// 256*pass + 64*w + 16*ht + m against inputs 32*ks + 8*g .. +7; fragment 16*(ht/2) + 2*ks + ht%2:
// the wave works through its 64 units in two halves of 32), then adds
// the pass's contribution to its 64 output columns (A operand: a piece of W2 transposed, output
// column 64*w + 16*(m/4) + 4*ct + m%4, the same column ownership as the output projection,
// against hidden units 256*pass + 32*kk + 8*g .. +7; fragment 32 + 4*kk + ct). Unit
// (((w*FFN_PASSES + pass)*64 + fragment)*64 + lane), lane = 16*g + m: one contiguous stream per wave.
constexpr int FFN_PASSES = 4;
constexpr int FFN_FRAGS = 64;         // fragments (1 KB each) per wave and pass
__global__ void pack_ffn_kernel(const uint16_t* w1, const uint16_t* w2, uint16_t* packed)
{
    const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (unit >= 4 * FFN_PASSES * FFN_FRAGS * 64) return;
    const int lane = (int)(unit & 63);
    const int j = (int)((unit >> 6) % FFN_FRAGS);
    const int pass = (int)((unit >> 12) % FFN_PASSES);
    const int w = (int)(unit >> 14);
    const int m = lane & 15, g = lane >> 4;
    if (j < 32) {
        const int ks = (j & 15) >> 1, ht = 2 * (j >> 4) + (j & 1);
        const int hidden = 256 * pass + 64 * w + 16 * ht + m;
        const int k0 = 32 * ks + 8 * g;
#pragma unroll
        for (int e = 0; e < 8; ++e) packed[unit * 8 + e] = w1[(int64_t)(k0 + e) * (4 * D) + hidden];
    } else {
        const int kk = (j - 32) >> 2, ct = (j - 32) & 3;
        const int col = 64 * w + 16 * (m >> 2) + 4 * ct + (m & 3);
        const int h0 = 256 * pass + 32 * kk + 8 * g;
#pragma unroll
        for (int e = 0; e < 8; ++e) packed[unit * 8 + e] = w2[(int64_t)(h0 + e) * D + col];
    }
}

// compile-time loop: f(integral_constant<int, I>) for I = 0 .. N-1
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

__global__ void sweep_init_kernel(uint32_t* flags, int64_t n, int64_t done_below, uint32_t* ctrl)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flags[i] = i < done_below ? 1u : 0u;
    if (i < 64) ctrl[i] = 0u;                     // [1] abort flag, [16..31] phase timers
}

// Transfers of slots [S0, S1) of a wave's four gates: lane 8*g + s of (lo, hi) holds the global
// address of the row, land + g*LAND_GATE + s*1024 is where it goes.
template <int S0, int S1>
__device__ __forceinline__ void issue_slots(uint32_t lo, uint32_t hi, uint32_t lane_off, uint32_t land)
{
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int sl = S0; sl < S1; ++sl) {
            const uint64_t a = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)lo, 8 * g + sl) |
                               ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi, 8 * g + sl) << 32);
            dma16_row((const void*)(uintptr_t)a, lane_off, land + (uint32_t)(g * LAND_GATE + sl * 1024));
        }
}

// x summed over the four 16-lane rows of a wave (lanes with equal lane % 16), in every lane:
// two row exchanges on the vector ALU instead of four trips through the LDS crossbar
__device__ __forceinline__ float sum_rows(float x)
{
    const uint32_t u = __float_as_uint(x);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);      // rows (0,1) and (2,3) exchanged
    const uint32_t v = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);      // halves exchanged
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

template <int W, bool TIMERS, bool FFN>
__global__ __launch_bounds__(256, 1) void sweep_kernel(dg4_sweep_args p)
{
    static_assert(W == 8, "the landing zone is laid out for cones of two hops");
    constexpr int NS = W - 2;                 // most sources a gate can have besides itself (6)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t (*sA)[LDS_STRIDE] = (uint16_t (*)[LDS_STRIDE])smem;                     // attention output, bf16
    uint16_t (*sH)[LDS_STRIDE] = sA + 2 * TILE;                                      // new embeddings, bf16
    uint16_t (*sKV)[KV_STRIDE] = (uint16_t (*)[KV_STRIDE])smem;                      // K|V rows on their way out
    float (*sRed)[4][2] = (float (*)[4][2])(smem + SMEM_RED);
    int& sAbort = *(int*)(smem + SMEM_ABORT);
    unsigned char* sLand = smem + SMEM_LAND;
    // LDS byte address of smem[0] for the transfers above
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    // the tile table is read-only for the whole kernel: fetched through the constant address space
    // (wave-uniform index, so the loads are scalar and do not count in vmcnt)
    const __attribute__((address_space(4))) uint64_t* tiles64 = (const __attribute__((address_space(4))) uint64_t*)p.tiles;
    auto tile_at = [&](int64_t i) __attribute__((always_inline)) -> uint2 {
        const uint64_t t = tiles64[p.tile_begin + i];
        return make_uint2((uint32_t)t, (uint32_t)(t >> 32));                          // first position, rows
    };
    // neighbour rows [gate][entry] and node ids [gate] of the tile in descriptor buffer `parity` (0..2)
    auto ent_of = [&](int parity) __attribute__((always_inline)) { return (const uint32_t (*)[8])(smem + SMEM_DESC + parity * DESC_BYTES); };
    auto ids_of = [&](int parity) __attribute__((always_inline)) { return (const int32_t*)(smem + SMEM_DESC + parity * DESC_BYTES + TILE * 8 * 4); };

    const int lane0 = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // wave-uniform, and known to be
    // Everything derived from the lane number (roles, LDS addresses) is recomputed at the start of
    // each phase from a copy the compiler cannot see through. Otherwise dozens of such values are
    // kept in registers across the whole loop, and the weights held there leave no room for that.
    int lane, grp, sub, my, c0;
    uint32_t lane16;
    const float* sBias;
    const uint4* sWoF;
    auto roles = [&]() __attribute__((always_inline)) {
        int t = lane0;
        __asm__ volatile("" : "+v"(t));
        lane = t; grp = t >> 4; sub = t & 15;
        lane16 = (uint32_t)t * 16u;
        my = 4 * wave + grp;              // attention role: this lane holds 16 features of gate `my`
        c0 = 64 * wave + 16 * grp;        // projection role: this lane holds 16 columns of gate `sub`
        sBias = (const float*)(smem + SMEM_BIAS) + (sub >> 1) * 4;          // this lane's head
        sWoF = (const uint4*)(smem + SMEM_WOF) + wave * 64 + lane;
    };
    roles();
    const uint32_t wave_land = lds0 + (uint32_t)(SMEM_LAND + 4 * wave * LAND_GATE);   // landing zone of this wave's gates
    // a ticket for a tile (a pair of tiles with the feed-forward sub-block): one lane only
    auto draw = [&]() __attribute__((always_inline)) -> int {
        const int k = (int)__hip_atomic_fetch_add(&p.ctrl[2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return FFN ? 2 * k : k;
    };
    // the first one now, the next two once the weights are in (the other workgroups start within
    // microseconds of this one, so the draws interleave: first tiles first)
    int first_ticket = 0;
    if (threadIdx.x == 0) first_ticket = draw();

    // The weights of this wave stay in registers for the whole kernel: its 4 column tiles of Wo
    // (128 vector registers) and its 8 column tiles of Wk|Wv (all 256 accumulation registers,
    // which the matrix cores read directly). Everything else below is written to need few
    // registers: every row a tile needs is gathered into LDS, not into registers.
    u32x4 wo_r[4][8];
    u32x4 wkv_r[8][8];
    {
        const uint4* wo = (const uint4*)p.wo_packed + (int64_t)wave * 4 * 8 * 64 + lane;
        const uint4* wkv = (const uint4*)p.wkv_packed + (int64_t)wave * 8 * 8 * 64 + lane;
        // (with the feed-forward sub-block Wo is fetched anew for every tile, at the end of the
        // attention: the sub-block needs the registers; only its last fragment, which sits in LDS, is
        // read here)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                if (!FFN || (nt == 3 && ks == 7)) wo_r[nt][ks] = __builtin_bit_cast(u32x4, wo[(nt * 8 + ks) * 64]);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) wkv_r[nt][ks] = __builtin_bit_cast(u32x4, wkv[(nt * 8 + ks) * 64]);
    }
    // (the last fragment of Wo and the bias table sit in LDS: the register file is full)
    if (threadIdx.x < 32) ((float*)(smem + SMEM_BIAS))[threadIdx.x] = p.rel_bias[threadIdx.x] * 1.4426950408889634f;   // in units of log 2
    ((uint4*)(smem + SMEM_WOF))[wave * 64 + lane] = __builtin_bit_cast(uint4, wo_r[3][7]);
    if (threadIdx.x == 0) sAbort = 0;

    // optional phase timers (thread 0, constant-rate clock): -, wait, attention, Wo, LN, KV, publish
    // (accumulated in LDS so that the timed build needs no more registers than the plain one)
    uint64_t* sProf = (uint64_t*)(smem + SMEM_PROF);
    uint64_t tick = 0;
    if (TIMERS && threadIdx.x == 0) {
        for (int i = 0; i < 8; ++i) sProf[i] = 0;
        tick = wall_clock64();
    }
    auto lap = [&](int phase) __attribute__((always_inline)) {
        if (TIMERS && threadIdx.x == 0) { const uint64_t now = wall_clock64(); sProf[phase] += now - tick; tick = now; }
    };
    auto flush = [&]() __attribute__((always_inline)) {
        if (TIMERS && threadIdx.x == 0)
            for (int i = 0; i < 8; ++i) atomicAdd((unsigned long long*)&p.prof[i], (unsigned long long)sProf[i]);
    };

    // All gathers go straight from global memory into LDS, 16 bytes per lane, no registers.
    // (1) what describes a tile: the packed neighbour rows of its 16 positions (512 B) and
    //     their node ids (64 B), one instruction, issued by wave 0. Both tables are padded by
    //     one tile on the host, so a ragged last tile reads valid memory.
    auto gather_desc = [&](int64_t p0, int parity) __attribute__((always_inline)) {
        if (wave == 0 && lane < 36) {
            const void* src = lane < 32 ? (const void*)(p.ell + p0 * W + lane * 4) : (const void*)(p.order + p0 + (lane - 32) * 4);
            dma16(src, lds0 + (uint32_t)(SMEM_DESC + parity * DESC_BYTES));
        }
    };
    // (2) rows that depend on nobody else: a gate's own Q|K|V (1.5 KB) and its residual row
    auto gather_own = [&](int64_t p0, int rows, int parity) __attribute__((always_inline)) {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int g = 4 * wave + gq;
            if (g >= rows) continue;
            const int64_t orig = __builtin_amdgcn_readfirstlane(ids_of(parity)[g]);
            const uint16_t* self = p.qkv_self + (p0 + g) * (3 * D);
            const uint32_t dst = lds0 + (uint32_t)(SMEM_LAND + g * LAND_GATE + LAND_SELF);
            dma16_row(self + D, lane16, dst);                                                                // K | V
            const uint16_t* tail = lane < 32 ? self + lane * 8 : p.x + orig * D + (lane - 32) * 8;          // Q | x
            dma16(tail, dst + 1024u);
        }
    };
    //     The same for a full tile (nearly all are), with few instructions: one scalar base walked
    //     from gate to gate for the K|V halves; for the second transfer (Q in lanes 0..31, the
    //     residual row in lanes 32..63) a per-lane base plus 512 * (3*gq | node id).
    auto gather_own_full = [&](int64_t p0, int parity) __attribute__((always_inline)) {
        const unsigned char* kv_row = (const unsigned char*)p.qkv_self + (p0 + 4 * wave) * (3 * D * 2) + D * 2;
        const bool lo = lane < 32;
        const uint64_t base = lo ? (uint64_t)(uintptr_t)p.qkv_self + (uint64_t)(p0 + 4 * wave) * (3 * D * 2) + lane16
                                 : (uint64_t)(uintptr_t)p.x + (lane16 - 512u);
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const uint32_t dst = wave_land + (uint32_t)(gq * LAND_GATE + LAND_SELF);
            dma16_row(kv_row + gq * (3 * D * 2), lane16, dst);                                              // K | V
            const uint32_t sel = lo ? 3u * gq : (uint32_t)ids_of(parity)[4 * wave + gq];
            dma16((const void*)(uintptr_t)(base + (uint64_t)sel * (D * 2)), dst + 1024u);                    // Q | x
        }
    };
    // (3) the K|V kilobyte of a source: one instruction per (gate, source), in a loop over the
    //     set bits of `take` (bit 16*gq + j = entry j of this wave's gate gq). Each lane holds
    //     "its" entry (entry `sub` of gate `my`) and the slot it lands in; slot s of a gate holds
    //     its s-th source. Row base addresses are wave-uniform (scalar arithmetic); the only
    //     per-lane part is the fixed 16-byte stride.
    auto gather_some = [&](uint32_t e_mine, uint32_t slot_mine, uint64_t& take, int most) __attribute__((always_inline)) {
        while (take && most-- > 0) {
            const int b = __builtin_ctzll(take);
            take &= take - 1;
            const uint32_t e = (uint32_t)__builtin_amdgcn_readlane((int)e_mine, b);
            const uint32_t slot = (uint32_t)__builtin_amdgcn_readlane((int)slot_mine, b);
            const int g = 4 * wave + (b >> 4);
            if (slot < (uint32_t)NS)
                dma16_row((const unsigned char*)p.kv + (uint64_t)(e & 0x3FFFFFFFu) * (2 * D * 2), (uint32_t)lane * 16u,
                          lds0 + (uint32_t)(SMEM_LAND + g * LAND_GATE) + slot * 1024u);
        }
    };
    // slot of "my" entry: how many sources of my gate come before it in the row
    auto slot_of = [&](uint64_t need) __attribute__((always_inline)) -> uint32_t {
        const uint32_t gate_bits = (uint32_t)(need >> (16 * grp)) & 0xFFFFu;
        return (uint32_t)__builtin_popcount(gate_bits & ((1u << sub) - 1u));
    };
    // The sources of this wave's gates: lane (grp, sub) watches entry `sub` of gate `my`.
    // Returns the ballot of lanes whose entry is a source; `*up` gets those whose flag is raised.
    auto look = [&](int parity, int rows, uint64_t* up, uint32_t* e_mine) __attribute__((always_inline)) -> uint64_t {
        const uint32_t e = sub < W ? ent_of(parity)[my][sub] : DG4_ELL_PAD;
        *e_mine = e;
        const bool need = my < rows && e != DG4_ELL_PAD && (e >> 30) != 0;
        const bool ok = need && __hip_atomic_load(p.flags + (e & 0x3FFFFFFFu), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
        *up = __ballot(ok);
        // No cache invalidation is needed once a flag is seen: a K|V row is written once per
        // sweep, through to device memory, before its flag; nobody reads it earlier, so no cache
        // of this compute unit or its L2 can hold an older copy. The fence only keeps the
        // compiler from moving row loads above the flag loads.
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        return __ballot(need);
    };
    // Flag snapshots without registers: every lane fetches the flag word of the entry it watches
    // (word 0 if it watches none) into its own LDS word; read back with looked() after a wait.
    auto look_async = [&](uint32_t e, bool need, int which) __attribute__((always_inline)) {
        dma4_fresh(p.flags, need ? (e & 0x3FFFFFFFu) * 4u : 0u, lds0 + (uint32_t)(SMEM_LOOK + which * 1024 + wave * 256));
    };
    auto looked = [&](int which) __attribute__((always_inline)) -> uint32_t {
        return ((const uint32_t*)(smem + SMEM_LOOK + which * 1024))[wave * 64 + lane];
    };
    // Block until the sources in `late` are published, then fetch them.
    auto wait_and_gather = [&](int parity, int rows, uint64_t late, uint64_t need) __attribute__((always_inline)) {
        uint32_t spins = 0;
        uint32_t e_mine = DG4_ELL_PAD;
        for (;;) {
            uint64_t up;
            (void)look(parity, rows, &up, &e_mine);
            if ((late & ~up) == 0) break;
            __builtin_amdgcn_s_sleep(1);
            if (++spins > p.spin_limit ||
                ((spins & 63u) == 0 && __hip_atomic_load(&p.ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                if (lane == 0) {
                    __hip_atomic_store(&p.ctrl[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    sAbort = 1;
                }
                break;
            }
        }
        gather_some(e_mine, slot_of(need), late, 64);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __asm__ volatile("" ::: "memory");
    };

    // Tiles are handed out by tickets (p.ctrl[2], zero at launch): a workgroup holds the tile it works
    // on and the next two, drawn in ascending order, and draws one more per tile; the drawn number
    // reaches the other waves through LDS. With the feed-forward sub-block a ticket is a PAIR of
    // tiles (2k, 2k+1) that one workgroup runs back to back; the table then holds an even number of
    // tiles. Tickets past the end are clamped where a descriptor is fetched (harmless, unused).
    // (Dealing runs of consecutive tiles to one XCD, so that gates sharing a source share an L2, was
    // measured and is not worth it: 80 % of a tile's source rows are distinct already inside the
    // tile, 71 % inside 32 consecutive tiles.)
    int* sTick = (int*)(smem + SMEM_ABORT) + 1;
    // (thread 0 keeps one more drawn ticket in `spare`: a draw takes about as long as a third of a
    // tile, so what a tile hands to the other waves was drawn during the tile before)
    int spare = 0;
    if (threadIdx.x == 0) {
        sTick[0] = first_ticket;
        sTick[1] = FFN ? first_ticket + 1 : draw();
        sTick[2] = draw();
        spare = draw();
    }
    __syncthreads();
    int q0 = __builtin_amdgcn_readfirstlane(sTick[0]);            // this tile, the next one, the one after
    int q1 = __builtin_amdgcn_readfirstlane(sTick[1]);
    int q2 = __builtin_amdgcn_readfirstlane(sTick[2]);
    if (q0 >= p.n_tiles) return;
    const int64_t last = p.n_tiles - 1;
    int d0 = 0, d1 = 1, d2 = 2;                   // descriptor buffers of this tile, the next one, the one after
    uint2 cur = tile_at(q0);                                          // first position, rows
    uint2 nxt = tile_at(q1 < last ? q1 : last);
    uint64_t late = 0, need_cur = 0;              // sources of the current tile not gathered yet / all of them
    {
        gather_desc(cur.x, 0);
        gather_desc(nxt.x, 1);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();                          // sAbort, descriptors of the first two tiles
        gather_own(cur.x, (int)cur.y, 0);
        uint64_t up;
        uint32_t e0;
        need_cur = look(0, (int)cur.y, &up, &e0);
        late = need_cur;                          // the first tile fetches all its sources at the top of the loop
    }
    int64_t pub_p0 = 0;                           // rows 4*wave .. of the previous tile still to be published
    int pub_rows = 0;
    int64_t pairA_p0 = 0;                         // feed-forward pairs: the first tile of the pair in progress ...
    int pairA_rows = 0;
    int64_t pairA_orig = 0;                       // ... and the node id of its gate `sub` (this lane's output row)
    int64_t pubA_p0 = 0;                          // and of the finished pair, still to be published
    int pubA_rows = 0;

    for (;;) {
        // keep the Wk|Wv tiles in the accumulation registers
#pragma unroll
        for (int nt = 0; nt < 8; ++nt)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) __asm__ volatile("" : "+a"(wkv_r[nt][ks]));

        const int64_t p0 = cur.x;
        const int rows = (int)cur.y;
        const bool has_next = q1 < p.n_tiles;
        // (a wave none of whose four gates exists in the next tile, as on the small tiles of narrow circuits,
        // has no rows to request for it)
        const bool wave_gathers = has_next && 4 * wave < (int)nxt.y;
        const bool second = FFN && (q0 & 1) != 0;             // second tile of a feed-forward pair
        const bool first = FFN && !second;
        roles();

        // ---------------- the previous tile's rows and this tile's gathers. Loads and stores of a
        // wave complete in order, and the last things it issued were the eight K|V row stores
        // of the previous tile: once at most eight operations are outstanding, every gather of
        // this tile has landed, and the attention can start while the stores are still on
        // their way. The flags of those rows (each wave raises the four it stored itself)
        // follow further down, once the stores have completed (= are written through, visible
        // to every compute unit). Only a wave that has to wait for late sources, or whose
        // previous tile was ragged (fewer stores), waits for everything here: the flags must
        // be up before any blocking wait, other workgroups may be waiting for them. (So does
        // every wave when the tiles are dealt level by level: there the readers follow closely.)
        auto publish = [&]() __attribute__((always_inline)) {
            if (lane < 4 && 4 * wave + lane < pub_rows)
                __hip_atomic_store(&p.flags[pub_p0 + 4 * wave + lane], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (FFN && lane < 4 && 4 * wave + lane < pubA_rows)
                __hip_atomic_store(&p.flags[pubA_p0 + 4 * wave + lane], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        bool published = false;
        // (a finished pair leaves sixteen row stores behind; the second tile of a pair has nothing
        // to publish but must see its own rows, which were requested last)
        const bool may_defer = !TIMERS && !p.eager_publish && !late &&
                               (FFN ? first && pub_rows == TILE && pubA_rows == TILE : pub_rows == TILE);
        if (!may_defer) {                     // (the timed build has a barrier right below: flags first)
            __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0), expcnt and lgkmcnt untouched
            __asm__ volatile("" ::: "memory");
            publish();
            published = true;
        } else if (FFN) {
            __builtin_amdgcn_s_waitcnt(0x4F70);       // vmcnt(16)
            __asm__ volatile("" ::: "memory");
        } else {
            __builtin_amdgcn_s_waitcnt(0x0F78);       // vmcnt(8)
            __asm__ volatile("" ::: "memory");
        }
        lap(6);
        // sources that were not published yet when this tile's gathers went out
        if (late) wait_and_gather(d0, rows, late, need_cur);
        if (TIMERS) __syncthreads();          // timers only: charge every wave's wait to phase 1
        lap(1);
        // the descriptor two tiles ahead travels during the attention below
        const uint2 nn = tile_at(q2 < last ? q2 : last);
        gather_desc(nn.x, d2);
        // the tile after those: the second of a pair follows its first, anything else takes the
        // spare ticket (further down, where a wait that is there anyway has covered its draw)
        const bool draws = !FFN || (q2 & 1) != 0;
        // A first look at the flags of the NEXT tile's sources (its descriptor came in a round
        // ago). Loaded by every lane, needed or not; looked at after the first attention round.
        uint32_t nent = DG4_ELL_PAD;
        bool nneed = false;
        if (has_next) {
            nent = sub < W ? ent_of(d1)[my][sub] : DG4_ELL_PAD;
            nneed = my < (int)nxt.y && nent != DG4_ELL_PAD && (nent >> 30) != 0;
        }
        look_async(nent, nneed, 0);
        if constexpr (FFN) {
            // Wo for this tile's output projection (the feed-forward sub-block needs its registers
            // in between, so it is not kept). Requested here, before any of the tile's transfers:
            // the loads are complete at the wait after the first attention pass, which the compiler
            // sees, and nothing further down waits on vector memory because of them. (The address
            // goes through an opaque copy: the loads must stay inside the loop; and it is typed as
            // global memory again, or the loads would be flat ones.)
            uint64_t wa = (uint64_t)(uintptr_t)((const uint4*)p.wo_packed + (int64_t)wave * 4 * 8 * 64 + lane);
            __asm__ volatile("" : "+v"(wa));
            const __attribute__((address_space(1))) u32x4* wl = (const __attribute__((address_space(1))) u32x4*)wa;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
                    if (!(nt == 3 && ks == 7)) wo_r[nt][ks] = wl[(nt * 8 + ks) * 64];
            __builtin_amdgcn_sched_barrier(0);
        }
        uint64_t need_nxt = 0, up_nxt = 0;
        uint32_t nslot = 0;
        uint32_t keep_lo = 0, keep_hi = 0;

        // ---------------- attention: gate `my`, lane owns 16 features (two lanes per head). Two
        // passes over the row: scores of all entries from the K halves, softmax over them in
        // registers, then the weighted sum over the V halves. Entries are handled in pairs; how
        // many pairs is the same for the whole wave (gates with fewer entries idle with weight
        // zero), because the wave also issues, after each pair of the second pass, the gathers of
        // the next tile into the source slots that pair has just finished reading: after pair r
        // every gate is done with its slots 0 .. 2r (a row holds at most one entry that is no source).
        {
            roles();
            const bool valid = my < rows;
            const unsigned char* land = sLand + my * LAND_GATE + sub * 32;
            uint32_t q[8];
            {
                const uint4* qp = (const uint4*)(land + LAND_Q);
                const uint4 a = qp[0], b = qp[1];
                q[0] = a.x; q[1] = a.y; q[2] = a.z; q[3] = a.w; q[4] = b.x; q[5] = b.y; q[6] = b.z; q[7] = b.w;
            }
            uint32_t e[8];
            {
                const uint4* ep = (const uint4*)&ent_of(d0)[my][0];
                const uint4 a = ep[0], b = ep[1];
                e[0] = a.x; e[1] = a.y; e[2] = a.z; e[3] = a.w; e[4] = b.x; e[5] = b.y; e[6] = b.z; e[7] = b.w;
            }
            // first pass: scores, in units of log 2 (scale and bias table carry the factor log2 e).
            // All eight entries of the row are processed, padding included (it reads the gate's
            // own rows and gets weight zero): no branches, so the loads of several entries are
            // in flight together.
            const float scale = 0.17677669529663687f * 1.4426950408889634f;           // log2(e) / sqrt(32)
            float sc[8];
            // per entry, 4 bits each: where its K|V sits (source slot 0..5, 6 = the gate's own rows)
            // and its relation code with a "present" bit (the register file is full: two registers
            // instead of sixteen)
            uint32_t where = 0, what = 0;
            {
                uint32_t slot = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool present = e[j] != DG4_ELL_PAD;                                   // entries are packed from 0
                    const bool src = present && (e[j] >> 30) != 0 && slot < (uint32_t)NS;
                    where |= (src ? slot : 6u) << (4 * j);
                    what |= (present ? 4u | (e[j] >> 30) : 3u) << (4 * j);
                    slot += src ? 1u : 0u;
                }
            }
            auto k_of = [&](int j) __attribute__((always_inline)) {                             // V sits 512 bytes after K
                return (const uint4*)(land + (((where >> (4 * j)) & 7u) << 10));
            };
            // (the rows of pair h+1 are requested before pair h is used: with one wave per SIMD
            // nothing else hides the LDS latency)
            uint4 kr[2][4];                               // [buffer][entry of the pair: two 16-byte halves each]
            float br[2][2];
            auto load_k = [&](int h, int bufi) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const uint4* kp = k_of(2 * h + j);
                    kr[bufi][2 * j] = kp[0]; kr[bufi][2 * j + 1] = kp[1];
                    br[bufi][j] = sBias[(what >> (4 * (2 * h + j))) & 3u];          // padding reads entry 3 of the table, unused
                }
            };
            load_k(0, 0);
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                if (h + 1 < 4) load_k(h + 1, (h + 1) & 1);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const uint4 k0 = kr[h & 1][2 * j], k1 = kr[h & 1][2 * j + 1];
                    float d0 = 0.f, d1 = 0.f;                     // two chains: the dot products issue back to back
                    d0 = dot2_bf16(q[0], k0.x, d0); d1 = dot2_bf16(q[1], k0.y, d1);
                    d0 = dot2_bf16(q[2], k0.z, d0); d1 = dot2_bf16(q[3], k0.w, d1);
                    d0 = dot2_bf16(q[4], k1.x, d0); d1 = dot2_bf16(q[5], k1.y, d1);
                    d0 = dot2_bf16(q[6], k1.z, d0); d1 = dot2_bf16(q[7], k1.w, d1);
                    const float d = Elem<bf16_t>::head_sum(d0 + d1);
                    const float t = fmaf(d, scale, br[h & 1][j]);
                    sc[2 * h + j] = (what >> (4 * (2 * h + j)) & 4u) ? t : -INFINITY;   // padding: weight 2^-inf = 0
                }
                __builtin_amdgcn_sched_barrier(0);            // no further hoisting: the register file is full
            }
            // the first look has had the first pass to come back (so has the descriptor fetch)
            uint32_t src_lo = 0, src_hi = 0;              // lane 8*gate + slot: row address of that source of the next tile
            {
                __builtin_amdgcn_s_waitcnt(0x0F70);
                __asm__ volatile("" ::: "memory");
                if (!published) publish();        // the previous tile's row stores have completed too
                if (draws && threadIdx.x == 0) { sTick[0] = spare; spare = draw(); }
                need_nxt = __ballot(nneed);
                const bool upl = nneed && looked(0) != 0u;
                up_nxt = __ballot(upl);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");     // row gathers stay below the flag loads
                nslot = slot_of(need_nxt);
                // Row addresses by (gate, slot), so that the issue below is straight-line code
                // with fixed lanes and fixed LDS addresses (with one wave per SIMD every
                // instruction counts): lanes scatter the address of their entry through LDS to
                // lane 8*gate + slot. Slots without a published source point at the first kilobyte
                // of the projected self rows: that transfer is wasted but harmless (its slot is
                // unused, or refilled later). It must not touch the K|V store: a row of it read
                // before it is written would leave a stale copy in this XCD's L2 for the gates
                // that read it as a source later.
                uint64_t* tmp = (uint64_t*)(smem + SMEM_LOOK + 2048) + wave * 32;
                if (lane < 32) tmp[lane] = (uint64_t)(uintptr_t)p.qkv_self;
                if (upl && nslot < (uint32_t)NS)
                    tmp[grp * 8 + nslot] = (uint64_t)(uintptr_t)p.kv + (uint64_t)(nent & 0x3FFFFFFFu) * (2 * D * 2);
                const uint64_t a = tmp[lane & 31];
                src_lo = (uint32_t)a; src_hi = (uint32_t)(a >> 32);
            }
            {
                const float mx = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
                float z = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) { sc[j] = __builtin_amdgcn_exp2f(sc[j] - mx); z += sc[j]; }
                const float rz = 1.0f / z;
#pragma unroll
                for (int j = 0; j < 8; ++j) sc[j] *= rz;
            }
            // second pass: weighted sum of the V halves, two entries at a time. After pair r every
            // gate is done with its slots 0 .. 2r (a row holds at most one entry that is no
            // source), so the next tile's sources for those slots can start to travel.
            float acc[16];
            uint4 vr[2][4];
            auto load_v = [&](int r, int bufi) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const uint4* vp = k_of(2 * r + j) + 32;
                    vr[bufi][2 * j] = vp[0]; vr[bufi][2 * j + 1] = vp[1];
                }
            };
            load_v(0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (r + 1 < 4) load_v(r + 1, (r + 1) & 1);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    float f[16];
                    Elem<bf16_t>::unpack(vr[r & 1][2 * j], vr[r & 1][2 * j + 1], f);
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] = (r == 0 && j == 0) ? sc[0] * f[i] : fmaf(sc[2 * r + j], f[i], acc[i]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // this pair's rows are in registers (so are the next pair's, which sit in higher
                // slots): its slots may be overwritten
                __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0)
                // (the gathers are spread out: a wave that issues more transfers than the memory
                // pipeline takes stalls until they have drained. Slots 0 .. 2 go here, 3 .. 5 below,
                // around the output projection)
                if (wave_gathers) {
                    if (r == 0) issue_slots<0, 1>(src_lo, src_hi, lane16, wave_land);
                    else if (r == 1) issue_slots<1, 3>(src_lo, src_hi, lane16, wave_land);
                }
            }
            keep_lo = src_lo; keep_hi = src_hi;
            uint4 oa, ob;
            if (valid) Elem<bf16_t>::pack(acc, oa, ob);
            else { oa = make_uint4(0, 0, 0, 0); ob = oa; }
            uint4* dst = (uint4*)&sA[my][sub * 16];
            dst[0] = oa; dst[1] = ob;
        }
        // a second look at the sources the first one found unpublished, answered while the matrix
        // cores work below
        const bool miss = nneed && ((up_nxt >> lane) & 1u) == 0u;
        const bool any_miss = (need_nxt & ~up_nxt) != 0;
        if (any_miss) look_async(nent, miss, 1);
        __syncthreads();                      // sA and the descriptor fetched above complete
        if (sAbort) { flush(); return; }
        const int q3 = draws ? __builtin_amdgcn_readfirstlane(sTick[0]) : q2 + 1;
        lap(2);
        if (wave_gathers) issue_slots<3, 5>(keep_lo, keep_hi, lane16, wave_land);
        if (second) {
            // the rows the first tile of the pair parked in global memory come back into the places
            // of the gates' own K|V, which the attention has finished with (512 bytes a gate, each
            // row shifted by 16 bytes against its neighbour's so that lanes of different gates hit
            // different banks)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int g = 4 * wave + gq;
                if (lane < 32)
                    dma16_fresh(p.park + ((int64_t)blockIdx.x * TILE + g) * D + lane * 8,
                                lds0 + (uint32_t)(SMEM_LAND + g * LAND_GATE + LAND_SELF + g * 16));
            }
        }

        // ---------------- output projection; lane (n = sub, g = grp) owns columns 64*wave + 16*g .. +15 of gate n
        roles();
        const int n = sub;
        const bool nvalid = n < rows;
        float t[16];
        {
            // (accumulators start from a literal zero operand: zero-filled registers would be kept
            // alive across the whole loop)
            f32x4 acc[4];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const uint4 b = *(const uint4*)&sA[n][8 * grp + ks * 32];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
                    acc[nt] = mfma16(nt == 3 && ks == 7 ? *sWoF : __builtin_bit_cast(uint4, wo_r[nt][ks]), b,
                                     ks == 0 ? (f32x4){0.f, 0.f, 0.f, 0.f} : acc[nt]);
            }
                if (wave_gathers) issue_slots<5, 6>(keep_lo, keep_hi, lane16, wave_land);
            float x[16];
            {
                const uint4* xp = (const uint4*)(sLand + n * LAND_GATE + LAND_X + c0 * 2);
                Elem<bf16_t>::unpack(xp[0], xp[1], x);
            }
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int i = 0; i < 4; ++i) t[nt * 4 + i] = acc[nt][i] + (p.epilogue ? x[nt * 4 + i] : 0.f);
        }
        const int64_t orig_n = ids_of(d0)[nvalid ? n : 0];
        lap(3);
        if (p.epilogue) {
            float s1 = 0.f, s2 = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s1 += t[i]; s2 = fmaf(t[i], t[i], s2); }
            s1 = sum_rows(s1); s2 = sum_rows(s2);
            if (grp == 0) { sRed[n][wave][0] = s1; sRed[n][wave][1] = s2; }
            __syncthreads();
                float a1 = 0.f, a2 = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) { a1 += sRed[n][w2][0]; a2 += sRed[n][w2][1]; }
            const float mean = a1 * (1.0f / D);
            const float var = fmaxf(a2 * (1.0f / D) - mean * mean, 0.f);
            const float rstd = rsqrtf(var + p.ln_eps);
#pragma unroll
            for (int i = 0; i < 16; ++i) t[i] = (t[i] - mean) * rstd;
        }
        if (any_miss) {
            // The second snapshot. Transfers complete in order, so this also waits for the gathers
            // issued during the attention; only waves that had a miss pay for it.
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __asm__ volatile("" ::: "memory");
            uint64_t up2 = __ballot(miss && looked(1) != 0u);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            up_nxt |= up2;
            gather_some(nent, nslot, up2, 64);
        }
        if (TIMERS && threadIdx.x == 0 && (need_nxt & ~up_nxt)) sProf[0] += 1;       // tiles with a late source
        {
            uint4 ha, hb;
            Elem<bf16_t>::pack(t, ha, hb);
            if (!FFN && nvalid) {
                uint4* hp = (uint4*)(p.h_out + orig_n * D + c0);
                hp[0] = ha; hp[1] = hb;
            }
            if (first) {                      // parked until the second tile of the pair has come this far
                uint4* pp = (uint4*)(p.park + ((int64_t)blockIdx.x * TILE + n) * D + c0);
                pp[0] = ha; pp[1] = hb;
            }
            uint4* hs = (uint4*)&sH[n][c0];
            hs[0] = ha; hs[1] = hb;
        }
        if (second) {                         // the parked rows have arrived (so have the next tile's sources so far)
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __asm__ volatile("" ::: "memory");
        }
        __syncthreads();                      // sH complete; every wave has read its residual rows
        lap(4);
        roles();
        // the landing zone of the gates' own rows is free now: the next tile's may come in (the
        // second tile of a feed-forward pair still needs the space: see below)
        auto gather_next_own = [&]() __attribute__((always_inline)) {
            if (has_next) {
                if ((int)nxt.y == TILE) gather_own_full(nxt.x, d1);
                else gather_own(nxt.x, (int)nxt.y, d1);
            }
        };
        if (!second) gather_next_own();

        // K|V projection of the rows in sH, out through LDS as 512-byte device-scope stores
        auto kv_out = [&](int64_t q0, int nrows) __attribute__((always_inline)) {
            f32x4 acc[8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const uint4 b = *(const uint4*)&sH[n][8 * grp + ks * 32];
#pragma unroll
                for (int nt = 0; nt < 8; ++nt)
                    acc[nt] = mfma16(__builtin_bit_cast(uint4, wkv_r[nt][ks]), b, ks == 0 ? (f32x4){0.f, 0.f, 0.f, 0.f} : acc[nt]);
            }
            uint4* dst = (uint4*)&sKV[n][128 * wave + 32 * grp];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const f32x4 u = acc[2 * h], v = acc[2 * h + 1];
                dst[h] = make_uint4(pack_bf16x2(u[0], u[1]), pack_bf16x2(u[2], u[3]),
                                    pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
            }
            __syncthreads();
            // wave w writes rows 4w..4w+3, 512 contiguous bytes per instruction, as device-scope
            // stores (written through the L2 of this XCD). Their flags follow at the top of the
            // next round, once the stores have completed.
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = 4 * wave + rr;
                if (r < nrows) {
                    uint64_t* gp = (uint64_t*)(p.kv + (q0 + r) * (2 * D));
                    const uint64_t* lp = (const uint64_t*)&sKV[r][0];
                    __hip_atomic_store(gp + lane, lp[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(gp + 64 + lane, lp[64 + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            __syncthreads();                  // sKV has been read; sA and sH may be written again
        };

        if constexpr (!FFN) {
            // ---------------- K|V projection of the new embeddings: lane owns columns 128*wave + 32*g .. +31
            kv_out(p0, rows);
            lap(5);
            pub_p0 = p0; pub_rows = rows;
        } else if (first) {
            // first tile of a pair: its rows are parked, the rest of its work happens with the second tile
            pairA_p0 = p0; pairA_rows = rows; pairA_orig = orig_n;
            pub_rows = 0; pubA_rows = 0;
        } else {
            // ---------------- feed-forward sub-block (Section 3.5 keeps the transformer structure around
            // the attention): h <- LN(h + max(h W1, 0) W2) for the 32 gates of the pair, tile A's rows
            // in the landing zone (own-K|V places), tile B's in sH. The megabyte of W1 | W2 fits
            // neither the registers nor LDS next to everything else, so it is streamed from the L2
            // cache, every wave its own contiguous stream, through a ring of RING fragments that
            // are requested RING products before the matrix cores need them; running two tiles
            // through one pass halves that stream, which is what bounds the phase (about 75 GB/s
            // per compute unit, whatever the depth of the ring). Per pass of 256 hidden units:
            // every wave forms 64 of the activations of both tiles (transposed, so that a lane ends
            // up with four consecutive hidden units of one gate), they are exchanged through LDS
            // (tile B: the idle attention buffer, tile A: the idle own-Q / residual places of the
            // landing zone), and every wave adds the pass's part of its own 64 output columns.
            constexpr int RING = 16;
            static_assert(FFN_FRAGS % RING == 0, "ring slots repeat from pass to pass");
            const uint4* wp = (const uint4*)p.ffn_packed + (int64_t)wave * (FFN_PASSES * FFN_FRAGS * 64) + lane;
            u32x4 ring[RING];
            static_for<0, RING>([&](auto I) __attribute__((always_inline)) { ring[I.value] = __builtin_bit_cast(u32x4, wp[I.value * 64]); });
            uint16_t (*sU)[LDS_STRIDE] = sA;
            const unsigned char* hA = sLand + n * (LAND_GATE + 16) + LAND_SELF;       // tile A: input rows
            unsigned char* uAp = sLand + n * (LAND_GATE + 16) + LAND_Q;               // tile A: activations of a pass
            f32x4 outA[4], outB[4];
#pragma unroll 1
            for (int pass = 0; pass < FFN_PASSES; ++pass) {
                const uint4* wq = wp + (int64_t)pass * (FFN_FRAGS * 64);
                const bool more = pass + 1 < FFN_PASSES;
                // Activations of hidden units 256*pass + 64*wave .. +63, transposed, 32 units at a time
                // (registers). The tiles' operands of the next group of products are read from LDS
                // while this group runs: with one wave per SIMD nothing else hides that latency.
                if (pass) {                       // the previous pass's activations have been read by every wave
                    __asm__ volatile("" ::: "memory");
                    __builtin_amdgcn_s_waitcnt(0xC07F);
                    __builtin_amdgcn_s_barrier();
                    __asm__ volatile("" ::: "memory");
                }
                static_for<0, 2>([&](auto HALF) __attribute__((always_inline)) {
                    constexpr int half = HALF.value;
                    f32x4 uA[2], uB[2];
                    uint4 a_cur = *(const uint4*)(hA + 16 * grp);
                    uint4 b_cur = *(const uint4*)&sH[n][8 * grp];
                    static_for<0, 8>([&](auto KS) __attribute__((always_inline)) {
                        constexpr int ks = KS.value;
                        uint4 a_nxt = a_cur, b_nxt = b_cur;
                        if (ks + 1 < 8) {
                            a_nxt = *(const uint4*)(hA + 16 * grp + (ks + 1) * 64);
                            b_nxt = *(const uint4*)&sH[n][8 * grp + (ks + 1) * 32];
                        }
#pragma unroll
                        for (int h2 = 0; h2 < 2; ++h2) {
                            const int j = 16 * half + 2 * ks + h2, slot = j % RING;
                            const uint4 frag = __builtin_bit_cast(uint4, ring[slot]);
                            uA[h2] = mfma16(frag, a_cur, ks == 0 ? (f32x4){0.f, 0.f, 0.f, 0.f} : uA[h2]);
                            uB[h2] = mfma16(frag, b_cur, ks == 0 ? (f32x4){0.f, 0.f, 0.f, 0.f} : uB[h2]);
                            ring[slot] = __builtin_bit_cast(u32x4, wq[(j + RING) * 64]);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        a_cur = a_nxt; b_cur = b_nxt;
                    });
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) {
                        const int col = 64 * wave + 32 * half + 16 * h2 + 4 * grp;
                        *(uint2*)(uAp + col * 2) =
                            make_uint2(pack_bf16x2(fmaxf(uA[h2][0], 0.f), fmaxf(uA[h2][1], 0.f)), pack_bf16x2(fmaxf(uA[h2][2], 0.f), fmaxf(uA[h2][3], 0.f)));
                        *(uint2*)&sU[n][col] =
                            make_uint2(pack_bf16x2(fmaxf(uB[h2][0], 0.f), fmaxf(uB[h2][1], 0.f)), pack_bf16x2(fmaxf(uB[h2][2], 0.f), fmaxf(uB[h2][3], 0.f)));
                    }
                });
                __asm__ volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xC07F);
                __builtin_amdgcn_s_barrier();
                __asm__ volatile("" ::: "memory");
                // this pass's part of output columns 64*wave + 16*grp .. +15
                {
                    uint4 a_cur = *(const uint4*)(uAp + 16 * grp);
                    uint4 b_cur = *(const uint4*)&sU[n][8 * grp];
                    static_for<0, 8>([&](auto KK) __attribute__((always_inline)) {
                        constexpr int kk = KK.value;
                        uint4 a_nxt = a_cur, b_nxt = b_cur;
                        if (kk + 1 < 8) {
                            a_nxt = *(const uint4*)(uAp + 16 * grp + (kk + 1) * 64);
                            b_nxt = *(const uint4*)&sU[n][8 * grp + (kk + 1) * 32];
                        }
#pragma unroll
                        for (int ct = 0; ct < 4; ++ct) {
                            const int j = 32 + 4 * kk + ct, slot = j % RING;
                            const uint4 frag = __builtin_bit_cast(uint4, ring[slot]);
                            outA[ct] = mfma16(frag, a_cur, (pass == 0 && kk == 0) ? (f32x4){0.f, 0.f, 0.f, 0.f} : outA[ct]);
                            outB[ct] = mfma16(frag, b_cur, (pass == 0 && kk == 0) ? (f32x4){0.f, 0.f, 0.f, 0.f} : outB[ct]);
                            if (j + RING < FFN_FRAGS || more)         // (past the end of this pass: the first fragments of the next)
                                ring[slot] = __builtin_bit_cast(u32x4, wq[(j + RING) * 64]);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        a_cur = a_nxt; b_cur = b_nxt;
                    });
                }
            }
            // residual (this lane's own 16 columns of its gate), LayerNorm, the new rows: both tiles
            float tA[16];
            {
                float h1[16];
                const uint4* hp = (const uint4*)&sH[n][c0];
                Elem<bf16_t>::unpack(hp[0], hp[1], h1);
#pragma unroll
                for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                    for (int i = 0; i < 4; ++i) t[ct * 4 + i] = outB[ct][i] + h1[ct * 4 + i];
                const uint4* ap = (const uint4*)(hA + c0 * 2);
                Elem<bf16_t>::unpack(ap[0], ap[1], h1);
#pragma unroll
                for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                    for (int i = 0; i < 4; ++i) tA[ct * 4 + i] = outA[ct][i] + h1[ct * 4 + i];
            }
            float s1 = 0.f, s2 = 0.f, r1 = 0.f, r2 = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s1 += t[i]; s2 = fmaf(t[i], t[i], s2); r1 += tA[i]; r2 = fmaf(tA[i], tA[i], r2); }
            s1 = sum_rows(s1); s2 = sum_rows(s2); r1 = sum_rows(r1); r2 = sum_rows(r2);
            float (*sRedA)[4][2] = (float (*)[4][2])(smem + SMEM_BYTES);
            __syncthreads();                  // every wave is done with the activations and with the input rows as operands
            if (grp == 0) { sRed[n][wave][0] = s1; sRed[n][wave][1] = s2; sRedA[n][wave][0] = r1; sRedA[n][wave][1] = r2; }
            __syncthreads();
            // the landing zone is free for good now
            gather_next_own();
            uint4 hB0, hB1;
            {
                float a1 = 0.f, a2 = 0.f, b1 = 0.f, b2 = 0.f;
#pragma unroll
                for (int w2 = 0; w2 < 4; ++w2) { a1 += sRed[n][w2][0]; a2 += sRed[n][w2][1]; b1 += sRedA[n][w2][0]; b2 += sRedA[n][w2][1]; }
                float mean = a1 * (1.0f / D);
                float rstd = rsqrtf(fmaxf(a2 * (1.0f / D) - mean * mean, 0.f) + p.ln_eps);
#pragma unroll
                for (int i = 0; i < 16; ++i) t[i] = (t[i] - mean) * rstd;
                Elem<bf16_t>::pack(t, hB0, hB1);
                if (nvalid) {
                    uint4* hp = (uint4*)(p.h_out + orig_n * D + c0);
                    hp[0] = hB0; hp[1] = hB1;
                }
                mean = b1 * (1.0f / D);
                rstd = rsqrtf(fmaxf(b2 * (1.0f / D) - mean * mean, 0.f) + p.ln_eps);
#pragma unroll
                for (int i = 0; i < 16; ++i) tA[i] = (tA[i] - mean) * rstd;
                uint4 hA0, hA1;
                Elem<bf16_t>::pack(tA, hA0, hA1);
                if (n < pairA_rows) {
                    uint4* hp = (uint4*)(p.h_out + pairA_orig * D + c0);
                    hp[0] = hA0; hp[1] = hA1;
                }
                uint4* hs = (uint4*)&sH[n][c0];
                hs[0] = hA0; hs[1] = hA1;
            }
            __syncthreads();                  // sH holds the final embeddings of tile A
            lap(7);
            kv_out(pairA_p0, pairA_rows);
            {
                uint4* hs = (uint4*)&sH[n][c0];
                hs[0] = hB0; hs[1] = hB1;
            }
            __syncthreads();                  // ... of tile B
            kv_out(p0, rows);
            lap(5);
            pub_p0 = p0; pub_rows = rows;
            pubA_p0 = pairA_p0; pubA_rows = pairA_rows;
        }

        if (!has_next) {
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __asm__ volatile("" ::: "memory");
            if (lane < 4 && 4 * wave + lane < pub_rows)
                __hip_atomic_store(&p.flags[pub_p0 + 4 * wave + lane], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (FFN && lane < 4 && 4 * wave + lane < pubA_rows)
                __hip_atomic_store(&p.flags[pubA_p0 + 4 * wave + lane], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            flush();
            return;
        }
        q0 = q1; q1 = q2; q2 = q3;
        { const int t = d0; d0 = d1; d1 = d2; d2 = t; }
        cur = nxt; nxt = nn;
        need_cur = need_nxt; late = need_nxt & ~up_nxt;
    }
}

}  // namespace

int dg4_launch_pack_wt(const void* w, int ld, int col0, int ntw, int waves, void* packed, hipStream_t s)
{
    const int64_t units = (int64_t)waves * ntw * 8 * 64;
    hipLaunchKernelGGL(pack_wt_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s,
                       (const uint16_t*)w, ld, col0, ntw, waves, (uint16_t*)packed);
    return hipGetLastError();
}

int dg4_launch_pack_ffn(const void* w1, const void* w2, void* packed, hipStream_t s)
{
    const int64_t units = 4 * FFN_PASSES * FFN_FRAGS * 64;
    hipLaunchKernelGGL(pack_ffn_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s,
                       (const uint16_t*)w1, (const uint16_t*)w2, (uint16_t*)packed);
    return hipGetLastError();
}

int dg4_launch_sweep_init(uint32_t* flags, uint32_t* ctrl, int64_t n_flags, int64_t done_below, hipStream_t s)
{
    hipLaunchKernelGGL(sweep_init_kernel, dim3((unsigned)((std::max<int64_t>(n_flags, 64) + 255) / 256)), dim3(256), 0, s,
                       flags, n_flags, done_below, ctrl);
    return hipGetLastError();
}

int dg4_launch_sweep(const dg4_sweep_args& a, hipStream_t s)
{
    if (a.n_tiles <= 0) return hipSuccess;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return hipErrorInvalidDevice;
    int64_t grid = std::min<int64_t>(cus, DG4_MAX_SWEEP_GROUPS);   // one workgroup per compute unit: its registers and LDS hold the weights
    if (a.ffn_packed) {
        if ((a.n_tiles & 1) || !a.park) return hipErrorInvalidValue;      // whole pairs only
        if (grid > a.n_tiles / 2) grid = a.n_tiles / 2;
    }
    if (grid > a.n_tiles) grid = a.n_tiles;
    void (*kern)(dg4_sweep_args) = nullptr;            // the LDS landing zone is laid out for cones of two hops
    if (a.ell_w == 8) {
        if (a.ffn_packed) kern = a.prof ? sweep_kernel<8, true, true> : sweep_kernel<8, false, true>;
        else kern = a.prof ? sweep_kernel<8, true, false> : sweep_kernel<8, false, false>;
    }
    if (!kern) return hipErrorInvalidValue;
    const int smem = SMEM_BYTES + (a.ffn_packed ? 512 : 0);      // pairs: a second LayerNorm exchange area
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), smem, s, a);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------------
// Bulk projection (bf16, hidden 256): out[r, 0..767] = S[idx(r), :] x Wqkv for many rows at once:
// Q | K | V of x for every gate before the sweep, or dg4_qkv_proj. HBM-bound (512 B in, 1.5 KB
// out per row). One persistent workgroup per compute unit keeps ALL of Wq|Wk|Wv in its
// registers (each wave 192 output columns: 96 fragments of a 32x32x16 product, 256 accumulation
// + 128 vector registers) and streams 32-row tiles past them: the rows of the next two tiles
// travel straight into LDS while this one is multiplied, results are transposed through LDS and
// leave as whole rows.
namespace {

typedef float f32x16s __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f32x16s mfma32(const uint4& a, const uint4& b, f32x16s c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8s, a), __builtin_bit_cast(bf16x8s, b), c, 0, 0, 0);
}

constexpr int PS_ROWS = 32;                              // rows per tile
constexpr int PS_XSTRIDE = 264;                          // bf16 per input row in LDS (16 bytes of padding)
constexpr int PS_OSTRIDE = 776;                          // bf16 per staged output row
constexpr int PS_OUT = 3 * PS_ROWS * PS_XSTRIDE * 2;     // a ring of three input tiles first
constexpr int PS_BYTES = PS_OUT + PS_ROWS * PS_OSTRIDE * 2;
constexpr int PS_NT = 6;                                 // column tiles of 32 per wave

// Weights as the A operand of a 32x32x16 product, 16-byte units: unit (((wave*6 + tile)*16 + ks)*64
// + lane) holds rows k = ks*16 + 8*(lane/32) .. +7 of column 192*wave + 96*hi + 16*tile + 4*a + b,
// where lane%32 = 8*a + 4*hi + b. With the rows of the tile as B operand, accumulator register
// 4*a + b of lane (n = lane%32, hi = lane/32) is then row n, column 192*wave + 96*hi + 16*tile +
// 4*a + b: every lane owns 96 contiguous columns of one row.
__global__ void pack_w32_kernel(const uint16_t* w, int ld, uint16_t* packed)
{
    const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (unit >= 4 * PS_NT * 16 * 64) return;
    const int lane = (int)(unit & 63);
    const int ks = (int)((unit >> 6) & 15);
    const int t = (int)(unit >> 10);                   // wave*6 + tile
    const int tile = t % PS_NT, wave = t / PS_NT;
    const int m = lane & 31;
    const int a = m >> 3, hi = (m >> 2) & 1, b = m & 3;
    const int col = 192 * wave + 96 * hi + 16 * tile + 4 * a + b;
    const int k0 = ks * 16 + 8 * (lane >> 5);
#pragma unroll
    for (int j = 0; j < 8; ++j) packed[unit * 8 + j] = w[(int64_t)(k0 + j) * ld + col];
}

__global__ __launch_bounds__(256, 1) void proj768_kernel(dg4_bulk_args p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, hi = lane >> 5;
    const __attribute__((address_space(4))) int32_t* gat = (const __attribute__((address_space(4))) int32_t*)p.gather;

    u32x4 wa[4][16], wb[PS_NT - 4][16];
    {
        const uint4* w = (const uint4*)p.w_packed + (int64_t)wave * PS_NT * 16 * 64 + lane;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) wa[nt][ks] = __builtin_bit_cast(u32x4, w[(nt * 16 + ks) * 64]);
#pragma unroll
        for (int nt = 4; nt < PS_NT; ++nt)
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) wb[nt - 4][ks] = __builtin_bit_cast(u32x4, w[(nt * 16 + ks) * 64]);
    }
    const int64_t n_rows = p.row_end - p.row_begin;
    const int64_t n_tiles = (n_rows + PS_ROWS - 1) / PS_ROWS;
    const int64_t G = gridDim.x;
    int64_t t = blockIdx.x;
    if (t >= n_tiles) return;

    // wave w fetches rows 8w .. 8w+7 of a tile, one 512-byte transfer each (lanes 0..31); rows
    // past the end are clamped to the last one (their results are not stored)
    auto rows_of = [&](int64_t tile, int64_t* sr) __attribute__((always_inline)) {
        int64_t r[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            r[q] = p.row_begin + tile * PS_ROWS + 8 * wave + q;
            if (r[q] >= p.row_end) r[q] = p.row_end - 1;
        }
        if (gat) {                               // (one branch, so that the eight index loads go out together)
#pragma unroll
            for (int q = 0; q < 8; ++q) sr[q] = (int64_t)gat[r[q]];
        } else {
#pragma unroll
            for (int q = 0; q < 8; ++q) sr[q] = r[q];
        }
    };
    auto fetch = [&](const int64_t* sr, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (lane < 32)
                dma16_row((const unsigned char*)p.src + sr[q] * (D * 2), (uint32_t)lane * 16u,
                          lds0 + (uint32_t)(buf * PS_ROWS * PS_XSTRIDE * 2 + (8 * wave + q) * PS_XSTRIDE * 2));
    };
    // this lane's three 16-byte pieces of a pair of output rows (3072 bytes = three 1 KB stores):
    // which row of the pair, where in the staged row, where in the caller's tensors
    uint32_t st_lds[3];
    int st_row[3];
    unsigned char* st_ptr[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int o = i * 1024 + lane * 16;
        st_row[i] = o >= 3 * D * 2 ? 1 : 0;
        const int cb = o - st_row[i] * 3 * D * 2;            // byte within the 1536-byte row
        st_lds[i] = (uint32_t)(PS_OUT + st_row[i] * PS_OSTRIDE * 2 + cb);
        st_ptr[i] = (unsigned char*)p.out[cb / (D * 2)] + cb % (D * 2);
    }

    {
        int64_t sr[8];
        rows_of(t, sr);
        fetch(sr, 0);
        if (t + G < n_tiles) { rows_of(t + G, sr); fetch(sr, 1); }
    }
    int buf = 0;                  // ring slot of this tile; the tile two rounds ahead goes into slot buf + 2
    int round = 0;
    for (;;) {
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) __asm__ volatile("" : "+a"(wa[nt][ks]));
        const bool has_next = t + G < n_tiles, has_next2 = t + 2 * G < n_tiles;
        const int64_t r0 = p.row_begin + t * PS_ROWS;
        int64_t next_rows[8];                   // (row numbers now, the transfers once the matrix cores are busy)
        if (has_next2) rows_of(t + 2 * G, next_rows);
        // Transfers and stores complete in issue order, so "this tile's rows have landed" is
        // "at most as many operations outstanding as were issued after them": the eight
        // transfers of the next tile (if there is one) and the twelve row stores of each of
        // the last two rounds. Nothing younger has to be waited for.
        if (round == 0) { if (has_next) __builtin_amdgcn_s_waitcnt(0x0F78); else __builtin_amdgcn_s_waitcnt(0x0F70); }        // 8 | 0
        else if (round == 1) { if (has_next) __builtin_amdgcn_s_waitcnt(0x4F74); else __builtin_amdgcn_s_waitcnt(0x0F7C); }   // 20 | 12
        else { if (has_next) __builtin_amdgcn_s_waitcnt(0x8F70); else __builtin_amdgcn_s_waitcnt(0x4F78); }                   // 32 | 24
        __asm__ volatile("" ::: "memory");
        __syncthreads();          // every wave's rows have landed; the staging rows have been read

        const uint16_t (*sX)[PS_XSTRIDE] = (const uint16_t (*)[PS_XSTRIDE])(smem + buf * PS_ROWS * PS_XSTRIDE * 2);
        uint16_t (*sO)[PS_OSTRIDE] = (uint16_t (*)[PS_OSTRIDE])(smem + PS_OUT);
#pragma unroll
        for (int cg = 0; cg < 3; ++cg) {        // two column tiles at a time
            f32x16s acc[2];
            // the tile as B operand, 16 k-steps, read through a window of four fragments: each
            // is requested three steps before its two products (one wave per SIMD: nothing else
            // hides the LDS latency)
            uint4 bw[4];
#pragma unroll
            for (int ks = 0; ks < 3; ++ks) bw[ks] = *(const uint4*)&sX[n][8 * hi + ks * 16];
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) {
                if (ks + 3 < 16) bw[(ks + 3) & 3] = *(const uint4*)&sX[n][8 * hi + (ks + 3) * 16];
                const uint4 b = bw[ks & 3];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int nt = cg * 2 + j;
                    const uint4 a = nt < 4 ? __builtin_bit_cast(uint4, wa[nt < 4 ? nt : 0][ks]) : __builtin_bit_cast(uint4, wb[nt < 4 ? 0 : nt - 4][ks]);
                    if (ks == 0) {
                        f32x16s z;
#pragma unroll
                        for (int i = 0; i < 16; ++i) z[i] = 0.f;
                        acc[j] = mfma32(a, b, z);
                    } else {
                        acc[j] = mfma32(a, b, acc[j]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (cg == 0 && has_next2) fetch(next_rows, buf >= 1 ? buf - 1 : 2);
            // lane (n, hi) owns columns 192*wave + 96*hi + 32*cg .. +31 of row n
            uint4* dst = (uint4*)&sO[n][192 * wave + 96 * hi + 32 * cg];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const f32x16s c = acc[j];
                dst[2 * j] = make_uint4(pack_bf16x2(c[0], c[1]), pack_bf16x2(c[2], c[3]), pack_bf16x2(c[4], c[5]), pack_bf16x2(c[6], c[7]));
                dst[2 * j + 1] = make_uint4(pack_bf16x2(c[8], c[9]), pack_bf16x2(c[10], c[11]), pack_bf16x2(c[12], c[13]), pack_bf16x2(c[14], c[15]));
            }
        }
        __syncthreads();          // staged rows complete
        // wave w stores rows 8w .. 8w+7, two at a time
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            uint4 piece[6];
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                for (int i = 0; i < 3; ++i)
                    piece[3 * pr + i] = *(const uint4*)(smem + st_lds[i] + (8 * wave + 4 * half + 2 * pr) * PS_OSTRIDE * 2);
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const int row = 8 * wave + 4 * half + 2 * pr + st_row[i];
                    if (r0 + row < p.row_end) *(uint4*)(st_ptr[i] + (r0 + row) * p.out_stride * 2) = piece[3 * pr + i];
                }
        }
        if (!has_next) return;
        t += G;
        buf = buf == 2 ? 0 : buf + 1;
        ++round;
    }
}

}  // namespace

int dg4_launch_pack_w32(const void* w, int ld, void* packed, hipStream_t s)
{
    hipLaunchKernelGGL(pack_w32_kernel, dim3(4 * PS_NT * 16 * 64 / 256), dim3(256), 0, s, (const uint16_t*)w, ld, (uint16_t*)packed);
    return hipGetLastError();
}

int dg4_launch_bulk_proj(const dg4_bulk_args& a, hipStream_t s)
{
    const int64_t rows = a.row_end - a.row_begin;
    if (rows <= 0) return hipSuccess;
    if (a.n_cols != 3 * D) return hipErrorInvalidValue;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return hipErrorInvalidDevice;
    const int64_t tiles = (rows + PS_ROWS - 1) / PS_ROWS;
    hipError_t e = hipFuncSetAttribute((const void*)proj768_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, PS_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(proj768_kernel, dim3((unsigned)std::min<int64_t>(cus, tiles)), dim3(256), PS_BYTES, s, a);
    return hipGetLastError();
}
