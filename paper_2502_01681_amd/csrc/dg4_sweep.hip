// The level sweep as ONE persistent dataflow kernel (bf16, hidden 256, one layer).
//
// The updating strategy (paper Section 3.4, Algorithm 2) orders the work level
// by level; what it requires is that a gate reads the FINAL embeddings of its
// cone sources and is itself computed once. Work is cut into tiles of 16
// level-sorted gates (never across a level boundary). Resident workgroups draw
// tiles from a global ticket counter in (level, id) order; a tile spins only on
// the "finished" flags of ITS sources, so several levels are in flight at once
// while every gate still sees exactly the values the level-by-level sweep
// would give it. A workgroup waits only for lower tickets, and those are held
// by workgroups that are already running, so the wait always ends; a bounded
// spin count turns any violation into an abort flag instead of a hang.
//
// Per tile: attention over the cone rows (lanes split the feature dimension,
// softmax in registers), output projection on the matrix cores with the tile
// as the B operand (so a lane ends up owning CONTIGUOUS output columns of one
// gate), residual + LayerNorm in registers, K|V projection of the new
// embeddings, publication of the rows and of the flags.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dg4_device.h"
#include "dg4_internal.h"

#ifndef DG4_SWEEP_RESIDENT_TILES
#define DG4_SWEEP_RESIDENT_TILES 6
#endif

namespace {

typedef __bf16 bf16x8s __attribute__((ext_vector_type(8)));

constexpr int TILE = DG4_TILE_ROWS;   // 16
constexpr int D = 256;
constexpr int LDS_STRIDE = D + 8;     // bf16 elements per LDS row (16 bytes of padding)
constexpr int KV_STRIDE = 2 * D + 8;
constexpr int RES = DG4_SWEEP_RESIDENT_TILES;   // column tiles of Wk|Wv (of 8 per wave) kept in registers
constexpr int SMEM_WO = D * D * 2;                                  // 128 KB
constexpr int SMEM_TILE = 3 * TILE * LDS_STRIDE * 2;                // sA, sX (spare), sH; sKV overlays sA + sX
static_assert(TILE * KV_STRIDE * 2 <= 2 * TILE * LDS_STRIDE * 2, "sKV must fit over sA and sX");
constexpr int SMEM_BYTES = SMEM_WO + SMEM_TILE + TILE * 4 * 2 * 4 + 16;

__device__ __forceinline__ f32x4 mfma16(const uint4& a, const uint4& b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8s, a), __builtin_bit_cast(bf16x8s, b), c, 0, 0, 0);
}

// acc[nt] += W_tile(nt) x tile, for the NT column tiles of one wave. The weight fragments
// (A operand) live in REGISTERS for the whole kernel: a workgroup of four waves holds the
// complete Wo (128 registers per lane) and Wk|Wv (256 per lane), so a tile costs no weight
// traffic at all. The gate rows (B operand) come from LDS.
template <int NT>
__device__ __forceinline__ void tile_gemm(const uint4 (&w)[NT][8], const uint16_t* __restrict__ brow, f32x4 (&acc)[NT])
{
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const uint4 b = *(const uint4*)(brow + ks * 32);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = mfma16(w[nt][ks], b, acc[nt]);
    }
}
// Same with the weight fragments in LDS (`w` already offset to this wave and lane).
template <int NT>
__device__ __forceinline__ void tile_gemm_lds(const uint4* __restrict__ w, const uint16_t* __restrict__ brow, f32x4 (&acc)[NT])
{
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const uint4 b = *(const uint4*)(brow + ks * 32);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = mfma16(w[(nt * 8 + ks) * 64], b, acc[nt]);
    }
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

__global__ void sweep_init_kernel(uint32_t* flags, int64_t n, int64_t done_below, uint32_t* ctrl)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flags[i] = i < done_below ? 1u : 0u;
    if (i < 64) ctrl[i] = 0u;                     // [0] ticket, [1] abort, [16..31] phase timers
}

template <int W>
__global__ __launch_bounds__(256, 1) void sweep_kernel(dg4_sweep_args p)
{
    // LDS: Wo in A-operand order (128 KB), then three row buffers. sKV (the tile's K|V rows on
    // their way out) overlays sA and sX, both dead by then; sH stays separate so that the K|V
    // projection can read it while sKV is being written.
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint4* sWo = (uint4*)smem;                                                       // [4*4*8*64]
    uint16_t (*sA)[LDS_STRIDE] = (uint16_t (*)[LDS_STRIDE])(smem + SMEM_WO);         // attention output, bf16
    uint16_t (*sH)[LDS_STRIDE] = sA + 2 * TILE;                                      // new embeddings, bf16
    uint16_t (*sKV)[KV_STRIDE] = (uint16_t (*)[KV_STRIDE])(smem + SMEM_WO);          // K|V rows, bf16
    float (*sRed)[4][2] = (float (*)[4][2])(smem + SMEM_WO + SMEM_TILE);
    int& sAbort = *(int*)(smem + SMEM_WO + SMEM_TILE + TILE * 4 * 2 * sizeof(float));

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int grp = lane >> 4, sub = lane & 15;
    constexpr bool EARLY_K = W <= 8;          // gather the next tile's K rows during this tile's projections
    const int64_t eoff = (int64_t)sub * 16;   // attention role: this lane's 16 features of gate 4*wave+grp
    const int c0 = 64 * wave + 16 * grp;      // projection role: this lane's 16 columns of gate `sub`

    // weights, loaded once: Wo into LDS; of this wave's 8 column tiles of Wk|Wv, RES stay in
    // registers for the whole kernel, the other 8-RES are re-read from L2 once per tile (after
    // the attention phase has released its registers).
    const uint4* wkv = (const uint4*)p.wkv_packed + (int64_t)wave * 8 * 8 * 64 + lane;
    uint4 wkv_r[RES][8];
    {
        const uint4* wo = (const uint4*)p.wo_packed;
        for (int i = threadIdx.x; i < 4 * 4 * 8 * 64; i += 256) sWo[i] = wo[i];
#pragma unroll
        for (int nt = 0; nt < RES; ++nt)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) wkv_r[nt][ks] = wkv[(nt * 8 + ks) * 64];
    }
    float bias[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) bias[i] = p.rel_bias[(sub >> 1) * 4 + i];
    if (threadIdx.x == 0) sAbort = 0;

    // optional phase timers (thread 0, constant-rate clock): -, wait, attention, Wo, LN, KV, publish
    uint64_t prof[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    uint64_t tick = p.prof ? wall_clock64() : 0;
    auto lap = [&](int phase) {
        if (p.prof && threadIdx.x == 0) { const uint64_t now = wall_clock64(); prof[phase] += now - tick; tick = now; }
    };
    auto flush = [&]() {
        if (p.prof && threadIdx.x == 0)
            for (int i = 0; i < 8; ++i) atomicAdd((unsigned long long*)&p.prof[i], (unsigned long long)prof[i]);
    };

    // Inputs of a tile that do not depend on other tiles travel ahead of it: the descriptor and
    // the neighbour row of "my" gate (attention role: gate 4*wave + grp) two tiles ahead, the
    // projected self rows of that gate and the residual row of gate `sub` (projection role) one
    // tile ahead.
    struct Desc { int64_t p0; int rows; uint32_t ent[W]; };
    struct Self { uint4 q0, q1, x0, x1; int64_t orig; };
    auto fetch_desc = [&](int64_t t, Desc& d) __attribute__((always_inline)) {
        const uint2 ti = p.tiles[p.tile_begin + t];
        d.p0 = ti.x; d.rows = (int)ti.y;
        const int r = 4 * wave + grp;
        const uint4* e4 = (const uint4*)(p.ell + (d.p0 + (r < d.rows ? r : 0)) * W);
#pragma unroll
        for (int i = 0; i < W / 4; ++i) {
            const uint4 v = e4[i];
            d.ent[4 * i] = v.x; d.ent[4 * i + 1] = v.y; d.ent[4 * i + 2] = v.z; d.ent[4 * i + 3] = v.w;
        }
    };
    auto fetch_self = [&](const Desc& d, Self& f) __attribute__((always_inline)) {
        const int r = 4 * wave + grp;
        const uint4* sp = (const uint4*)(p.qkv_self + (d.p0 + (r < d.rows ? r : 0)) * (3 * D) + eoff);
        f.q0 = sp[0]; f.q1 = sp[1];
        f.orig = p.order[d.p0 + (sub < d.rows ? sub : 0)];
        const uint4* xp = (const uint4*)(p.x + f.orig * D + c0);
        f.x0 = xp[0]; f.x1 = xp[1];
    };
    // One look at the flags of my gate's sources (lane `sub` watches entry `sub`): true if some
    // source of one of this wave's four gates is not published yet.
    auto pending = [&](const Desc& d) __attribute__((always_inline)) -> bool {
        uint32_t mine = DG4_ELL_PAD;
#pragma unroll
        for (int i = 0; i < W; ++i) if (sub == i) mine = d.ent[i];
        const bool need = 4 * wave + grp < d.rows && mine != DG4_ELL_PAD && (mine >> 30) != 0;
        const bool wait = need && __hip_atomic_load(p.flags + (mine & 0x3FFFFFFFu), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u;
        const bool any = __any(wait);
        // No cache invalidation is needed once a flag is seen: a K|V row is written once per
        // sweep, through to device memory, before its flag; nobody reads it earlier, so no cache
        // of this compute unit or its L2 can hold an older copy. The fence only keeps the
        // compiler from moving row loads above the flag loads.
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        return any;
    };
    // K (which = 0) or V (1) rows of my gate's sources. The gate itself reads the projection of
    // its own x; padding slots read that row too (their weight is zero) so every lane always
    // loads from a valid address.
    auto gather = [&](const Desc& d, int which, uint4 (&ra)[W], uint4 (&rb)[W]) __attribute__((always_inline)) {
        const int r = 4 * wave + grp;
        const uint16_t* self = p.qkv_self + (d.p0 + (r < d.rows ? r : 0)) * (3 * D) + (1 + which) * D + eoff;
#pragma unroll
        for (int j = 0; j < W; ++j) {
            const uint32_t e = d.ent[j];
            const bool src = r < d.rows && e != DG4_ELL_PAD && (e >> 30) != 0;
            const uint4* rp = (const uint4*)(src ? p.kv + (int64_t)(e & 0x3FFFFFFFu) * (2 * D) + which * D + eoff : self);
            ra[j] = rp[0]; rb[j] = rp[1];
        }
    };

    // Tiles are dealt round-robin: workgroup b owns tiles b, b + G, b + 2G, ... (G = grid size,
    // one workgroup per compute unit, so all of them are resident together). A tile waits only
    // for lower-numbered tiles, each owned by a workgroup that is running.
    const int64_t G = gridDim.x;
    int64_t ticket = blockIdx.x;
    if (ticket >= p.n_tiles) return;
    Desc cur, nxt;
    Self cself, nself;
    // (tickets past the end are clamped: the fetch is harmless and its result unused)
    const int64_t last = p.n_tiles - 1;
    fetch_desc(ticket, cur);
    fetch_desc(ticket + G < last ? ticket + G : last, nxt);
    fetch_self(cur, cself);
    uint4 ka[W], kb[W];                           // K rows of the tile about to be attended
    bool k_ready = false;                         // ... already gathered (early, during the previous tile)
    __syncthreads();                              // sWo, sAbort

    for (;;) {
        const int64_t p0 = cur.p0;
        const int rows = cur.rows;
        const bool has_next = ticket + G < p.n_tiles;

        // ---------------- attention: gate (4*wave + grp), lane owns 16 features
        {
            const int r = 4 * wave + grp;
            const bool valid = r < rows;
            if (!k_ready) {
                // wait until every source of this wave's gates is published
                uint32_t spins = 0;
                while (pending(cur)) {
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
                gather(cur, 0, ka, kb);
            }
            if (p.prof) __syncthreads();      // timers only: charge every wave's wait to phase 1
            lap(1);
            uint4 va[W], vb[W];
            gather(cur, 1, va, vb);

            float q[16];
            Elem<bf16_t>::unpack(cself.q0, cself.q1, q);
            const float scale = 0.17677669529663687f;     // 1/sqrt(32)
            float s[W];
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < W; ++j) {
                float k[16];
                Elem<bf16_t>::unpack(ka[j], kb[j], k);
                float dot = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) dot = fmaf(q[i], k[i], dot);
                dot = Elem<bf16_t>::head_sum(dot);
                const uint32_t rel = cur.ent[j] >> 30;
                const float b = rel == 0 ? bias[0] : rel == 1 ? bias[1] : rel == 2 ? bias[2] : bias[3];
                s[j] = cur.ent[j] != DG4_ELL_PAD ? fmaf(dot, scale, b) : -INFINITY;
                mx = fmaxf(mx, s[j]);
            }
            float z = 0.f;
#pragma unroll
            for (int j = 0; j < W; ++j) { s[j] = __expf(s[j] - mx); z += s[j]; }
            const float rz = 1.0f / z;
            float acc[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
            for (int j = 0; j < W; ++j) {
                float v[16];
                Elem<bf16_t>::unpack(va[j], vb[j], v);
                const float al = s[j] * rz;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = fmaf(al, v[i], acc[i]);
            }
            uint4 oa, ob;
            if (valid) Elem<bf16_t>::pack(acc, oa, ob);
            else { oa = make_uint4(0, 0, 0, 0); ob = oa; }
            uint4* dst = (uint4*)&sA[r][eoff];
            dst[0] = oa; dst[1] = ob;
        }
        // ---------------- while this tile goes through its projections: the non-resident weight
        // tiles, the next tile's self rows, a first look at its flags and, if they are all up,
        // its K rows (gathered early, they overlap with the matrix work below)
        __builtin_amdgcn_sched_barrier(0);
        uint4 wkv_s[8 - RES][8];
#pragma unroll
        for (int nt = RES; nt < 8; ++nt)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) wkv_s[nt - RES][ks] = wkv[(nt * 8 + ks) * 64];
        fetch_self(nxt, nself);
        k_ready = EARLY_K && has_next && !pending(nxt);
        if (k_ready) gather(nxt, 0, ka, kb);
        Desc nn;
        fetch_desc(ticket + 2 * G < last ? ticket + 2 * G : last, nn);
        __syncthreads();
        if (sAbort) { flush(); return; }
        lap(2);

        // ---------------- output projection; lane (n = sub, g = grp) owns columns 64*wave + 16*g .. +15 of gate n
        const int n = sub;
        const bool nvalid = n < rows;
        float t[16];
        {
            f32x4 acc[4];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
            tile_gemm_lds<4>(sWo + wave * 4 * 8 * 64 + lane, &sA[n][8 * grp], acc);
            float x[16];
            Elem<bf16_t>::unpack(cself.x0, cself.x1, x);
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int i = 0; i < 4; ++i) t[nt * 4 + i] = acc[nt][i] + (p.epilogue ? x[nt * 4 + i] : 0.f);
        }
        lap(3);
        if (p.epilogue) {
            float s1 = 0.f, s2 = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s1 += t[i]; s2 = fmaf(t[i], t[i], s2); }
            s1 += __shfl_xor(s1, 16); s2 += __shfl_xor(s2, 16);
            s1 += __shfl_xor(s1, 32); s2 += __shfl_xor(s2, 32);
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
        {
            uint4 ha, hb;
            Elem<bf16_t>::pack(t, ha, hb);
            if (nvalid) {
                uint4* hp = (uint4*)(p.h_out + cself.orig * D + c0);
                hp[0] = ha; hp[1] = hb;
            }
            uint4* hs = (uint4*)&sH[n][c0];
            hs[0] = ha; hs[1] = hb;
        }
        __syncthreads();
        lap(4);

        // ---------------- K|V projection of the new embeddings: lane owns columns 128*wave + 32*g .. +31
        {
            f32x4 acc[8];
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) acc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const uint4 b = *(const uint4*)&sH[n][8 * grp + ks * 32];
#pragma unroll
                for (int nt = 0; nt < RES; ++nt) acc[nt] = mfma16(wkv_r[nt][ks], b, acc[nt]);
#pragma unroll
                for (int nt = RES; nt < 8; ++nt) acc[nt] = mfma16(wkv_s[nt - RES][ks], b, acc[nt]);
            }
            uint4* dst = (uint4*)&sKV[n][128 * wave + 32 * grp];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const f32x4 u = acc[2 * h], v = acc[2 * h + 1];
                dst[h] = make_uint4(pack_bf16x2(u[0], u[1]), pack_bf16x2(u[2], u[3]),
                                    pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
            }
            __syncthreads();
            // wave w writes rows 4w..4w+3, 512 contiguous bytes per instruction. Device-scope
            // stores: written through the L2 of this XCD; complete = visible to every compute unit.
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = 4 * wave + rr;
                if (r < rows) {
                    uint64_t* gp = (uint64_t*)(p.kv + (p0 + r) * (2 * D));
                    const uint64_t* lp = (const uint64_t*)&sKV[r][0];
                    __hip_atomic_store(gp + lane, lp[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(gp + 64 + lane, lp[64 + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        // ---------------- publish: every wave first waits until its own row stores have completed
        // (vmcnt(0); the barrier alone does not wait for global stores), then the flags go out
        __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0), expcnt and lgkmcnt untouched
        __syncthreads();
        lap(5);
        if (wave == 0 && lane < rows)
            __hip_atomic_store(&p.flags[p0 + lane], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lap(6);

        if (!has_next) { flush(); return; }
        ticket += G;
        cur.p0 = nxt.p0; cur.rows = nxt.rows; nxt.p0 = nn.p0; nxt.rows = nn.rows;
#pragma unroll
        for (int i = 0; i < W; ++i) { cur.ent[i] = nxt.ent[i]; nxt.ent[i] = nn.ent[i]; }
        cself.q0 = nself.q0; cself.q1 = nself.q1; cself.x0 = nself.x0; cself.x1 = nself.x1;
        cself.orig = nself.orig;
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

int dg4_launch_sweep(const dg4_sweep_args& a, int64_t n_flags, int64_t done_below, int wgs_per_cu, hipStream_t s)
{
    if (a.n_tiles <= 0) return hipSuccess;
    hipLaunchKernelGGL(sweep_init_kernel, dim3((unsigned)((std::max<int64_t>(n_flags, 64) + 255) / 256)), dim3(256), 0, s,
                       a.flags, n_flags, done_below, a.ctrl);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return hipErrorInvalidDevice;
    (void)wgs_per_cu;                  // one workgroup per compute unit: its registers and LDS hold the weights
    int64_t grid = cus;
    if (grid > a.n_tiles) grid = a.n_tiles;
    void (*kern)(dg4_sweep_args) = a.ell_w == 8 ? sweep_kernel<8> : a.ell_w == 16 ? sweep_kernel<16>
                                  : a.ell_w == 4 ? sweep_kernel<4> : nullptr;
    if (!kern) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), SMEM_BYTES, s, a);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------------
// Bulk projection (bf16, hidden 256): out[r, :] = S[idx(r), :] x W for many rows at once, e.g.
// Q | K | V of x for every gate before the sweep, or dg4_qkv_proj. HBM-bound (512 B in, 1.5 KB
// out per row), so the aim is full-width rows in and out with the matrix cores kept fed:
// a wave owns 64 rows (two 32-row B operands held in registers for all of K = 256) and walks
// over the output columns two 32-column tiles at a time; the weight tiles (A operand) stream
// from L2 and are each used for both row blocks. With the rows as B operand a lane ends up with
// 32 CONTIGUOUS output columns of one row per tile pair (64-byte stores).
namespace {

typedef float f32x16s __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f32x16s mfma32(const uint4& a, const uint4& b, f32x16s c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8s, a), __builtin_bit_cast(bf16x8s, b), c, 0, 0, 0);
}

// Packed order, 16-byte units: unit ((tile*16 + ks)*64 + lane) holds rows k = ks*16 + 8*(lane/32) .. +7
// of column  col0 + (tile/2)*64 + g*32 + (tile%2)*16 + a*4 + b,  where m = lane%32 = 8a + 4g + b.
__global__ void pack_w32_kernel(const uint16_t* w, int ld, int col0, int n_cols, uint16_t* packed)
{
    const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t units = (int64_t)(n_cols / 32) * 16 * 64;
    if (unit >= units) return;
    const int lane = (int)(unit & 63);
    const int ks = (int)((unit >> 6) & 15);
    const int tile = (int)(unit >> 10);
    const int m = lane & 31;
    const int a = m >> 3, g = (m >> 2) & 1, b = m & 3;
    const int col = col0 + (tile >> 1) * 64 + g * 32 + (tile & 1) * 16 + a * 4 + b;
    const int k0 = ks * 16 + 8 * (lane >> 5);
#pragma unroll
    for (int j = 0; j < 8; ++j) packed[unit * 8 + j] = w[(int64_t)(k0 + j) * ld + col];
}

__global__ __launch_bounds__(256, 2) void bulk_proj_kernel(dg4_bulk_args p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int n = lane & 31, g = lane >> 5;
    const int64_t r0 = p.row_begin + ((int64_t)blockIdx.x * 4 + wave) * 64;
    if (r0 >= p.row_end) return;

    // the two 32-row blocks of this wave as B operands for all 16 k-steps
    uint4 act[2][16];
    int64_t orow[2];
    bool ok[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        int64_t r = r0 + rb * 32 + n;
        ok[rb] = r < p.row_end;
        if (!ok[rb]) r = p.row_end - 1;                  // clamp: loads stay in bounds, stores are masked
        orow[rb] = r;
        const int64_t sr = p.gather ? (int64_t)p.gather[r] : r;
        const uint4* sp = (const uint4*)(p.src + sr * D);
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) act[rb][ks] = sp[ks * 2 + g];
    }
    const uint4* wp = (const uint4*)p.w_packed + lane;
    const int n_pairs = p.n_cols / 64;
    for (int pr = 0; pr < n_pairs; ++pr) {
        f32x16s acc[2][2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[rb][t][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) {
            const uint4 w0 = wp[((int64_t)(2 * pr) * 16 + ks) * 64];
            const uint4 w1 = wp[((int64_t)(2 * pr + 1) * 16 + ks) * 64];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                acc[rb][0] = mfma32(w0, act[rb][ks], acc[rb][0]);
                acc[rb][1] = mfma32(w1, act[rb][ks], acc[rb][1]);
            }
        }
        // lane (n, g): columns pr*64 + g*32 + t*16 + a*4 + b  <-  acc[rb][t][4a + b]
        const int col = pr * 64 + g * 32;
        uint16_t* base = p.out[col / D] + (col % D);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            if (!ok[rb]) continue;
            uint4* op = (uint4*)(base + orow[rb] * p.out_stride);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const f32x16s c = acc[rb][t];
                op[2 * t] = make_uint4(pack_bf16x2(c[0], c[1]), pack_bf16x2(c[2], c[3]), pack_bf16x2(c[4], c[5]), pack_bf16x2(c[6], c[7]));
                op[2 * t + 1] = make_uint4(pack_bf16x2(c[8], c[9]), pack_bf16x2(c[10], c[11]), pack_bf16x2(c[12], c[13]), pack_bf16x2(c[14], c[15]));
            }
        }
    }
}

}  // namespace

int dg4_launch_pack_w32(const void* w, int ld, int col0, int n_cols, void* packed, hipStream_t s)
{
    const int64_t units = (int64_t)(n_cols / 32) * 16 * 64;
    hipLaunchKernelGGL(pack_w32_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s,
                       (const uint16_t*)w, ld, col0, n_cols, (uint16_t*)packed);
    return hipGetLastError();
}

int dg4_launch_bulk_proj(const dg4_bulk_args& a, hipStream_t s)
{
    const int64_t rows = a.row_end - a.row_begin;
    if (rows <= 0) return hipSuccess;
    if (a.n_cols % 64) return hipErrorInvalidValue;
    hipLaunchKernelGGL(bulk_proj_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, s, a);
    return hipGetLastError();
}
