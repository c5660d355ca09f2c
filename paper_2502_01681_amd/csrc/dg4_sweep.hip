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

namespace {

typedef __bf16 bf16x8s __attribute__((ext_vector_type(8)));

constexpr int TILE = DG4_TILE_ROWS;   // 16
constexpr int D = 256;
constexpr int LDS_STRIDE = D + 8;     // bf16 elements per LDS row (16 bytes of padding)

__device__ __forceinline__ f32x4 mfma16(const uint4& a, const uint4& b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8s, a), __builtin_bit_cast(bf16x8s, b), c, 0, 0, 0);
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
    if (i < 4) ctrl[i] = 0u;                      // [0] ticket, [1] abort, [2] tiles finished
}

template <int W>
__global__ __launch_bounds__(256) void sweep_kernel(dg4_sweep_args p)
{
    __shared__ __attribute__((aligned(16))) uint16_t sA[TILE][LDS_STRIDE];   // attention output, bf16
    __shared__ __attribute__((aligned(16))) uint16_t sH[TILE][LDS_STRIDE];   // new embeddings, bf16
    __shared__ float sRed[TILE][4][2];
    __shared__ int sTicket;
    __shared__ int sAbort;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int grp = lane >> 4, sub = lane & 15;
    constexpr int CH = W < 8 ? W : 8;         // neighbour rows in flight per pass

    const uint4* wo = (const uint4*)p.wo_packed;
    const uint4* wkv = (const uint4*)p.wkv_packed;

    for (;;) {
        if (threadIdx.x == 0) {
            const uint32_t aborted = __hip_atomic_load(&p.ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t t = aborted ? 0xFFFFFFFFu
                                       : __hip_atomic_fetch_add(&p.ctrl[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sTicket = t < (uint32_t)p.n_tiles ? (int)t : -1;
            sAbort = 0;
        }
        __syncthreads();
        const int ticket = sTicket;
        if (ticket < 0) return;
        const uint2 ti = p.tiles[p.tile_begin + ticket];
        const int64_t p0 = ti.x;
        const int rows = (int)ti.y;

        // ---------------- attention: gate (4*wave + grp), lane owns 16 features
        {
            const int r = 4 * wave + grp;
            const bool valid = r < rows;
            const int64_t row = p0 + (valid ? r : 0);
            const int64_t eoff = (int64_t)sub * 16;
            const int head = sub >> 1;

            uint32_t ent[W];
            {
                const uint4* e4 = (const uint4*)(p.ell + row * W);
#pragma unroll
                for (int i = 0; i < W / 4; ++i) {
                    const uint4 t = e4[i];
                    ent[4 * i] = t.x; ent[4 * i + 1] = t.y; ent[4 * i + 2] = t.z; ent[4 * i + 3] = t.w;
                }
            }
            // wait until every source of this gate is published: lane `sub` watches entry `sub`
            {
                uint32_t mine = DG4_ELL_PAD;
#pragma unroll
                for (int i = 0; i < W; ++i) if (sub == i) mine = ent[i];
                bool need = valid && mine != DG4_ELL_PAD && (mine >> 30) != 0;
                const uint32_t* f = p.flags + (mine & 0x3FFFFFFFu);
                uint32_t spins = 0;
                bool gave_up = false;
                for (;;) {
                    if (need && __hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) need = false;
                    if (!__any(need)) break;
                    __builtin_amdgcn_s_sleep(2);
                    if (++spins > p.spin_limit ||
                        ((spins & 63u) == 0 && __hip_atomic_load(&p.ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                        gave_up = true;
                        break;
                    }
                }
                if (gave_up) {
                    if (lane == 0) {
                        __hip_atomic_store(&p.ctrl[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        sAbort = 1;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            }

            float q[16];
            const uint16_t* self = p.qkv_self + row * (3 * D) + eoff;
            {
                const uint4* qp = (const uint4*)self;
                Elem<bf16_t>::unpack(qp[0], qp[1], q);
            }
            float bias[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) bias[i] = p.rel_bias[head * 4 + i];

            auto src_row = [&](uint32_t e, int which) -> const uint4* {   // which: 0 = K, 1 = V
                const uint32_t rel = e >> 30;
                const int64_t idx = e & 0x3FFFFFFFu;
                const uint16_t* b = rel == 0 ? self + (1 + which) * D
                                             : p.kv + idx * (2 * D) + which * D + eoff;
                return (const uint4*)b;
            };

            float s[W];
            const float scale = 0.17677669529663687f;     // 1/sqrt(32)
#pragma unroll
            for (int c0 = 0; c0 < W; c0 += CH) {
                uint4 ka[CH], kb[CH];
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    if (valid && ent[c0 + j] != DG4_ELL_PAD) {
                        const uint4* kp = src_row(ent[c0 + j], 0);
                        ka[j] = kp[0]; kb[j] = kp[1];
                    } else {
                        ka[j] = make_uint4(0, 0, 0, 0); kb[j] = ka[j];
                    }
                }
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    float k[16];
                    Elem<bf16_t>::unpack(ka[j], kb[j], k);
                    float dot = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) dot = fmaf(q[i], k[i], dot);
                    dot = Elem<bf16_t>::head_sum(dot);
                    const uint32_t rel = ent[c0 + j] >> 30;
                    const float b = rel == 0 ? bias[0] : rel == 1 ? bias[1] : rel == 2 ? bias[2] : bias[3];
                    s[c0 + j] = ent[c0 + j] != DG4_ELL_PAD ? fmaf(dot, scale, b) : -INFINITY;
                }
            }
            float mx = s[0];
#pragma unroll
            for (int j = 1; j < W; ++j) mx = fmaxf(mx, s[j]);
            float z = 0.f;
#pragma unroll
            for (int j = 0; j < W; ++j) { s[j] = __expf(s[j] - mx); z += s[j]; }
            const float rz = 1.0f / z;

            float acc[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
            for (int c0 = 0; c0 < W; c0 += CH) {
                uint4 va[CH], vb[CH];
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    if (valid && ent[c0 + j] != DG4_ELL_PAD) {
                        const uint4* vp = src_row(ent[c0 + j], 1);
                        va[j] = vp[0]; vb[j] = vp[1];
                    } else {
                        va[j] = make_uint4(0, 0, 0, 0); vb[j] = va[j];
                    }
                }
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    float v[16];
                    Elem<bf16_t>::unpack(va[j], vb[j], v);
                    const float al = s[c0 + j] * rz;
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] = fmaf(al, v[i], acc[i]);
                }
            }
            uint4 oa, ob;
            if (valid) Elem<bf16_t>::pack(acc, oa, ob);
            else { oa = make_uint4(0, 0, 0, 0); ob = oa; }
            uint4* dst = (uint4*)&sA[r][eoff];
            dst[0] = oa; dst[1] = ob;
        }
        __syncthreads();
        if (sAbort) return;

        // ---------------- output projection; lane (n = sub, g = grp) owns columns 64*wave + 16*g .. +15 of gate n
        const int n = sub;
        const bool nvalid = n < rows;
        const int64_t prow = p0 + (nvalid ? n : 0);
        const int64_t orig = p.order[prow];
        const int c0 = 64 * wave + 16 * grp;
        float t[16];
        {
            // residual row, issued before the matrix work
            const uint4* xp = (const uint4*)(p.x + orig * D + c0);
            const uint4 xa = xp[0], xb = xp[1];
            f32x4 acc[4];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const uint4 b = *(const uint4*)&sA[n][ks * 32 + 8 * grp];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    const uint4 a = wo[(((int64_t)wave * 4 + nt) * 8 + ks) * 64 + lane];
                    acc[nt] = mfma16(a, b, acc[nt]);
                }
            }
            float x[16];
            Elem<bf16_t>::unpack(xa, xb, x);
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int i = 0; i < 4; ++i) t[nt * 4 + i] = acc[nt][i] + (p.epilogue ? x[nt * 4 + i] : 0.f);
        }
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
                uint4* hp = (uint4*)(p.h_out + orig * D + c0);
                hp[0] = ha; hp[1] = hb;
            }
            uint4* hs = (uint4*)&sH[n][c0];
            hs[0] = ha; hs[1] = hb;
        }
        __syncthreads();

        // ---------------- K|V projection of the new embeddings: lane owns columns 128*wave + 32*g .. +31
        if (p.publish_kv) {
            f32x4 acc[8];
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) acc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const uint4 b = *(const uint4*)&sH[n][ks * 32 + 8 * grp];
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) {
                    const uint4 a = wkv[(((int64_t)wave * 8 + nt) * 8 + ks) * 64 + lane];
                    acc[nt] = mfma16(a, b, acc[nt]);
                }
            }
            if (nvalid) {
                uint4* kvp = (uint4*)(p.kv + prow * (2 * D) + 128 * wave + 32 * grp);
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const f32x4 u = acc[2 * h], v = acc[2 * h + 1];
                    kvp[h] = make_uint4(pack_bf16x2(u[0], u[1]), pack_bf16x2(u[2], u[3]),
                                        pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
                }
            }
        }
        // ---------------- publish: rows first (made visible device-wide), then the flags
        __syncthreads();
        if (wave == 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            if (lane < rows) __hip_atomic_store(&p.flags[p0 + lane], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
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
    hipLaunchKernelGGL(sweep_init_kernel, dim3((unsigned)((std::max<int64_t>(n_flags, 4) + 255) / 256)), dim3(256), 0, s,
                       a.flags, n_flags, done_below, a.ctrl);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return hipErrorInvalidDevice;
    int64_t grid = (int64_t)cus * wgs_per_cu;
    if (grid > a.n_tiles) grid = a.n_tiles;
    if (a.ell_w == 8) hipLaunchKernelGGL(sweep_kernel<8>, dim3((unsigned)grid), dim3(256), 0, s, a);
    else if (a.ell_w == 16) hipLaunchKernelGGL(sweep_kernel<16>, dim3((unsigned)grid), dim3(256), 0, s, a);
    else if (a.ell_w == 4) hipLaunchKernelGGL(sweep_kernel<4>, dim3((unsigned)grid), dim3(256), 0, s, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}
