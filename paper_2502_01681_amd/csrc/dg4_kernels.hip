// Device kernels for gfx950 (MI355X, wave64) and their launchers.
//
//  attn_kernel   scores + segmented softmax + aggregation over cone rows
//                (Section 3.5; single-source rows get alpha = 1, Section 3.7).
//                HBM-bound gather: lanes split the FEATURE dimension of a row,
//                the <= 15 neighbours are looped over in registers, so the
//                softmax needs no cross-lane traffic and no score tensor exists.
//  pack_w_kernel re-tiles a row-major weight into MFMA B-operand order.
//  gemm_kernel   rows x packed weight on the matrix cores (the dense
//                projections), optionally fused with residual + LayerNorm.
//  ffn_kernel    the position-wise feed-forward sub-block of the transformer
//                layer (Section 3.5), both products, rectifier, residual and
//                LayerNorm in one pass; the 4d hidden activations never leave
//                the registers.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dg4_device.h"
#include "dg4_internal.h"
#include "dg4_rowops.h"

namespace {

// ------------------------------------------------------------------ attention

// One destination row per group of LPR lanes.
template <typename T, int D, int W>
__global__ __launch_bounds__(256) void attn_kernel(dg4_attn_args p)
{
    constexpr int EPL = Elem<T>::EPL;
    constexpr int LPR = D / EPL;              // lanes per row
    constexpr int RPW = 64 / LPR;             // rows per wave
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int sub = lane % LPR;
    const int64_t row = p.row_begin + ((int64_t)blockIdx.x * 4 + wave) * RPW + lane / LPR;
    if (row >= p.row_end) return;             // whole lane groups leave together
    float acc[EPL];
    attend_row<T, D, W>(p, row, sub, acc);
    uint4 oa, ob;
    Elem<T>::pack(acc, oa, ob);
    uint4* op = (uint4*)((T*)p.a + row * p.a_stride + (int64_t)sub * EPL);
    op[0] = oa; op[1] = ob;
}

// The same for rows of any width (cones deeper than three hops, up to 2^(k+1)-1 sources). S lane
// groups share a row: group `part` walks the chunks of CH entries part, part + S, ... with a
// running maximum, denominator and weighted sum (the softmax is unchanged by the rescaling), and
// the S partial results are merged through LDS by the first group. Long rows of few gates per
// level thus keep many loads in flight. Rows are padded at the end only, to a multiple of four.
template <typename T, int D, int S>
__global__ __launch_bounds__(256) void attn_wide_kernel(const dg4_attn_args p)
{
    constexpr int EPL = Elem<T>::EPL;
    constexpr int LPR = D / EPL;              // lanes per lane group
    constexpr int G = 256 / LPR;              // lane groups per workgroup
    constexpr int RPB = G / S;                // rows per workgroup
    constexpr int CH = S == G ? 8 : 4;        // sources per step (a whole workgroup per row: few steps, more loads in flight)
    static_assert(G % S == 0, "lane groups per row must divide the workgroup");
    __shared__ float part_m[S > 1 ? 256 : 1], part_z[S > 1 ? 256 : 1], part_acc[S > 1 ? 256 * EPL : 1];
    const int group = threadIdx.x / LPR;
    const int sub = threadIdx.x % LPR;
    const int part = group % S;
    const int64_t row = p.row_begin + (int64_t)blockIdx.x * RPB + group / S;
    const bool active = row < p.row_end;

    const int64_t eoff = (int64_t)sub * EPL;
    const int head = (int)(eoff >> 5);
    float m = -INFINITY, z = 0.f;
    float acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;
    if (active) {
        float q[EPL];
        {
            const uint4* qp = (const uint4*)((const T*)p.q + row * p.q_stride + eoff);
            Elem<T>::unpack(qp[0], qp[1], q);
        }
        float bias[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) bias[i] = p.rel_bias[head * 4 + i];
        const float scale = 0.17677669529663687f;     // 1/sqrt(32)
        const uint32_t* erow = p.ell + row * (int64_t)p.ell_w;
        // the CH entries at c0 (padding past the table: its width is a multiple of four, not of eight)
        auto entries = [&](int c0, uint32_t (&e)[CH]) __attribute__((always_inline)) {
#pragma unroll
            for (int q = 0; q < CH; q += 4) {
                const uint4 e4 = c0 + q < p.ell_w ? *(const uint4*)(erow + c0 + q) : make_uint4(DG4_ELL_PAD, DG4_ELL_PAD, DG4_ELL_PAD, DG4_ELL_PAD);
                e[q] = e4.x; e[q + 1] = e4.y; e[q + 2] = e4.z; e[q + 3] = e4.w;
            }
        };
        uint32_t ent[CH], ahead[CH];
        entries(part * CH, ent);
        for (int c0 = part * CH; c0 < p.ell_w; c0 += S * CH) {
            if (ent[0] == DG4_ELL_PAD) break;         // the same for all lanes of the group
            uint4 ka[CH], kb[CH], va[CH], vb[CH];
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                if (ent[j] != DG4_ELL_PAD) {
                    const uint32_t rel = ent[j] >> 30;
                    const int64_t idx = ent[j] & 0x3FFFFFFFu;
                    const T* kr = rel == 0 ? (const T*)p.k_self + row * p.self_stride : (const T*)p.k_src + idx * p.src_stride;
                    const T* vr = rel == 0 ? (const T*)p.v_self + row * p.self_stride : (const T*)p.v_src + idx * p.src_stride;
                    const uint4* kp = (const uint4*)(kr + eoff);
                    const uint4* vp = (const uint4*)(vr + eoff);
                    ka[j] = kp[0]; kb[j] = kp[1]; va[j] = vp[0]; vb[j] = vp[1];
                } else {
                    ka[j] = make_uint4(0, 0, 0, 0); kb[j] = ka[j]; va[j] = ka[j]; vb[j] = ka[j];
                }
            }
            entries(c0 + S * CH, ahead);              // the next step's entries travel with this step's rows
            float sc[CH];
            float cm = m;
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                float k[EPL];
                Elem<T>::unpack(ka[j], kb[j], k);
                float dot = 0.f;
#pragma unroll
                for (int i = 0; i < EPL; ++i) dot = fmaf(q[i], k[i], dot);
                dot = Elem<T>::head_sum(dot);
                const uint32_t rel = ent[j] >> 30;
                const float b = rel == 0 ? bias[0] : rel == 1 ? bias[1] : rel == 2 ? bias[2] : bias[3];
                sc[j] = ent[j] != DG4_ELL_PAD ? fmaf(dot, scale, b) : -INFINITY;
                cm = fmaxf(cm, sc[j]);
            }
            const float corr = __expf(m - cm);        // 0 on the first chunk (m = -inf, cm finite)
            z *= corr;
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] *= corr;
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                float v[EPL];
                Elem<T>::unpack(va[j], vb[j], v);
                const float pj = __expf(sc[j] - cm);  // 0 for padding
                z += pj;
#pragma unroll
                for (int i = 0; i < EPL; ++i) acc[i] = fmaf(pj, v[i], acc[i]);
            }
            m = cm;
#pragma unroll
            for (int j = 0; j < CH; ++j) ent[j] = ahead[j];
        }
    }
    if (S > 1) {
        part_m[threadIdx.x] = m; part_z[threadIdx.x] = z;
#pragma unroll
        for (int i = 0; i < EPL; ++i) part_acc[i * 256 + threadIdx.x] = acc[i];
        __syncthreads();
        if (!active || part != 0) return;
        // group 0 of the row holds the row's first chunk, so its maximum is finite
        float mm = m;
#pragma unroll
        for (int s = 1; s < S; ++s) mm = fmaxf(mm, part_m[threadIdx.x + s * LPR]);
        const float c0 = __expf(m - mm);
        z *= c0;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] *= c0;
#pragma unroll
        for (int s = 1; s < S; ++s) {
            const int t = threadIdx.x + s * LPR;
            const float cs = __expf(part_m[t] - mm);  // 0 for a part that saw no entry
            z = fmaf(part_z[t], cs, z);
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] = fmaf(part_acc[i * 256 + t], cs, acc[i]);
        }
    } else if (!active) {
        return;
    }
    const float rz = 1.0f / z;
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] *= rz;
    uint4 oa, ob;
    Elem<T>::pack(acc, oa, ob);
    uint4* op = (uint4*)((T*)p.a + row * p.a_stride + eoff);
    op[0] = oa; op[1] = ob;
}

template <typename T, int D>
int launch_attn_w(const dg4_attn_args& a, hipStream_t s)
{
    constexpr int RPB = 4 * (64 / (D / Elem<T>::EPL));     // rows per block
    const int64_t rows = a.row_end - a.row_begin;
    if (rows <= 0) return hipSuccess;
    const unsigned grid = (unsigned)((rows + RPB - 1) / RPB);
    switch (a.ell_w) {
    case 4: hipLaunchKernelGGL((attn_kernel<T, D, 4>), dim3(grid), dim3(256), 0, s, a); break;
    case 8: hipLaunchKernelGGL((attn_kernel<T, D, 8>), dim3(grid), dim3(256), 0, s, a); break;
    case 16: hipLaunchKernelGGL((attn_kernel<T, D, 16>), dim3(grid), dim3(256), 0, s, a); break;
    default: {
        // the split depends on the table's width alone, so a row's result does not depend on the
        // range of rows a call covers
        if (a.ell_w < 4 || a.ell_w % 4) return hipErrorInvalidValue;
        constexpr int G = 256 / (D / Elem<T>::EPL);
        if (a.ell_w > 64)
            hipLaunchKernelGGL((attn_wide_kernel<T, D, G>), dim3((unsigned)rows), dim3(256), 0, s, a);
        else
            hipLaunchKernelGGL((attn_wide_kernel<T, D, 4>), dim3((unsigned)((rows + G / 4 - 1) / (G / 4))), dim3(256), 0, s, a);
        break;
    }
    }
    return hipGetLastError();
}

// ------------------------------------------------------------- weight packing

// Packed order, in 16-byte units: unit ((nt*KC + c)*64 + lane) holds, for
// column n = nt*32 + lane%32 and half kg = lane/32, the E consecutive rows
// k = (2c + kg)*E .. +E-1 (E = 8 bf16 or 4 floats): exactly what one lane
// feeds to the B operand of a 32x32 MFMA for K-chunk c.
template <typename T>
__global__ void pack_w_kernel(const T* w, int ld, int col0, int n_cols, int k_dim, T* packed)
{
    constexpr int E = 16 / sizeof(T);
    const int KC = k_dim / (2 * E);
    const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t units = (int64_t)(n_cols / 32) * KC * 64;
    if (unit >= units) return;
    const int lane = (int)(unit & 63);
    const int c = (int)((unit >> 6) % KC);
    const int nt = (int)((unit >> 6) / KC);
    const int n = col0 + nt * 32 + (lane & 31);
    const int k0 = (2 * c + (lane >> 5)) * E;
#pragma unroll
    for (int j = 0; j < E; ++j) packed[unit * E + j] = w[(int64_t)(k0 + j) * ld + n];
}

// ----------------------------------------------------------------------- GEMM

// One wave = 32 rows x all output columns. The wave keeps its 32 x D slice of
// the A operand in registers and streams the packed weight tiles.
// Accumulator element i of a lane sits at row 8*(i/4) + 4*(lane/32) + i%4,
// column lane%32 of the 32x32 tile.
template <typename T, int D, bool LN>
__global__ __launch_bounds__(256) void gemm_kernel(dg4_gemm_args p)
{
    constexpr int E = 16 / sizeof(T);
    constexpr int KC = D / (2 * E);
    constexpr int NT_LN = D / 32;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int m = lane & 31, kg = lane >> 5;
    // Either every wave takes its own 32 rows and all columns, or (split: wide outputs, few rows,
    // as in a level of the sweep) the four waves of a workgroup share 32 rows and take a quarter
    // of the columns each, which puts four times as many compute units to work.
    const bool split = !LN && p.split != 0;
    const int64_t r0 = p.row_begin + (split ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * 4 + wave) * 32;
    constexpr int TS = 32 + E;                    // row stride of a staged 32x32 tile
    constexpr int TPR = 32 / E;                   // 16-byte pieces per row of a tile
    __shared__ __attribute__((aligned(16))) T tile[LN ? 1 : 4][LN ? 1 : 32 * TS];
    if (r0 >= p.row_end) return;

    uint4 a[KC];
    {
        int64_t r = r0 + m;
        if (r >= p.row_end) r = p.row_end - 1;          // clamp: loads stay in bounds, stores are masked
        const int64_t ar = p.a_gather ? (int64_t)p.a_gather[r] : r;
        const uint4* ap = (const uint4*)((const T*)p.a + ar * p.a_stride);
#pragma unroll
        for (int c = 0; c < KC; ++c) a[c] = ap[2 * c + kg];
    }
    const uint4* wp = (const uint4*)p.w_packed;

    // rows this lane's accumulator elements belong to
    int64_t orow[16];
    bool ok[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t r = r0 + 8 * (i / 4) + 4 * kg + (i % 4);
        ok[i] = r < p.row_end;
        orow[i] = ok[i] ? r : p.row_end - 1;
    }

    // The packed weight is one linear stream of 16-byte-per-lane fragments (tile nt, chunk c at
    // nt*KC + c). It is read through a ring of RING fragments requested RING products ahead:
    // with 32 rows per wave a level's kernel has few waves, and each would otherwise wait out
    // the full memory latency once per fragment. Fragments are handled in groups of GROUP (a
    // multiple of both RING and KC), so that every register index below is a compile-time constant.
    constexpr int RING = 16;
    constexpr int GROUP = KC > RING ? KC : RING;
    constexpr int TPG = GROUP / KC;               // column tiles per group
    uint4 ring[RING];
    const int64_t all = (int64_t)(p.n_cols / 32) * KC;
    // this wave's part of the stream: a multiple of GROUP fragments (checked by the launcher)
    const int64_t first = split ? wave * (all / 4) : 0;
    const int64_t total = split ? first + all / 4 : all;
#pragma unroll
    for (int j = 0; j < RING; ++j) ring[j] = wp[(first + j) * 64 + lane];

    if constexpr (!LN) {
        for (int64_t f0 = first; f0 < total; f0 += GROUP) {
            f32x16 acc;
#pragma unroll
            for (int j = 0; j < GROUP; ++j) {
                const int c = j % KC;
                if (c == 0) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
                }
                Mma<T>::run(a[c], ring[j % RING], acc);
                if (f0 + j + RING < total) ring[j % RING] = wp[(f0 + j + RING) * 64 + lane];
                if (c == KC - 1) {
                    // the 32x32 tile leaves through this wave's own corner of LDS, as 16-byte pieces
                    // of rows (LDS operations of a wave complete in order: no barrier)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        Elem<T>::store1(tile[wave], (int64_t)(8 * (i / 4) + 4 * kg + (i % 4)) * TS + m, acc[i]);
                    const int col = (int)(f0 / KC + j / KC) * 32;
                    T* base = (T*)p.out[col / D] + col % D;
#pragma unroll
                    for (int q = 0; q < 32 * TPR / 64; ++q) {
                        const int piece = lane + 64 * q, row = piece / TPR, cc = piece % TPR;
                        const uint4 v = *(const uint4*)&tile[wave][row * TS + cc * E];
                        const int64_t r = r0 + row;
                        if (r < p.row_end) {
                            const int64_t orr = p.out_scatter ? (int64_t)p.out_scatter[r] : r;
                            *(uint4*)(base + orr * p.out_stride + cc * E) = v;
                            if (p.out2) *(uint4*)((T*)p.out2 + r * p.out2_stride + col + cc * E) = v;
                        }
                    }
                }
            }
        }
    } else {
        f32x16 acc[NT_LN];
        static_assert(NT_LN % TPG == 0, "whole groups");
#pragma unroll
        for (int g = 0; g < NT_LN / TPG; ++g) {
#pragma unroll
            for (int j = 0; j < GROUP; ++j) {
                const int c = j % KC, nt = g * TPG + j / KC;
                if (c == 0) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[nt][i] = 0.f;
                }
                Mma<T>::run(a[c], ring[j % RING], acc[nt]);
                if (g * GROUP + j + RING < NT_LN * KC) ring[j % RING] = wp[(int64_t)(g * GROUP + j + RING) * 64 + lane];
            }
        }
        // residual, then LayerNorm over each row (no affine, biased variance)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t rr = p.resid_gather ? (int64_t)p.resid_gather[orow[i]] : orow[i];
            float s1 = 0.f;
#pragma unroll
            for (int nt = 0; nt < NT_LN; ++nt) {
                acc[nt][i] += Elem<T>::load1(p.resid, rr * p.resid_stride + nt * 32 + m);
                s1 += acc[nt][i];
            }
            const float mean = sum_over_32_lanes(s1) * (1.0f / D);
            float s2 = 0.f;
#pragma unroll
            for (int nt = 0; nt < NT_LN; ++nt) { const float t = acc[nt][i] - mean; s2 = fmaf(t, t, s2); }
            const float rstd = rsqrtf(sum_over_32_lanes(s2) * (1.0f / D) + p.ln_eps);
            if (!ok[i]) continue;
            const int64_t orr = p.out_scatter ? (int64_t)p.out_scatter[orow[i]] : orow[i];
#pragma unroll
            for (int nt = 0; nt < NT_LN; ++nt) {
                const float y = (acc[nt][i] - mean) * rstd;
                Elem<T>::store1(p.out[0], orr * p.out_stride + nt * 32 + m, y);
                if (p.out2) Elem<T>::store1(p.out2, orow[i] * p.out2_stride + nt * 32 + m, y);
            }
        }
    }
}

// gemm_kernel<.., LN = true> for launches with few rows: the four waves of a workgroup share 32 rows
// and take a quarter of the D output columns each (four times as many compute units at work, a
// quarter of the weight stream per wave); the LayerNorm sums are completed through LDS.
// KV: the normalised rows also go, rounded to T, through LDS into a second product with the packed
// [D, 2D] weight p.kv_w_packed, each wave taking a quarter of its 2D columns (the K | V rows of the
// gates of a one-layer sweep, otherwise a launch of their own).
// AW > 0: the rows' operand is not read from memory but computed here, the attention of the 32
// rows over neighbour rows of width AW (attend_row, two or four rows per lane group, through LDS
// into the operand layout): attention, output projection, LayerNorm and K | V in one launch.
template <typename T, int D, bool KV, int AW>
__global__ __launch_bounds__(256) void gemm_ln_split_kernel(dg4_gemm_args p, dg4_attn_args t)
{
    constexpr int E = 16 / sizeof(T);
    constexpr int KC = D / (2 * E);
    constexpr int NTW = D / 32 / 4;               // column tiles per wave
    constexpr int RING = 16;
    constexpr int GROUP = KC > RING ? KC : RING;
    static_assert((NTW * KC) % GROUP == 0, "whole groups per wave");
    __shared__ float part[2][4][32];
    // The 32 rows of the workgroup pass through LDS twice, as whole 16-byte pieces on the global
    // side: first the residual rows (in), then the normalised rows (out, and the operand of the K | V
    // product). Element-wise traffic of the accumulator layout (2 or 4 bytes per lane and access)
    // stays inside LDS.
    constexpr int YS = D + E;                     // row stride: 16 bytes of padding
    constexpr int CPR = D / E;                    // 16-byte pieces per row
    constexpr int PPT = 32 * CPR / 256;           // pieces per thread
    __shared__ __attribute__((aligned(16))) T ybuf[32 * YS];
    constexpr int TS = 32 + E;                    // row stride of a staged 32x32 tile
    constexpr int TPR = 32 / E;                   // 16-byte pieces per row of a tile
    __shared__ __attribute__((aligned(16))) T tile[KV ? 4 : 1][KV ? 32 * TS : 1];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int m = lane & 31, kg = lane >> 5;
    const int64_t r0 = p.row_begin + (int64_t)blockIdx.x * 32;

    uint4 a[KC];
    if constexpr (AW == 0) {
        int64_t r = r0 + m;
        if (r >= p.row_end) r = p.row_end - 1;          // clamp: loads stay in bounds, stores are masked
        const int64_t ar = p.a_gather ? (int64_t)p.a_gather[r] : r;
        const uint4* ap = (const uint4*)((const T*)p.a + ar * p.a_stride);
#pragma unroll
        for (int c = 0; c < KC; ++c) a[c] = ap[2 * c + kg];
    }
    const uint4* wp = (const uint4*)p.w_packed + (int64_t)wave * NTW * KC * 64 + lane;
    uint4 ring[RING];
#pragma unroll
    for (int j = 0; j < RING; ++j) ring[j] = wp[j * 64];
    if constexpr (AW > 0) {
        constexpr int EPL = Elem<T>::EPL, LPR = D / EPL, G = 256 / LPR;
        const int group = (int)threadIdx.x / LPR, sub = (int)threadIdx.x % LPR;
#pragma unroll 1
        for (int rr = group; rr < 32; rr += G) {
            int64_t row = r0 + rr;
            if (row >= p.row_end) row = p.row_end - 1;  // computed again, never stored
            float av[EPL];
            attend_row<T, D, AW>(t, row, sub, av);
            uint4 oa, ob;
            Elem<T>::pack(av, oa, ob);
            uint4* op = (uint4*)&ybuf[rr * YS + sub * EPL];
            op[0] = oa; op[1] = ob;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < KC; ++c) a[c] = *(const uint4*)&ybuf[m * YS + (2 * c + kg) * E];
        __syncthreads();                          // the space is used again for the residual rows
    }
    // this thread's pieces of the rows: the residual now, where the results go later
    uint4 rpiece[PPT];
    int64_t pidx[PPT];                            // row of out[0] for the piece (-1: past the end)
#pragma unroll
    for (int q = 0; q < PPT; ++q) {
        const int piece = (int)threadIdx.x + 256 * q, row = piece / CPR, c = piece % CPR;
        const int64_t r = r0 + row;
        const int64_t rc = r < p.row_end ? r : p.row_end - 1;
        const int64_t rr = p.resid_gather ? (int64_t)p.resid_gather[rc] : rc;
        pidx[q] = r < p.row_end ? (p.out_scatter ? (int64_t)p.out_scatter[rc] : rc) : -1;
        rpiece[q] = *((const uint4*)((const T*)p.resid + rr * p.resid_stride) + c);
    }
    f32x16 acc[NTW];
#pragma unroll
    for (int j = 0; j < NTW * KC; ++j) {
        const int c = j % KC, nt = j / KC;
        if (c == 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[nt][i] = 0.f;
        }
        Mma<T>::run(a[c], ring[j % RING], acc[nt]);
        if (j + RING < NTW * KC) ring[j % RING] = wp[(j + RING) * 64];
    }
    constexpr int NTW2 = 2 * D / 32 / 4;          // column tiles of K | V per wave
    const uint4* wp2 = (const uint4*)p.kv_w_packed + (int64_t)wave * NTW2 * KC * 64 + lane;
    if constexpr (KV) {                           // the second product's first fragments, under the LayerNorm
#pragma unroll
        for (int j = 0; j < RING; ++j) ring[j] = wp2[j * 64];
    }
#pragma unroll
    for (int q = 0; q < PPT; ++q) {
        const int piece = (int)threadIdx.x + 256 * q;
        *(uint4*)&ybuf[(piece / CPR) * YS + (piece % CPR) * E] = rpiece[q];
    }
    __syncthreads();
    // residual, then LayerNorm over each row (no affine, biased variance), in two passes
    const int col0 = wave * NTW * 32 + m;
    float mean[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = 8 * (i / 4) + 4 * kg + (i % 4);
        float s1 = 0.f;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            acc[nt][i] += Elem<T>::load1(ybuf, (int64_t)row * YS + col0 + nt * 32);
            s1 += acc[nt][i];
        }
        s1 = sum_over_32_lanes(s1);
        if (m == 0) part[0][wave][row] = s1;
    }
    __syncthreads();                              // (also: every wave has taken its residual values)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = 8 * (i / 4) + 4 * kg + (i % 4);
        mean[i] = (part[0][0][row] + part[0][1][row] + part[0][2][row] + part[0][3][row]) * (1.0f / D);
        float s2 = 0.f;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) { const float t = acc[nt][i] - mean[i]; s2 = fmaf(t, t, s2); }
        s2 = sum_over_32_lanes(s2);
        if (m == 0) part[1][wave][row] = s2;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = 8 * (i / 4) + 4 * kg + (i % 4);
        const float rstd = rsqrtf((part[1][0][row] + part[1][1][row] + part[1][2][row] + part[1][3][row]) * (1.0f / D) + p.ln_eps);
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
            Elem<T>::store1(ybuf, (int64_t)row * YS + col0 + nt * 32, (acc[nt][i] - mean[i]) * rstd);
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PPT; ++q) {
        if (pidx[q] < 0) continue;
        const int piece = (int)threadIdx.x + 256 * q, row = piece / CPR, c = piece % CPR;
        const uint4 v = *(const uint4*)&ybuf[row * YS + c * E];
        *((uint4*)((T*)p.out[0] + pidx[q] * p.out_stride) + c) = v;
        if (p.out2) *((uint4*)((T*)p.out2 + (r0 + row) * p.out2_stride) + c) = v;
    }
    if constexpr (KV) {
        // (rows past the end hold the last row's values: computed, never stored)
        uint4 a2[KC];
#pragma unroll
        for (int c = 0; c < KC; ++c) a2[c] = *(const uint4*)&ybuf[m * YS + (2 * c + kg) * E];
        static_assert((NTW2 * KC) % GROUP == 0, "whole groups per wave");
        f32x16 kv;
#pragma unroll
        for (int j = 0; j < NTW2 * KC; ++j) {
            const int c = j % KC, nt = j / KC;
            if (c == 0) {
#pragma unroll
                for (int i = 0; i < 16; ++i) kv[i] = 0.f;
            }
            Mma<T>::run(a2[c], ring[j % RING], kv);
            if (j + RING < NTW2 * KC) ring[j % RING] = wp2[(j + RING) * 64];
            if (c == KC - 1) {
                // the 32x32 tile leaves through this wave's own corner of LDS, as 16-byte pieces
                // (LDS operations of a wave complete in order: no barrier)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    Elem<T>::store1(tile[wave], (int64_t)(8 * (i / 4) + 4 * kg + (i % 4)) * TS + m, kv[i]);
                const int col = (wave * NTW2 + nt) * 32;
#pragma unroll
                for (int q = 0; q < 32 * TPR / 64; ++q) {
                    const int piece = lane + 64 * q, row = piece / TPR, cc = piece % TPR;
                    const uint4 v = *(const uint4*)&tile[wave][row * TS + cc * E];
                    if (r0 + row < p.row_end)
                        *(uint4*)((T*)p.kv_out + (r0 + row) * p.kv_stride + col + cc * E) = v;
                }
            }
        }
    }
}

template <typename T, int D>
int launch_gemm_t(const dg4_gemm_args& a, const dg4_attn_args* att, hipStream_t s)
{
    const int64_t rows = a.row_end - a.row_begin;
    if (rows <= 0) return hipSuccess;
    unsigned grid = (unsigned)((rows + 127) / 128);
    // the kernel reads the weight stream in whole groups of fragments
    constexpr int KC = D / (2 * (16 / (int)sizeof(T)));
    constexpr int GROUP = KC > 16 ? KC : 16;
    const int64_t frags = (int64_t)(a.n_cols / 32) * KC;
    if (a.n_cols % 32 != 0 || frags % GROUP != 0) return hipErrorInvalidValue;
    if (a.epilogue) {
        if (a.n_cols != D) return hipErrorInvalidValue;
        constexpr bool can_split = ((D / 32 / 4) * KC) % GROUP == 0 && (D / 32) % 4 == 0;
        // (always the same kernel for a given shape, whatever the number of rows: the two sum the
        // LayerNorm statistics in different orders, and the embeddings must not depend on how the
        // rows were cut into launches)
        if constexpr (can_split) {
            const dim3 g32((unsigned)((rows + 31) / 32));
            const dg4_attn_args none{};
            const int aw = att ? att->ell_w : 0;
            if (att && (att->row_begin != a.row_begin || att->row_end != a.row_end)) return hipErrorInvalidValue;
#define DG4_LAUNCH_LN(KV_, AW_) hipLaunchKernelGGL((gemm_ln_split_kernel<T, D, KV_, AW_>), g32, dim3(256), 0, s, a, att ? *att : none)
            if (a.kv_out) {
                switch (aw) {
                case 0: DG4_LAUNCH_LN(true, 0); break;
                case 4: DG4_LAUNCH_LN(true, 4); break;
                case 8: DG4_LAUNCH_LN(true, 8); break;
                case 16: DG4_LAUNCH_LN(true, 16); break;
                default: return hipErrorInvalidValue;
                }
            } else {
                switch (aw) {
                case 0: DG4_LAUNCH_LN(false, 0); break;
                case 4: DG4_LAUNCH_LN(false, 4); break;
                case 8: DG4_LAUNCH_LN(false, 8); break;
                case 16: DG4_LAUNCH_LN(false, 16); break;
                default: return hipErrorInvalidValue;
                }
            }
#undef DG4_LAUNCH_LN
        } else {
            if (a.kv_out || att) return hipErrorInvalidValue;
            hipLaunchKernelGGL((gemm_kernel<T, D, true>), dim3(grid), dim3(256), 0, s, a);
        }
    } else {
        if (a.out2 && a.n_cols != D) return hipErrorInvalidValue;
        dg4_gemm_args b = a;
        // few rows (less than two workgroups per compute unit the plain way): split the columns over the waves
        b.split = (a.n_cols / 32) % 4 == 0 && (frags / 4) % GROUP == 0 && rows < 128 * 512 ? 1 : 0;
        if (b.split) grid = (unsigned)((rows + 31) / 32);
        hipLaunchKernelGGL((gemm_kernel<T, D, false>), dim3(grid), dim3(256), 0, s, b);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------ feed-forward

// W2 [4d, d] in the order the second product of ffn_kernel consumes it. The first product
// leaves, in accumulator element i of lane (m, kg), the activation of hidden unit
// 32*hc + 8*(i/4) + 4*kg + i%4 for row m; E consecutive elements (i = q*E .. q*E+E-1) form one
// A operand. 16-byte unit (((hc*G + q)*NT + nt)*64 + lane) holds the E matching rows of W2 for
// column nt*32 + lane%32, G = 16/E groups per 32 hidden units.
template <typename T>
__global__ void pack_w2_kernel(const T* w2, int d, T* packed)
{
    constexpr int E = 16 / sizeof(T);
    constexpr int G = 16 / E;
    const int NT = d / 32;
    const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t units = (int64_t)(4 * d / 32) * G * NT * 64;
    if (unit >= units) return;
    const int lane = (int)(unit & 63);
    int64_t t = unit >> 6;
    const int nt = (int)(t % NT); t /= NT;
    const int q = (int)(t % G);
    const int hc = (int)(t / G);
    const int n = nt * 32 + (lane & 31), kg = lane >> 5;
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int i = q * E + j;
        const int hidden = 32 * hc + 8 * (i / 4) + 4 * kg + (i % 4);
        packed[unit * E + j] = w2[(int64_t)hidden * d + n];
    }
}

template <typename T> struct Act;
template <> struct Act<bf16_t> {      // 16 activations -> two bf16 A operands
    __device__ static void pack(const f32x16& u, uint4* a)
    {
#pragma unroll
        for (int q = 0; q < 2; ++q)
            a[q] = make_uint4(pack_bf16x2(u[8 * q], u[8 * q + 1]), pack_bf16x2(u[8 * q + 2], u[8 * q + 3]),
                              pack_bf16x2(u[8 * q + 4], u[8 * q + 5]), pack_bf16x2(u[8 * q + 6], u[8 * q + 7]));
    }
};
template <> struct Act<float> {       // 16 activations -> four groups of four fp32 A operands
    __device__ static void pack(const f32x16& u, uint4* a)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            a[q] = make_uint4(__float_as_uint(u[4 * q]), __float_as_uint(u[4 * q + 1]),
                              __float_as_uint(u[4 * q + 2]), __float_as_uint(u[4 * q + 3]));
    }
};

// out = LN(h + max(h W1, 0) W2) for 32 rows per workgroup. The four waves split the 4d hidden
// units; each computes its slice of the activations TRANSPOSED (W1 tile as the A operand, the
// rows of h as B), so that the accumulator of the first product is, element for element, the A
// operand of the second (with W2 packed to match) and nothing moves between lanes. The four
// partial results are summed through LDS in a fixed order: (w0 + w2) + (w1 + w3).
template <typename T, int D>
__global__ __launch_bounds__(256) void ffn_kernel(dg4_ffn_args p)
{
    constexpr int E = 16 / sizeof(T);
    constexpr int KC = D / (2 * E);
    constexpr int NT = D / 32;
    constexpr int G = 16 / E;
    constexpr int CPW = D / 32;                 // chunks of 32 hidden units per wave (4d / 32 / 4)
    __shared__ float red[2][NT * 16 * 64];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int m = lane & 31, kg = lane >> 5;
    const int64_t r0 = p.row_begin + (int64_t)blockIdx.x * 32;

    uint4 a[KC];
    {
        int64_t r = r0 + m;
        if (r >= p.row_end) r = p.row_end - 1;          // clamp: loads stay in bounds, stores are masked
        const uint4* ap = (const uint4*)((const T*)p.h + r * p.h_stride);
#pragma unroll
        for (int c = 0; c < KC; ++c) a[c] = ap[2 * c + kg];
    }
    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nt][i] = 0.f;

    const uint4* w1p = (const uint4*)p.w1_packed + lane;
    const uint4* w2p = (const uint4*)p.w2_packed + lane;
#pragma unroll 2
    for (int ch = 0; ch < CPW; ++ch) {
        const int64_t hc = wave * CPW + ch;
        f32x16 u;
#pragma unroll
        for (int i = 0; i < 16; ++i) u[i] = 0.f;
#pragma unroll
        for (int c = 0; c < KC; ++c) Mma<T>::run(w1p[(hc * KC + c) * 64], a[c], u);
#pragma unroll
        for (int i = 0; i < 16; ++i) u[i] = fmaxf(u[i], 0.f);
        uint4 ua[G];
        Act<T>::pack(u, ua);
#pragma unroll
        for (int q = 0; q < G; ++q)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) Mma<T>::run(ua[q], w2p[((hc * G + q) * NT + nt) * 64], acc[nt]);
    }

    if (wave >= 2) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) red[wave - 2][(nt * 16 + i) * 64 + lane] = acc[nt][i];
    }
    __syncthreads();
    if (wave < 2) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[nt][i] += red[wave][(nt * 16 + i) * 64 + lane];
    }
    __syncthreads();
    if (wave == 1) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) red[0][(nt * 16 + i) * 64 + lane] = acc[nt][i];
    }
    __syncthreads();
    if (wave != 0) return;

    // wave 0: total, residual, LayerNorm (no affine, biased variance), store
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        int64_t r = r0 + 8 * (i / 4) + 4 * kg + (i % 4);
        const bool ok = r < p.row_end;
        if (!ok) r = p.row_end - 1;
        float s1 = 0.f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            acc[nt][i] += red[0][(nt * 16 + i) * 64 + lane];
            acc[nt][i] += Elem<T>::load1(p.h, r * p.h_stride + nt * 32 + m);
            s1 += acc[nt][i];
        }
        const float mean = sum_over_32_lanes(s1) * (1.0f / D);
        float s2 = 0.f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) { const float t = acc[nt][i] - mean; s2 = fmaf(t, t, s2); }
        const float rstd = rsqrtf(sum_over_32_lanes(s2) * (1.0f / D) + p.ln_eps);
        if (!ok) continue;
        const int64_t orr = p.out_scatter ? (int64_t)p.out_scatter[r] : r;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const float y = (acc[nt][i] - mean) * rstd;
            Elem<T>::store1(p.out, orr * p.out_stride + nt * 32 + m, y);
            if (p.out2) Elem<T>::store1(p.out2, r * p.out2_stride + nt * 32 + m, y);
        }
    }
}

// ------------------------------------------------- feed-forward, many rows at once (bf16, d = 256)
//
// dg4_ffn_fwd over a whole matrix is bound by how often the megabyte of W1 | W2 has to come from
// the L2 cache: ffn_kernel above reads it once per 32 rows. Here a workgroup takes 64 rows, keeps
// them in LDS, and streams the weights once for all of them: one contiguous stream per wave, in
// four passes of 256 hidden units. Per pass a wave forms the activations of its 64 hidden units
// for all 64 rows (transposed, W1 piece as the A operand), rectifies and writes them to LDS,
// and after a barrier adds the pass's part of ITS 64 output columns for all rows (the output
// accumulators, 64 registers, stay put over the passes). Residual + LayerNorm from registers with
// the row sums completed through LDS; the result leaves through LDS as whole 16-byte pieces.
// Two workgroups share a compute unit (70 KB of LDS and at most 256 registers each), so that one
// computes while the other waits at a barrier or for its rows: measured 1.18 ms for 1M rows, against
// 1.32 ms with 96 rows and one workgroup per compute unit (a third less weight traffic, no overlap).
constexpr int FB_ROWS = 64, FB_RT = 2, FB_STRIDE = 264, FB_PASSES = 4, FB_FRAGS = 64, FB_RING = 8;
constexpr int FB_SMEM = 2 * FB_ROWS * FB_STRIDE * 2 + 2 * 4 * FB_ROWS * 4;

// Stream order, 16-byte units: (((w*4 + pass)*64 + j)*64 + lane), lane = 32*kg + m.
//  j < 32 : first product, hidden tile t = j/16, k-step ks = j%16:
//           W1[16*ks + 8*kg + e][256*pass + 64*w + 32*t + m], e = 0..7
//  j >= 32: second product, k-step ks = (j-32)/2, column tile ct = (j-32)%2:
//           W2[256*pass + 16*ks + 8*kg + e][64*w + 32*ct + m]
__global__ void pack_ffn_bulk_kernel(const uint16_t* w1, const uint16_t* w2, uint16_t* packed)
{
    const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (unit >= 4 * FB_PASSES * FB_FRAGS * 64) return;
    const int lane = (int)(unit & 63);
    const int j = (int)((unit >> 6) % FB_FRAGS);
    const int pass = (int)((unit >> 12) % FB_PASSES);
    const int w = (int)(unit >> 14);
    const int m = lane & 31, kg = lane >> 5;
    if (j < 32) {
        const int t = j >> 4, ks = j & 15;
        const int hidden = 256 * pass + 64 * w + 32 * t + m;
#pragma unroll
        for (int e = 0; e < 8; ++e) packed[unit * 8 + e] = w1[(int64_t)(16 * ks + 8 * kg + e) * 1024 + hidden];
    } else {
        const int ks = (j - 32) >> 1, ct = (j - 32) & 1;
        const int col = 64 * w + 32 * ct + m;
#pragma unroll
        for (int e = 0; e < 8; ++e) packed[unit * 8 + e] = w2[(int64_t)(256 * pass + 16 * ks + 8 * kg + e) * 256 + col];
    }
}

__device__ __forceinline__ void lds_barrier()      // LDS traffic only: the weight loads in flight are not drained
{
    __asm__ volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    __asm__ volatile("" ::: "memory");
}

__global__ __launch_bounds__(256, 2) void ffn_bulk_kernel(dg4_ffn_args p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char fb_smem[];
    uint16_t (*sH)[FB_STRIDE] = (uint16_t (*)[FB_STRIDE])fb_smem;
    uint16_t (*sU)[FB_STRIDE] = sH + FB_ROWS;
    float (*sPart)[4][FB_ROWS] = (float (*)[4][FB_ROWS])(fb_smem + 2 * FB_ROWS * FB_STRIDE * 2);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, kg = lane >> 5;
    const int64_t r0 = p.row_begin + (int64_t)blockIdx.x * FB_ROWS;
    const uint16_t* h = (const uint16_t*)p.h;

    // the rows of this workgroup (past the end: the last row again; never stored)
#pragma unroll
    for (int i = 0; i < FB_ROWS * 32 / 256; ++i) {
        const int chunk = tid + 256 * i, row = chunk >> 5, c16 = chunk & 31;
        int64_t r = r0 + row;
        if (r >= p.row_end) r = p.row_end - 1;
        *(uint4*)&sH[row][c16 * 8] = *(const uint4*)(h + r * p.h_stride + c16 * 8);
    }
    const uint4* wp = (const uint4*)p.w1_packed + (int64_t)wave * (FB_PASSES * FB_FRAGS * 64) + lane;
    uint4 ring[FB_RING];
#pragma unroll
    for (int j = 0; j < FB_RING; ++j) ring[j] = wp[j * 64];
    __syncthreads();

    f32x16 out[2][FB_RT];
#pragma unroll 1
    for (int pass = 0; pass < FB_PASSES; ++pass) {
        const uint4* wq = wp + (int64_t)pass * (FB_FRAGS * 64);
        const bool more = pass + 1 < FB_PASSES;
        if (pass) lds_barrier();                  // the previous pass's activations have been read by every wave
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f32x16 u[FB_RT];
            // (the rows' operands of the next step are read from LDS while this step's products run)
            uint4 bc[FB_RT], bn[FB_RT];
#pragma unroll
            for (int rt = 0; rt < FB_RT; ++rt) bc[rt] = *(const uint4*)&sH[32 * rt + m][8 * kg];
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) {
                const int j = 16 * t + ks;
#pragma unroll
                for (int rt = 0; rt < FB_RT; ++rt) bn[rt] = ks + 1 < 16 ? *(const uint4*)&sH[32 * rt + m][16 * (ks + 1) + 8 * kg] : bc[rt];
#pragma unroll
                for (int rt = 0; rt < FB_RT; ++rt) {
                    if (ks == 0) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) u[rt][i] = 0.f;
                    }
                    Mma<bf16_t>::run(ring[j % FB_RING], bc[rt], u[rt]);
                }
                ring[j % FB_RING] = wq[(j + FB_RING) * 64];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int rt = 0; rt < FB_RT; ++rt) bc[rt] = bn[rt];
            }
            // rectified, to LDS by row: element i of the accumulator is hidden unit 8*(i/4) + 4*kg + i%4 of the tile
#pragma unroll
            for (int rt = 0; rt < FB_RT; ++rt)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *(uint2*)&sU[32 * rt + m][64 * wave + 32 * t + 8 * q + 4 * kg] =
                        make_uint2(pack_bf16x2(fmaxf(u[rt][4 * q], 0.f), fmaxf(u[rt][4 * q + 1], 0.f)),
                                   pack_bf16x2(fmaxf(u[rt][4 * q + 2], 0.f), fmaxf(u[rt][4 * q + 3], 0.f)));
        }
        lds_barrier();
        {
            uint4 bc[FB_RT], bn[FB_RT];
#pragma unroll
            for (int rt = 0; rt < FB_RT; ++rt) bc[rt] = *(const uint4*)&sU[32 * rt + m][8 * kg];
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) {
#pragma unroll
                for (int rt = 0; rt < FB_RT; ++rt) bn[rt] = ks + 1 < 16 ? *(const uint4*)&sU[32 * rt + m][16 * (ks + 1) + 8 * kg] : bc[rt];
#pragma unroll
                for (int ct = 0; ct < 2; ++ct) {
                    const int j = 32 + 2 * ks + ct;
#pragma unroll
                    for (int rt = 0; rt < FB_RT; ++rt) {
                        if (pass == 0 && ks == 0) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) out[ct][rt][i] = 0.f;
                        }
                        Mma<bf16_t>::run(ring[j % FB_RING], bc[rt], out[ct][rt]);
                    }
                    if (j + FB_RING < FB_FRAGS || more) ring[j % FB_RING] = wq[(j + FB_RING) * 64];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int rt = 0; rt < FB_RT; ++rt) bc[rt] = bn[rt];
            }
        }
    }

    // residual and LayerNorm (no affine, biased variance, two passes). Lane (m, kg) holds, of row
    // 32*rt + m, the columns 64*wave + 32*ct + 8*q + 4*kg + r (accumulator element 4*q + r).
    float mean[FB_RT];
#pragma unroll
    for (int rt = 0; rt < FB_RT; ++rt) {
        float s1 = 0.f;
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint2 hv = *(const uint2*)&sH[32 * rt + m][64 * wave + 32 * ct + 8 * q + 4 * kg];
                out[ct][rt][4 * q] += bf16_lo(hv.x); out[ct][rt][4 * q + 1] += bf16_hi(hv.x);
                out[ct][rt][4 * q + 2] += bf16_lo(hv.y); out[ct][rt][4 * q + 3] += bf16_hi(hv.y);
#pragma unroll
                for (int r = 0; r < 4; ++r) s1 += out[ct][rt][4 * q + r];
            }
        s1 += __shfl_xor(s1, 32);
        if (kg == 0) sPart[0][wave][32 * rt + m] = s1;
    }
    __syncthreads();                              // also: every wave is done with the activations in sU
#pragma unroll
    for (int rt = 0; rt < FB_RT; ++rt) {
        const int row = 32 * rt + m;
        mean[rt] = (sPart[0][0][row] + sPart[0][1][row] + sPart[0][2][row] + sPart[0][3][row]) * (1.0f / 256);
        float s2 = 0.f;
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) { const float d = out[ct][rt][i] - mean[rt]; s2 = fmaf(d, d, s2); }
        s2 += __shfl_xor(s2, 32);
        if (kg == 0) sPart[1][wave][row] = s2;
    }
    __syncthreads();
#pragma unroll
    for (int rt = 0; rt < FB_RT; ++rt) {
        const int row = 32 * rt + m;
        const float rstd = rsqrtf((sPart[1][0][row] + sPart[1][1][row] + sPart[1][2][row] + sPart[1][3][row]) * (1.0f / 256) + p.ln_eps);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float y[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) y[r] = (out[ct][rt][4 * q + r] - mean[rt]) * rstd;
                *(uint2*)&sU[row][64 * wave + 32 * ct + 8 * q + 4 * kg] = make_uint2(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
            }
    }
    __syncthreads();
    uint16_t* o = (uint16_t*)p.out;
    uint16_t* o2 = (uint16_t*)p.out2;
#pragma unroll
    for (int i = 0; i < FB_ROWS * 32 / 256; ++i) {
        const int chunk = tid + 256 * i, row = chunk >> 5, c16 = chunk & 31;
        const int64_t r = r0 + row;
        if (r >= p.row_end) continue;
        const uint4 v = *(const uint4*)&sU[row][c16 * 8];
        const int64_t orr = p.out_scatter ? (int64_t)p.out_scatter[r] : r;
        *(uint4*)(o + orr * p.out_stride + c16 * 8) = v;
        if (o2) *(uint4*)(o2 + r * p.out2_stride + c16 * 8) = v;
    }
}

template <typename T, int D>
int launch_ffn_t(const dg4_ffn_args& a, hipStream_t s)
{
    const int64_t rows = a.row_end - a.row_begin;
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL((ffn_kernel<T, D>), dim3((unsigned)((rows + 31) / 32)), dim3(256), 0, s, a);
    return hipGetLastError();
}

// Structural encoding (paper Section 3.5, Eq. 2): out[v] = x[v] + (level*w_l + b_l) + (OutAND*w_and +
// b_and) + (OutNOT*w_not + b_not). Elementwise and HBM-bound (a row in, a row out, 12 bytes of
// integer features): one thread per 16 bytes of a row, the [6, d] embedding table comes from cache.
template <typename T, int D>
__global__ __launch_bounds__(256) void struct_encode_kernel(const T* x, const int32_t* feat, const float* emb, T* out, int64_t n)
{
    constexpr int E = 16 / (int)sizeof(T);           // elements per thread
    constexpr int U = D / E;                         // threads per row
    constexpr int RPB = 256 / U;                     // rows per block and step
    const int c0 = (int)(threadIdx.x % U) * E;
    // this thread's slice of the six embedding rows stays in registers while it walks down the rows
    float wl[E], bl[E], wa[E], ba[E], wn[E], bn[E];
#pragma unroll
    for (int i = 0; i < E; ++i) {
        wl[i] = emb[c0 + i]; bl[i] = emb[D + c0 + i]; wa[i] = emb[2 * D + c0 + i];
        ba[i] = emb[3 * D + c0 + i]; wn[i] = emb[4 * D + c0 + i]; bn[i] = emb[5 * D + c0 + i];
    }
    for (int64_t v = (int64_t)blockIdx.x * RPB + threadIdx.x / U; v < n; v += (int64_t)gridDim.x * RPB) {
        const float lev = (float)feat[3 * v], oa = (float)feat[3 * v + 1], on = (float)feat[3 * v + 2];
        const uint4 raw = *(const uint4*)(x + v * D + c0);
        float f[8];
        if (sizeof(T) == 4) {
            f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y); f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
        } else {
            const uint32_t w4[4] = { raw.x, raw.y, raw.z, raw.w };
#pragma unroll
            for (int i = 0; i < 4; ++i) { f[2 * i] = bf16_lo(w4[i]); f[2 * i + 1] = bf16_hi(w4[i]); }
        }
        // the three linear layers, summed in the order of Eq. 2, then added to the feature
#pragma unroll
        for (int i = 0; i < E; ++i) f[i] += fmaf(lev, wl[i], bl[i]) + fmaf(oa, wa[i], ba[i]) + fmaf(on, wn[i], bn[i]);
        uint4 o;
        if (sizeof(T) == 4) {
            o = make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
        } else {
            o = make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
        }
        *(uint4*)(out + v * D + c0) = o;
    }
}

template <typename T, int D>
int launch_struct_encode_t(const void* x, const int32_t* feat, const float* emb, void* out, int64_t n, hipStream_t s)
{
    constexpr int RPB = 256 / (D / (16 / (int)sizeof(T)));
    const int64_t blocks = std::min<int64_t>((n + RPB - 1) / RPB, 256 * 16);      // 16 workgroups per compute unit
    hipLaunchKernelGGL((struct_encode_kernel<T, D>), dim3((unsigned)blocks), dim3(256), 0, s,
                       (const T*)x, feat, emb, (T*)out, n);
    return hipGetLastError();
}

}  // namespace

int dg4_launch_struct_encode(int dtype, int hidden, const void* x, const int32_t* feat, const float* emb, void* out,
                             int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    if (dtype == DG4_F32)
        return hidden == 128 ? launch_struct_encode_t<float, 128>(x, feat, emb, out, n, s) : launch_struct_encode_t<float, 256>(x, feat, emb, out, n, s);
    return hidden == 128 ? launch_struct_encode_t<uint16_t, 128>(x, feat, emb, out, n, s) : launch_struct_encode_t<uint16_t, 256>(x, feat, emb, out, n, s);
}

// shapes whose epilogue kernel can carry the K | V product (gemm_ln_split_kernel)
bool dg4_gemm_fuses_kv(int dtype, int hidden)
{
    const int e = dtype == DG4_F32 ? 4 : 8;
    const int kc = hidden / (2 * e), group = kc > 16 ? kc : 16;
    return (hidden / 32) % 4 == 0 && ((hidden / 32 / 4) * kc) % group == 0;
}

int dg4_launch_attn(int dtype, int hidden, const dg4_attn_args& a, hipStream_t s)
{
    if (dtype == DG4_F32) return hidden == 128 ? launch_attn_w<float, 128>(a, s) : launch_attn_w<float, 256>(a, s);
    return hidden == 128 ? launch_attn_w<bf16_t, 128>(a, s) : launch_attn_w<bf16_t, 256>(a, s);
}

int dg4_launch_pack_w(int dtype, const void* w, int ld, int col0, int n_cols, int k_dim, void* packed, hipStream_t s)
{
    const int e = dtype == DG4_F32 ? 4 : 8;
    const int64_t units = (int64_t)(n_cols / 32) * (k_dim / (2 * e)) * 64;
    const unsigned grid = (unsigned)((units + 255) / 256);
    if (dtype == DG4_F32)
        hipLaunchKernelGGL(pack_w_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)w, ld, col0, n_cols, k_dim, (float*)packed);
    else
        hipLaunchKernelGGL(pack_w_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, (const uint16_t*)w, ld, col0, n_cols, k_dim, (uint16_t*)packed);
    return hipGetLastError();
}

int dg4_launch_pack_w2(int dtype, const void* w2, int hidden, void* packed, hipStream_t s)
{
    const int e = dtype == DG4_F32 ? 4 : 8;
    const int64_t units = (int64_t)(4 * hidden / 32) * (16 / e) * (hidden / 32) * 64;
    const unsigned grid = (unsigned)((units + 255) / 256);
    if (dtype == DG4_F32)
        hipLaunchKernelGGL(pack_w2_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)w2, hidden, (float*)packed);
    else
        hipLaunchKernelGGL(pack_w2_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, (const uint16_t*)w2, hidden, (uint16_t*)packed);
    return hipGetLastError();
}

int dg4_launch_pack_ffn_bulk(const void* w1, const void* w2, void* packed, hipStream_t s)
{
    const int64_t units = 4 * FB_PASSES * FB_FRAGS * 64;
    hipLaunchKernelGGL(pack_ffn_bulk_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s,
                       (const uint16_t*)w1, (const uint16_t*)w2, (uint16_t*)packed);
    return hipGetLastError();
}

int dg4_launch_ffn_bulk(const dg4_ffn_args& a, hipStream_t s)
{
    const int64_t rows = a.row_end - a.row_begin;
    if (rows <= 0) return hipSuccess;
    hipError_t e = hipFuncSetAttribute((const void*)ffn_bulk_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, FB_SMEM);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ffn_bulk_kernel, dim3((unsigned)((rows + FB_ROWS - 1) / FB_ROWS)), dim3(256), FB_SMEM, s, a);
    return hipGetLastError();
}

int dg4_launch_ffn(int dtype, int hidden, const dg4_ffn_args& a, hipStream_t s)
{
    if (dtype == DG4_F32) return hidden == 128 ? launch_ffn_t<float, 128>(a, s) : launch_ffn_t<float, 256>(a, s);
    return hidden == 128 ? launch_ffn_t<bf16_t, 128>(a, s) : launch_ffn_t<bf16_t, 256>(a, s);
}

int dg4_launch_gemm(int dtype, int hidden, const dg4_gemm_args& a, hipStream_t s)
{
    if (dtype == DG4_F32) return hidden == 128 ? launch_gemm_t<float, 128>(a, nullptr, s) : launch_gemm_t<float, 256>(a, nullptr, s);
    return hidden == 128 ? launch_gemm_t<bf16_t, 128>(a, nullptr, s) : launch_gemm_t<bf16_t, 256>(a, nullptr, s);
}

// The epilogue product with its rows' operand computed in the same launch: the attention `att`
// (same row range, neighbour rows of width 4, 8 or 16) instead of a.a. Shapes for which
// dg4_gemm_fuses_kv() holds.
int dg4_launch_attn_gemm(int dtype, int hidden, const dg4_attn_args& att, const dg4_gemm_args& a, hipStream_t s)
{
    if (!a.epilogue) return hipErrorInvalidValue;
    if (dtype == DG4_F32) return hidden == 128 ? launch_gemm_t<float, 128>(a, &att, s) : launch_gemm_t<float, 256>(a, &att, s);
    return hidden == 128 ? launch_gemm_t<bf16_t, 128>(a, &att, s) : launch_gemm_t<bf16_t, 256>(a, &att, s);
}
