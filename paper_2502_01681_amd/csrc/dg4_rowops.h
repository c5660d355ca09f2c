// Per-row device functions shared by the level-by-level kernels and the persistent dataflow kernel:
// the attention of one destination row, the matrix-core product step, a row sum. One definition, so
// that a gate's arithmetic is the same whichever kernel computes it.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dg4_device.h"
#include "dg4_internal.h"

namespace {

// The attention of one destination row (Section 3.5), by a group of LPR = D / EPL lanes of which this
// lane is number `sub`: every lane owns 32 contiguous bytes of each 512-byte (or 256 / 1024-byte) row
// it touches and ends with its EPL elements of the row's result. `ent`: the packed neighbour row;
// q_row, k_self, v_self: the destination's own rows (any address space); sources at k_src / v_src +
// index * src_stride elements; rel_bias [heads, 4]. CH: neighbour rows requested together (a matter of
// latency against registers only: the arithmetic of a row does not depend on it). V_EARLY (needs CH == W):
// the V rows are requested together with the K rows, before the scores are formed.
template <typename T, int D, int W, int CH = (W < 8 ? W : 8), bool V_EARLY = false>
__device__ __forceinline__ void attend_core(const uint32_t (&ent)[W], const T* q_row, const T* k_self, const T* v_self,
                                            const T* k_src, const T* v_src, int64_t src_stride, const float* rel_bias,
                                            int sub, float (&acc)[Elem<T>::EPL])
{
    constexpr int EPL = Elem<T>::EPL;
    static_assert(W % CH == 0, "whole passes");
    const int64_t eoff = (int64_t)sub * EPL;  // element offset of this lane inside a row
    const int head = (int)(eoff >> 5);

    float q[EPL];
    {
        const uint4* qp = (const uint4*)(q_row + eoff);
        Elem<T>::unpack(qp[0], qp[1], q);
    }
    float bias[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) bias[i] = rel_bias[head * 4 + i];

    auto src_row = [&](const T* self_row, const T* src_base, uint32_t e) -> const uint4* {
        const uint32_t rel = e >> 30;
        const int64_t idx = e & 0x3FFFFFFFu;
        const T* r = rel == 0 ? self_row : src_base + idx * src_stride;
        return (const uint4*)(r + eoff);
    };

    static_assert(!V_EARLY || CH == W, "all rows at once");
    uint4 va0[V_EARLY ? W : 1], vb0[V_EARLY ? W : 1];
    // pass 1: scores
    float s[W];
    const float scale = 0.17677669529663687f;     // 1/sqrt(32)
#pragma unroll
    for (int c0 = 0; c0 < W; c0 += CH) {
        uint4 ka[CH], kb[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            if (ent[c0 + j] != DG4_ELL_PAD) {
                const uint4* kp = src_row(k_self, k_src, ent[c0 + j]);
                ka[j] = kp[0]; kb[j] = kp[1];
            } else {
                ka[j] = make_uint4(0, 0, 0, 0); kb[j] = ka[j];
            }
        }
        if constexpr (V_EARLY) {
#pragma unroll
            for (int j = 0; j < W; ++j) {
                if (ent[j] != DG4_ELL_PAD) {
                    const uint4* vp = src_row(v_self, v_src, ent[j]);
                    va0[j] = vp[0]; vb0[j] = vp[1];
                } else {
                    va0[j] = make_uint4(0, 0, 0, 0); vb0[j] = va0[j];
                }
            }
        }
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            float k[EPL];
            Elem<T>::unpack(ka[j], kb[j], k);
            float dot = 0.f;
#pragma unroll
            for (int i = 0; i < EPL; ++i) dot = fmaf(q[i], k[i], dot);
            dot = Elem<T>::head_sum(dot);
            const uint32_t rel = ent[c0 + j] >> 30;
            const float b = rel == 0 ? bias[0] : rel == 1 ? bias[1] : rel == 2 ? bias[2] : bias[3];
            s[c0 + j] = ent[c0 + j] != DG4_ELL_PAD ? fmaf(dot, scale, b) : -INFINITY;
        }
    }
    // softmax over the row, in this lane (all lanes of a head hold the same s)
    float mx = s[0];
#pragma unroll
    for (int j = 1; j < W; ++j) mx = fmaxf(mx, s[j]);
    float z = 0.f;
#pragma unroll
    for (int j = 0; j < W; ++j) { s[j] = __expf(s[j] - mx); z += s[j]; }
    const float rz = 1.0f / z;

    // pass 2: aggregation
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;
#pragma unroll
    for (int c0 = 0; c0 < W; c0 += CH) {
        uint4 va[CH], vb[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            if constexpr (V_EARLY) {
                va[j] = va0[j]; vb[j] = vb0[j];
            } else if (ent[c0 + j] != DG4_ELL_PAD) {
                const uint4* vp = src_row(v_self, v_src, ent[c0 + j]);
                va[j] = vp[0]; vb[j] = vp[1];
            } else {
                va[j] = make_uint4(0, 0, 0, 0); vb[j] = va[j];
            }
        }
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            float v[EPL];
            Elem<T>::unpack(va[j], vb[j], v);
            const float al = s[c0 + j] * rz;
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] = fmaf(al, v[i], acc[i]);
        }
    }
}

// A table of rows in global memory as a structured buffer: row i at base + i * row_bytes, rows_total
// rows. A load through it takes a row index and a byte offset inside the row; an index at or past
// rows_total reads as zeros and costs no memory request (the range check of buffer addressing), which
// is how a lane skips a row without a branch.
typedef int dg4_i32x4 __attribute__((ext_vector_type(4)));
__device__ dg4_i32x4 dg4_struct_buffer_load16(dg4_i32x4 rsrc, int vindex, int voffset, int soffset, int aux)
    __asm("llvm.amdgcn.struct.buffer.load.v4i32");
__device__ __forceinline__ dg4_i32x4 row_buffer(const void* base, uint32_t row_bytes, uint32_t rows_total)
{
    const uint64_t a = (uint64_t)(uintptr_t)base;
    dg4_i32x4 r;
    r.x = (int)(uint32_t)a;
    r.y = (int)(((uint32_t)(a >> 32) & 0xFFFFu) | (row_bytes << 16));      // stride in bits 16..29, no swizzling
    r.z = (int)rows_total;                                                  // records of `row_bytes`
    r.w = 0x00020000;                                                       // 32-bit data format, raw dwords
    return r;
}
__device__ __forceinline__ uint4 row_load16(dg4_i32x4 rsrc, uint32_t row, uint32_t byte_off)
{
    const dg4_i32x4 v = dg4_struct_buffer_load16(rsrc, (int)row, (int)byte_off, 0, 0);
    return make_uint4((uint32_t)v.x, (uint32_t)v.y, (uint32_t)v.z, (uint32_t)v.w);
}

// The same attention with as few trips to memory as the registers allow, for the persistent kernel: the
// row is walked in chunks of eight entries, K and V halves of a chunk requested together, with a
// running maximum, denominator and weighted sum (the softmax is unchanged by the rescaling; the
// result differs from attend_core's by rounding only). The gate's own rows (q_row, k_self, v_self:
// LDS) are taken first, while the first chunk travels. Sources are rows of the structured buffer `kv`
// (K in the first half of a row, V in the second); entries that are no source (the gate itself,
// padding) ask for row kv_rows, past the end: zeros, no request, no branch, so the requests of a chunk
// go out back to back and are waited for one by one. The K halves of the next chunk are requested as
// soon as the scores of this one are formed.
template <typename T, int D, int W>
__device__ __forceinline__ void attend_chunked(const uint32_t (&ent)[W], const T* q_row, const T* k_self, const T* v_self,
                                               dg4_i32x4 kv, uint32_t kv_rows, const float* rel_bias, int sub,
                                               float (&acc)[Elem<T>::EPL])
{
    constexpr int EPL = Elem<T>::EPL, CH = 8, NC = W / CH;
    static_assert(W % CH == 0, "whole chunks");
    const int64_t eoff = (int64_t)sub * EPL;
    const int head = (int)(eoff >> 5);
    auto is_source = [&](uint32_t e) __attribute__((always_inline)) { return e != DG4_ELL_PAD && (e >> 30) != 0; };
    auto fetch = [&](uint32_t half, int c0, uint4 (&a)[CH], uint4 (&b)[CH]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const uint32_t e = ent[c0 + j];
            const uint32_t row = is_source(e) ? (e & 0x3FFFFFFFu) : kv_rows;
            a[j] = row_load16(kv, row, half * (uint32_t)(D * sizeof(T)) + (uint32_t)sub * 32u);
            b[j] = row_load16(kv, row, half * (uint32_t)(D * sizeof(T)) + (uint32_t)sub * 32u + 16u);
        }
    };
    float bias[4];                                // (requested before the rows: loads return in order)
#pragma unroll
    for (int i = 0; i < 4; ++i) bias[i] = rel_bias[head * 4 + i];
    uint4 ka[CH], kb[CH], va[CH], vb[CH];
    fetch(0, 0, ka, kb);
    fetch(1, 0, va, vb);

    const uint4 qa = ((const uint4*)(q_row + eoff))[0], qb = ((const uint4*)(q_row + eoff))[1];
    const float scale = 0.17677669529663687f;     // 1/sqrt(32)
    // the gate itself (every row built by this library holds it; one without it starts from nothing)
    uint32_t lowest = ent[0];
#pragma unroll
    for (int j = 1; j < W; ++j) lowest = lowest < ent[j] ? lowest : ent[j];
    const bool has_self = (lowest >> 30) == 0;
    float m, z;
    {
        const uint4* kp = (const uint4*)(k_self + eoff);
        const uint4* vp = (const uint4*)(v_self + eoff);
        float v[EPL];
        Elem<T>::unpack(vp[0], vp[1], v);
        const float dot = Elem<T>::head_sum(Elem<T>::dot(qa, qb, kp[0], kp[1]));
        m = has_self ? fmaf(dot, scale, bias[0]) : -INFINITY;
        z = has_self ? 1.f : 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] = has_self ? v[i] : 0.f;
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (c > 0) fetch(1, c * CH, va, vb);
        float s[CH];
        float cm = m;
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const float dot = Elem<T>::head_sum(Elem<T>::dot(qa, qb, ka[j], kb[j]));
            const uint32_t e = ent[c * CH + j];
            const uint32_t rel = e >> 30;
            const float b = rel == 1 ? bias[1] : rel == 2 ? bias[2] : bias[3];
            s[j] = is_source(e) ? fmaf(dot, scale, b) : -INFINITY;
            cm = fmaxf(cm, s[j]);
        }
        if (c + 1 < NC) fetch(0, (c + 1) * CH, ka, kb);
        // (a chunk without sources leaves everything as it is: corr = 1, every weight 0; the first chunk
        // of a row without the gate itself holds a source, so cm is finite whenever m is not)
        const float corr = __expf(m - cm);
        z *= corr;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] *= corr;
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            float v[EPL];
            Elem<T>::unpack(va[j], vb[j], v);
            const float pj = __expf(s[j] - cm);   // 0 for what is no source
            z += pj;
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] = fmaf(pj, v[i], acc[i]);
        }
        m = cm;
    }
    const float rz = 1.0f / z;
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] *= rz;
}

// the packed neighbour row `row` of a table of width W
template <int W>
__device__ __forceinline__ void load_entries(const uint32_t* ell, int64_t row, uint32_t (&ent)[W])
{
    const uint4* e4 = (const uint4*)(ell + row * W);
#pragma unroll
    for (int i = 0; i < W / 4; ++i) {
        const uint4 t = e4[i];
        ent[4 * i] = t.x; ent[4 * i + 1] = t.y; ent[4 * i + 2] = t.z; ent[4 * i + 3] = t.w;
    }
}

// attend_core on the tensors of a launch: destination row `row` of p
template <typename T, int D, int W>
__device__ __forceinline__ void attend_row(const dg4_attn_args& p, int64_t row, int sub, float (&acc)[Elem<T>::EPL])
{
    uint32_t ent[W];
    load_entries<W>(p.ell, row, ent);
    attend_core<T, D, W>(ent, (const T*)p.q + row * p.q_stride, (const T*)p.k_self + row * p.self_stride,
                         (const T*)p.v_self + row * p.self_stride, (const T*)p.k_src, (const T*)p.v_src, p.src_stride,
                         p.rel_bias, sub, acc);
}

// One step of a 32-row product on the matrix cores: 16 bytes of A (rows) and of B (packed weight)
// per lane; accumulator element i of lane (m = lane % 32, kg = lane / 32) is row 8*(i/4) + 4*kg + i%4,
// column m of the 32x32 tile.
template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    __device__ static void run(const uint4& a, const uint4& b, f32x16& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    __device__ static void run(const uint4& a, const uint4& b, f32x16& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

__device__ __forceinline__ float sum_over_32_lanes(float v)
{
    v += __shfl_xor(v, 1); v += __shfl_xor(v, 2); v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 8); v += __shfl_xor(v, 16);
    return v;
}

}  // namespace
