// Device-side helpers shared by the kernels: bf16 conversion, lane exchange,
// and the per-dtype view of a lane's 32 bytes of a feature row.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct bf16_t { uint16_t bits; };   // storage only

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// float -> bfloat16 bits, round to nearest even (NaN kept quiet).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
// two floats -> packed bfloat16 pair, round to nearest even, in one instruction
// (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Lane exchange inside a group of 4 lanes by data-parallel primitives.
__device__ __forceinline__ float xor1(float v)   // lane ^ 1
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float xor2(float v)   // lane ^ 2
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int EPL = 8;                 // elements in a lane's 32 bytes
    __device__ static void unpack(const uint4& a, const uint4& b, float* f)
    {
        f[0] = __uint_as_float(a.x); f[1] = __uint_as_float(a.y); f[2] = __uint_as_float(a.z); f[3] = __uint_as_float(a.w);
        f[4] = __uint_as_float(b.x); f[5] = __uint_as_float(b.y); f[6] = __uint_as_float(b.z); f[7] = __uint_as_float(b.w);
    }
    __device__ static void pack(const float* f, uint4& a, uint4& b)
    {
        a = make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
        b = make_uint4(__float_as_uint(f[4]), __float_as_uint(f[5]), __float_as_uint(f[6]), __float_as_uint(f[7]));
    }
    // the lane's part of a dot product of two rows, from their 32 bytes as loaded
    __device__ static float dot(const uint4& qa, const uint4& qb, const uint4& ka, const uint4& kb)
    {
        float q[8], k[8];
        unpack(qa, qb, q); unpack(ka, kb, k);
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) d = fmaf(q[i], k[i], d);
        return d;
    }
    __device__ static float head_sum(float p) { p += xor1(p); p += xor2(p); return p; }   // 4 lanes per head
    __device__ static float load1(const void* p, int64_t i) { return ((const float*)p)[i]; }
    __device__ static void store1(void* p, int64_t i, float v) { ((float*)p)[i] = v; }
};
template <> struct Elem<bf16_t> {
    static constexpr int EPL = 16;
    __device__ static void unpack(const uint4& a, const uint4& b, float* f)
    {
        const uint32_t w[8] = { a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w };
#pragma unroll
        for (int i = 0; i < 8; ++i) { f[2 * i] = bf16_lo(w[i]); f[2 * i + 1] = bf16_hi(w[i]); }
    }
    __device__ static void pack(const float* f, uint4& a, uint4& b)
    {
        a = make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
        b = make_uint4(pack_bf16x2(f[8], f[9]), pack_bf16x2(f[10], f[11]), pack_bf16x2(f[12], f[13]), pack_bf16x2(f[14], f[15]));
    }
    // (pairs of bfloat16 multiplied and added in one instruction, fp32 accumulation, two chains)
    __device__ static float dot(const uint4& qa, const uint4& qb, const uint4& ka, const uint4& kb)
    {
        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
        auto d2 = [](uint32_t a, uint32_t b, float c) {
            return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
        };
        float d0 = 0.f, d1 = 0.f;
        d0 = d2(qa.x, ka.x, d0); d1 = d2(qa.y, ka.y, d1);
        d0 = d2(qa.z, ka.z, d0); d1 = d2(qa.w, ka.w, d1);
        d0 = d2(qb.x, kb.x, d0); d1 = d2(qb.y, kb.y, d1);
        d0 = d2(qb.z, kb.z, d0); d1 = d2(qb.w, kb.w, d1);
        return d0 + d1;
    }
    __device__ static float head_sum(float p) { p += xor1(p); return p; }                   // 2 lanes per head
    __device__ static float load1(const void* p, int64_t i) { return bf16_lo(((const uint16_t*)p)[i]); }
    __device__ static void store1(void* p, int64_t i, float v) { ((uint16_t*)p)[i] = (uint16_t)f32_to_bf16_bits(v); }
};


}  // namespace
