// The level sweep as one persistent dataflow kernel, for every shape: fp32 or bf16, hidden 128 or 256,
// cones of up to three hops (neighbour rows of 8 or 16 entries), any number of stacked layers.
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
// Per tile: wait for the "published" flags of the sources of its gates; then per layer the attention
// over the cone rows (lanes split the feature dimension, attend_core), the output projection with
// residual + LayerNorm on the matrix cores (the four waves split the columns, the packed weight
// streams from the L2 cache through a ring of fragments), and the Q | K | V projection of the new
// state for the next layer, into LDS; after the last layer the embeddings go out and K | V of every
// layer are projected from them into the store of finished gates, followed by a device-scope
// release and the flags. The arithmetic of a row is, operation for operation, that of the
// level-by-level kernels (attn_kernel, gemm_ln_split_kernel, gemm_kernel): same bits.
//
// Visibility between compute units follows the memory model as the compiler implements it for
// gfx950: a writer's rows are ordinary stores followed by a release fence at agent scope (every
// thread, for its own stores), a workgroup barrier, and release stores of the flags; a reader polls
// the flags with agent-scope atomic loads and issues an acquire fence at agent scope before the
// first load of a source row. No row is read before its flag has been seen.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "dg4_device.h"
#include "dg4_internal.h"
#include "dg4_rowops.h"

namespace {

constexpr int FT = 32;                    // gates per tile

// compile-time loop: f(integral_constant<int, I>) for I = 0 .. N-1
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

template <typename T, int D>
struct FlowShape {
    static constexpr int E = 16 / (int)sizeof(T);     // elements per 16 bytes
    static constexpr int KC = D / (2 * E);            // k-chunks of a product (16 for both supported shapes... checked below)
    static constexpr int YS = D + E;                  // row stride of a staged row (16 bytes of padding)
    static constexpr int QS = 3 * D + E;              // row stride of the staged Q | K | V rows
    static constexpr int TS = 32 + E;                 // row stride of a staged 32x32 output tile
    static constexpr int CPR = D / E;                 // 16-byte pieces per row
    static constexpr int TPR = 32 / E;                // 16-byte pieces per row of a 32x32 tile
    static constexpr int RING = 16;
    static constexpr size_t row_buf = (size_t)FT * YS * sizeof(T);
    static constexpr size_t tile_buf = (size_t)4 * 32 * TS * sizeof(T);
    static constexpr size_t part_buf = 2 * 4 * 32 * sizeof(float);
    static constexpr size_t ctl_buf = 16;
    static constexpr size_t qkv_buf = (size_t)FT * QS * sizeof(T);
    static constexpr size_t smem(bool multi) { return 2 * row_buf + tile_buf + part_buf + ctl_buf + (multi ? qkv_buf : 0); }
};

// rows [32] x packed weight columns: the fragments of `n_tiles` column tiles, KC each, starting at
// column tile `first_tile` of the stream wp (already offset by the lane), through a ring of KC
// fragments requested one tile ahead. emit(column tile, accumulator) is called per finished tile.
template <typename T, int KC, typename F>
__device__ __forceinline__ void stream_product(const uint4 (&a)[KC], const uint4* wp, int first_tile, int n_tiles, F&& emit)
{
    static_assert(KC == 16, "the ring is one column tile deep");
    uint4 ring[KC];
    const uint4* w = wp + (int64_t)first_tile * KC * 64;
#pragma unroll
    for (int c = 0; c < KC; ++c) ring[c] = w[c * 64];
#pragma unroll 1
    for (int t = 0; t < n_tiles; ++t) {
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        const bool more = t + 1 < n_tiles;
        const uint4* wn = w + (int64_t)(t + 1) * KC * 64;
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            Mma<T>::run(a[c], ring[c], acc);
            if (more) ring[c] = wn[c * 64];
        }
        emit(first_tile + t, acc);
    }
}
// the same for a number of tiles known at compile time: emit(index 0 .. NT-1 as a constant, accumulator)
template <typename T, int KC, int NT, typename F>
__device__ __forceinline__ void stream_product_fixed(const uint4 (&a)[KC], const uint4* wp, int first_tile, F&& emit)
{
    static_assert(KC == 16, "the ring is one column tile deep");
    uint4 ring[KC];
    const uint4* w = wp + (int64_t)first_tile * KC * 64;
#pragma unroll
    for (int c = 0; c < KC; ++c) ring[c] = w[c * 64];
    static_for<0, NT>([&](auto I) __attribute__((always_inline)) {
        constexpr int t = I.value;
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            Mma<T>::run(a[c], ring[c], acc);
            if (t + 1 < NT) ring[c] = w[((t + 1) * KC + c) * 64];
        }
        emit(I, acc);
    });
}

template <typename T, int D, int AW>
__global__ __launch_bounds__(256) void flow_kernel(dg4_flow_args p)
{
    using S = FlowShape<T, D>;
    constexpr int E = S::E, KC = S::KC, YS = S::YS, QS = S::QS, TS = S::TS, CPR = S::CPR, TPR = S::TPR;
    constexpr int EPL = Elem<T>::EPL, LPR = D / EPL;
    static_assert(LPR == 16 && AW <= LPR, "one lane per neighbour entry while waiting");
    static_assert(KC == 16, "fp32 with hidden 128 or bf16 with hidden 256");
    constexpr int NTW = D / 32 / 4;               // column tiles of the output projection per wave
    constexpr int PPT = FT * CPR / 256;           // 16-byte pieces of the tile's rows per thread

    extern __shared__ __attribute__((aligned(16))) unsigned char flow_smem[];
    T* buf0 = (T*)flow_smem;
    T* buf1 = (T*)(flow_smem + S::row_buf);
    T* stage = (T*)(flow_smem + 2 * S::row_buf);                       // [4][32 * TS]
    float (*part)[4][32] = (float (*)[4][32])(flow_smem + 2 * S::row_buf + S::tile_buf);
    int* ctl = (int*)(flow_smem + 2 * S::row_buf + S::tile_buf + S::part_buf);     // [0] ticket, [1] abort
    T* qkvbuf = (T*)(flow_smem + 2 * S::row_buf + S::tile_buf + S::part_buf + S::ctl_buf);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, kg = lane >> 5;
    const int group = tid / LPR, sub = tid % LPR;  // attention role: rows `group` and `group + 16` of the tile
    const int L = p.n_layers;

    if (tid == 0) ctl[1] = 0;
    for (;;) {
        if (tid == 0) ctl[0] = (int)__hip_atomic_fetch_add(&p.ctrl[2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();                          // (also: the previous tile is done with every buffer)
        const int64_t t = ctl[0];
        if (t >= p.n_tiles || ctl[1]) break;
        int64_t p0;
        int rows;
        if (p.pairs) {
            const uint2 ta = p.tiles[p.tile_begin + 2 * t], tb = p.tiles[p.tile_begin + 2 * t + 1];
            p0 = ta.x; rows = (int)(ta.y + tb.y);
        } else {
            const uint2 ta = p.tiles[p.tile_begin + t];
            p0 = ta.x; rows = (int)ta.y;
        }
        // rows past the end of a ragged tile repeat its last gate: computed, never stored
        auto pos_of = [&](int r) { return p0 + (r < rows ? r : rows - 1); };

        T* resid = buf0;                          // the running state s_l
        T* ybuf = buf1;                           // attention output, then the normalised rows

        // s_0 = X rows of the tile's gates, as 16-byte pieces
        int64_t pidx[PPT];                        // node id of the piece's row (-1: past the end)
#pragma unroll
        for (int q = 0; q < PPT; ++q) {
            const int piece = tid + 256 * q, row = piece / CPR, c = piece % CPR;
            const int64_t id = p.order[pos_of(row)];
            pidx[q] = row < rows ? id : -1;
            *(uint4*)&resid[row * YS + c * E] = *((const uint4*)((const T*)p.x + id * D) + c);
        }

        // ---- the sources of this wave's eight gates must be published: lane `sub` of a gate's
        // group watches entry `sub` of the gate's row
        {
            const int64_t ra = pos_of(group), rb = pos_of(group + 16);
            const uint32_t ea = sub < AW ? p.ell[ra * AW + sub] : DG4_ELL_PAD;
            const uint32_t eb = sub < AW ? p.ell[rb * AW + sub] : DG4_ELL_PAD;
            const bool wa = ea != DG4_ELL_PAD && (ea >> 30) != 0, wb = eb != DG4_ELL_PAD && (eb >> 30) != 0;
            const uint32_t* fa = p.flags + (wa ? (ea & 0x3FFFFFFFu) : 0u);
            const uint32_t* fb = p.flags + (wb ? (eb & 0x3FFFFFFFu) : 0u);
            uint32_t spins = 0;
            for (;;) {
                const bool ok = (!wa || __hip_atomic_load(fa, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) &&
                                (!wb || __hip_atomic_load(fb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u);
                if (__ballot(!ok) == 0) break;
                __builtin_amdgcn_s_sleep(2);
                if (++spins > p.spin_limit ||
                    ((spins & 63u) == 0 && __hip_atomic_load(&p.ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                    // give up: the tile is computed from whatever is there (every access stays in
                    // bounds), nothing of it is published, and the workgroup leaves after it
                    if (lane == 0) {
                        __hip_atomic_store(&p.ctrl[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        ctl[1] = 1;
                    }
                    break;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }

        for (int l = 0; l < L; ++l) {
            const bool last = l == L - 1;
            // ---- attention of layer l: the gate's own Q, K, V from the projection of x (layer 0) or
            // from LDS (its running state, projected at the end of the previous layer); sources from
            // the store of finished gates, layer l
            {
                const T* kvl = (const T*)p.kv + (int64_t)l * p.kv_layer_stride;
                const float* bias = p.rel_bias + l * (D / 32) * 4;
#pragma unroll 1
                for (int rr = group; rr < FT; rr += 256 / LPR) {
                    const int64_t pos = pos_of(rr);
                    uint32_t ent[AW];
                    load_entries<AW>(p.ell, pos, ent);
                    const T* qrow = l == 0 ? (const T*)p.qkv_self + pos * (3 * D) : qkvbuf + (rr < rows ? rr : rows - 1) * QS;
                    float av[EPL];
                    attend_core<T, D, AW>(ent, qrow, qrow + D, qrow + 2 * D, kvl, kvl + D, 2 * D, bias, sub, av);
                    uint4 oa, ob;
                    Elem<T>::pack(av, oa, ob);
                    uint4* op = (uint4*)&ybuf[rr * YS + sub * EPL];
                    op[0] = oa; op[1] = ob;
                }
            }
            __syncthreads();
            // ---- s_{l+1} = LN(s_l + a Wo_l): wave w takes columns [w*NTW*32, (w+1)*NTW*32)
            uint4 a[KC];
#pragma unroll
            for (int c = 0; c < KC; ++c) a[c] = *(const uint4*)&ybuf[m * YS + (2 * c + kg) * E];
            f32x16 acc[NTW];
            {
                const uint4* wp = (const uint4*)((const char*)p.wo_packed + (int64_t)l * p.w_layer_stride) + lane;
                stream_product_fixed<T, KC, NTW>(a, wp, wave * NTW, [&](auto NT, const f32x16& v) __attribute__((always_inline)) {
                    acc[NT.value] = v;
                });
            }
            __syncthreads();                      // every wave holds its operand: ybuf may be written
            const int col0 = wave * NTW * 32 + m;
            if (p.epilogue) {
                float mean[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = 8 * (i / 4) + 4 * kg + (i % 4);
                    float s1 = 0.f;
#pragma unroll
                    for (int nt = 0; nt < NTW; ++nt) {
                        acc[nt][i] += Elem<T>::load1(resid, (int64_t)row * YS + col0 + nt * 32);
                        s1 += acc[nt][i];
                    }
                    s1 = sum_over_32_lanes(s1);
                    if (m == 0) part[0][wave][row] = s1;
                }
                __syncthreads();
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = 8 * (i / 4) + 4 * kg + (i % 4);
                    mean[i] = (part[0][0][row] + part[0][1][row] + part[0][2][row] + part[0][3][row]) * (1.0f / D);
                    float s2 = 0.f;
#pragma unroll
                    for (int nt = 0; nt < NTW; ++nt) { const float t2 = acc[nt][i] - mean[i]; s2 = fmaf(t2, t2, s2); }
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
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = 8 * (i / 4) + 4 * kg + (i % 4);
#pragma unroll
                    for (int nt = 0; nt < NTW; ++nt) Elem<T>::store1(ybuf, (int64_t)row * YS + col0 + nt * 32, acc[nt][i]);
                }
            }
            __syncthreads();                      // ybuf = s_{l+1}, rounded to T
#pragma unroll
            for (int c = 0; c < KC; ++c) a[c] = *(const uint4*)&ybuf[m * YS + (2 * c + kg) * E];

            if (!last) {
                // ---- Q | K | V of the new state for the next layer, into LDS: wave w takes a quarter of the 3D columns
                constexpr int NTQ = 3 * D / 32 / 4;
                const uint4* wp = (const uint4*)((const char*)p.wqkv_packed + (int64_t)(l + 1) * p.w_layer_stride) + lane;
                stream_product_fixed<T, KC, NTQ>(a, wp, wave * NTQ, [&](auto NT, const f32x16& v) __attribute__((always_inline)) {
                    const int ct = wave * NTQ + NT.value;
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        Elem<T>::store1(qkvbuf, (int64_t)(8 * (i / 4) + 4 * kg + (i % 4)) * QS + ct * 32 + m, v[i]);
                });
                // the new state is the next layer's residual; the old one's space takes the next attention output
                T* tmp = resid; resid = ybuf; ybuf = tmp;
                __syncthreads();
                continue;
            }

            // ---- the embeddings of the tile's gates go out, by node id
#pragma unroll
            for (int q = 0; q < PPT; ++q) {
                if (pidx[q] < 0) continue;
                const int piece = tid + 256 * q, row = piece / CPR, c = piece % CPR;
                *((uint4*)((T*)p.h_out + pidx[q] * D) + c) = *(const uint4*)&ybuf[row * YS + c * E];
            }
            // ---- K | V of every layer from the final embeddings: wave w takes a quarter of the 2D*L columns
            if (p.project_kv) {
                const int ntk = 2 * D / 32 * L / 4;
                const uint4* wp = (const uint4*)p.wkv_packed + lane;
                T* st = stage + wave * 32 * TS;
                stream_product<T, KC>(a, wp, wave * ntk, ntk, [&](int ct, const f32x16& v) {
                    // the 32x32 tile leaves through this wave's own corner of LDS, as 16-byte pieces of
                    // rows (LDS operations of a wave complete in order: no barrier)
#pragma unroll
                    for (int i = 0; i < 16; ++i) Elem<T>::store1(st, (int64_t)(8 * (i / 4) + 4 * kg + (i % 4)) * TS + m, v[i]);
                    const int col = ct * 32;
                    T* base = (T*)p.kv + (int64_t)(col / (2 * D)) * p.kv_layer_stride + col % (2 * D);
#pragma unroll
                    for (int q = 0; q < 32 * TPR / 64; ++q) {
                        const int piece = lane + 64 * q, row = piece / TPR, cc = piece % TPR;
                        const uint4 val = *(const uint4*)&st[row * TS + cc * E];
                        if (row < rows) *(uint4*)(base + (p0 + row) * (2 * D) + cc * E) = val;
                    }
                });
            }
        }
        // ---- publish: every thread's rows are written through before the flags go up
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
        if (ctl[1]) break;                        // an aborted tile publishes nothing
        if (tid < rows) __hip_atomic_store(&p.flags[p0 + tid], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <typename T, int D>
int launch_flow_t(const dg4_flow_args& a, hipStream_t s)
{
    using S = FlowShape<T, D>;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return hipErrorInvalidDevice;
    const size_t smem = S::smem(a.n_layers > 1);
    void (*kern)(dg4_flow_args) = a.ell_w == 8 ? flow_kernel<T, D, 8> : a.ell_w == 16 ? flow_kernel<T, D, 16> : nullptr;
    if (!kern) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    // as many workgroups as stay resident (tiles are handed out by tickets, so fewer resident ones
    // only cost speed): two per compute unit when the LDS allows it
    const int per_cu = smem * 2 <= 160 * 1024 ? 2 : 1;
    const int64_t grid = std::min<int64_t>((int64_t)cus * per_cu, a.n_tiles);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), smem, s, a);
    return hipGetLastError();
}

}  // namespace

bool dg4_flow_supports(int dtype, int hidden, int ell_w)
{
    return ((dtype == DG4_F32 && hidden == 128) || (dtype == DG4_BF16 && hidden == 256)) && (ell_w == 8 || ell_w == 16);
}

int dg4_launch_flow(int dtype, int hidden, const dg4_flow_args& a, hipStream_t s)
{
    if (a.n_tiles <= 0) return hipSuccess;
    if (!dg4_flow_supports(dtype, hidden, a.ell_w) || a.n_layers < 1) return hipErrorInvalidValue;
    return dtype == DG4_F32 ? launch_flow_t<float, 128>(a, s) : launch_flow_t<bf16_t, 256>(a, s);
}
