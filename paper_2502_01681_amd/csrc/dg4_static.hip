// dg4_qkv_proj for callers that cannot allocate device memory (code under HIP graph capture, tight
// serving loops): the packed copy of the weight, which dg4_qkv_proj keeps in a workspace the caller
// brings, lives in a file-scope device array instead. Nothing here (nor below it) calls hipMalloc,
// hipFree or any allocating routine.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "dg4_internal.h"

// 512 KB: every supported shape but fp32 with hidden 256 (768 KB), which is turned away.
static __device__ __align__(256) unsigned char scratch[DG4_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
void* g_scratch[MAX_DEVICES];       // per device: the address of ITS copy of the array (null: not asked yet)

// The device address of `scratch` on the current device. In host code the array's name is only a
// handle for the runtime; the address comes from hipGetSymbolAddress, once per device.
int scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return DG4_EHIP;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return DG4_EHIP;
        g_scratch[dev] = ptr;
    }
    *out = g_scratch[dev];
    return DG4_OK;
}

}  // namespace

extern "C" int64_t dg4_static_scratch_bytes(void) { return DG4_STATIC_SCRATCH_BYTES; }

extern "C" int dg4_qkv_proj_static(const dg4_layer_cfg* cfg, const void* S, int64_t row_begin, int64_t row_end,
                                   const void* Wqkv, void* Q, void* K, void* V, void* stream)
{
    const int rc = dg4_qkv_proj_check(cfg, S, row_begin, row_end, Wqkv, Q, K, V);
    if (rc != DG4_OK) return rc;
    // the packed weight must fit the array (checked before any device call)
    if (dg4_proj_workspace_bytes(cfg) > (int64_t)DG4_STATIC_SCRATCH_BYTES) return DG4_EWORKSPACE;
    if (row_end == row_begin) return DG4_OK;
    void* packed = nullptr;
    const int rs = scratch_of_current_device(&packed);
    if (rs != DG4_OK) return rs;
    // every byte of the packed weight that the product reads is rewritten by this call's packing
    // kernel, on the same stream, before it: nothing of an earlier call's contents is used
    return dg4_qkv_proj_run(cfg, S, row_begin, row_end, Wqkv, Q, K, V, packed, (hipStream_t)stream);
}
