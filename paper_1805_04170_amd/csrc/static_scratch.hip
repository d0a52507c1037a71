// tt_fc_forward_static: the forward execute call for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  Same three phases as tt_fc_forward (Sec. 4.2.1 /
// Sec. 5.2 of arXiv 1805.04170); the scratch that the conversion, product and reduction kernels need (aligned copies of
// the operands, fp32 partial sums of reduction cuts) lives in a device array that is part of this library's code
// object instead of a caller's workspace.
//
// The array's name is only a host-side handle: host code must never pass it to a kernel or a copy.  Its device
// address is looked up once per device with hipGetSymbolAddress (every GPU holds its own copy at its own address) and
// only that address is used afterwards.
#include "tt_device.h"
#include <cstddef>
#include <cstdint>
#include <mutex>
#include "tensor_tiling.h"

namespace {

constexpr size_t kScratchBytes = TT_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::once_flag g_once[kMaxDevices];
void *g_ptr[kMaxDevices];      // device address of this device's copy of the array; written once, under g_once
tt_status g_status[kMaxDevices];

// address of the current device's scratch array
tt_status scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TT_EDEVICE;
    std::call_once(g_once[dev], [dev] {
        void *p = nullptr;
        // the calling thread's current device is `dev`: the lookup returns that device's copy
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        g_ptr[dev] = e == hipSuccess ? p : nullptr;
        g_status[dev] = (e == hipSuccess && p && (reinterpret_cast<uintptr_t>(p) & 255) == 0) ? TT_OK : TT_EDEVICE;
    });
    if (g_status[dev] != TT_OK) return g_status[dev];
    *out = g_ptr[dev];
    return TT_OK;
}

} // namespace

extern "C" tt_status tt_fc_forward_static(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                                          tt_tiling tY, const uint8_t *forms, const void *const *X, const void *const *W,
                                          void *const *Y, void *stream)
{
    size_t need = 0;
    tt_status st = tt_fc_workspace_bytes(layer, batch, k, dtype, TT_OP_FWD, tX, tW, tY, tY, tX, forms, nullptr, 0, &need);
    if (st != TT_OK) return st;
    if (need > kScratchBytes) return TT_EWORKSPACE; // the layer needs more scratch than the library holds
    void *ws = nullptr;
    if ((st = scratch_of_current_device(&ws)) != TT_OK) return st;
    // every scratch block is written in full (by a conversion or a product) before anything reads it, so nothing
    // has to be cleared between calls although the array keeps the last call's contents
    return tt_fc_forward(layer, batch, k, dtype, tX, tW, tY, forms, X, W, Y, ws, kScratchBytes, stream);
}
