// Host-side helpers shared by the launch code of the kernel files.
#pragma once
#include "tt_device.h"
#include <cstddef>
#include <cstdlib>
#include <mutex>
#include <unordered_map>
#include "tensor_tiling.h"

namespace tt {

// Launch heuristics can be overridden through environment variables only in development builds (-DTT_TUNING); the
// product build reads no environment and every launch decision is a pure function of the call's arguments.
inline int tuning_int(const char *name, int dflt)
{
#ifdef TT_TUNING
    const char *e = std::getenv(name);
    return e ? std::atoi(e) : dflt;
#else
    (void)name;
    return dflt;
#endif
}

// Kernels that use more dynamic LDS than the default limit need the limit raised once per kernel.  The set of kernels
// already raised is the only state the launch code keeps; it is guarded, and raising twice would be harmless.
inline tt_status ensure_dynamic_lds(const void *kernel, size_t bytes)
{
    static std::mutex mu;
    static std::unordered_map<const void *, size_t> done;
    std::lock_guard<std::mutex> lock(mu);
    auto it = done.find(kernel);
    if (it != done.end() && it->second >= bytes) return TT_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return TT_EDEVICE;
    done[kernel] = bytes;
    return TT_OK;
}

} // namespace tt
