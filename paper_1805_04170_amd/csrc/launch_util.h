// Host-side helpers shared by the launch code of the kernel files.
#pragma once
#include "tt_device.h"
#include <cstddef>
#include <cstdlib>
#include <mutex>
#include <unordered_map>
#include "tensor_tiling.h"
#include "tt_internal.h"

namespace tt {

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
