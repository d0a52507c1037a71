// Host build of the library (lock-step emulation): the shard-product kernels and their launch code.
#define TT_HOST_EMULATION 1
#include <cstdint>
namespace tt {
namespace {
// what the kernels' `extern __shared__` arrays refer to here (one name per kernel family)
alignas(16) thread_local uint16_t smem[80 * 1024];
alignas(16) thread_local char smem2[160 * 1024], smem3[160 * 1024], smem4[160 * 1024];
}
} // namespace tt
#include "gemm.hip"
#include "gemm3.hip"

// (registered by the thread that loads the library, which is the one that calls it)
static const int g_registered = (emu_register_lds(tt::smem, sizeof(tt::smem)), emu_register_lds(tt::smem2, sizeof(tt::smem2)),
                                 emu_register_lds(tt::smem3, sizeof(tt::smem3)), emu_register_lds(tt::smem4, sizeof(tt::smem4)));
