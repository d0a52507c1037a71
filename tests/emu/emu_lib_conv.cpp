// Host build of the library (lock-step emulation): the convolution kernels and their launch code.
#define TT_HOST_EMULATION 1
#include <cstdint>
namespace tt {
namespace {
alignas(16) thread_local uint16_t smem[80 * 1024]; // what the kernels' `extern __shared__ uint16_t smem[]` refers to here
}
} // namespace tt
#include "conv.hip"

static const int g_registered = emu_register_lds(tt::smem, sizeof(tt::smem));
