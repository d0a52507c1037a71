// Convolution layer entry points.  The implicit-GEMM kernels are not in this build yet: the calls validate their
// arguments and report TT_EUNSUPPORTED so that callers fail loudly instead of silently computing nothing.
#include "exec_common.h"

extern "C" tt_status tt_conv_workspace_bytes(const tt_layer *layer, int64_t, int, int, int, tt_tiling, tt_tiling,
                                             tt_tiling, tt_tiling, tt_tiling, const uint8_t *, const uint8_t *, int,
                                             size_t *bytes)
{
    if (!layer || !bytes) return TT_EINVAL;
    return TT_EUNSUPPORTED;
}
extern "C" tt_status tt_conv_forward(const tt_layer *layer, int64_t, int, int, tt_tiling, tt_tiling, tt_tiling,
                                     const uint8_t *, const void *const *, const void *const *, void *const *, void *,
                                     size_t, void *)
{
    if (!layer) return TT_EINVAL;
    return TT_EUNSUPPORTED;
}
extern "C" tt_status tt_conv_backward(const tt_layer *layer, int64_t, int, int, tt_tiling, tt_tiling, tt_tiling,
                                      tt_tiling, tt_tiling, const uint8_t *, const uint8_t *, const void *const *,
                                      const void *const *, const void *const *, const void *const *, void *const *,
                                      void *const *, void *, size_t, void *)
{
    if (!layer) return TT_EINVAL;
    return TT_EUNSUPPORTED;
}
