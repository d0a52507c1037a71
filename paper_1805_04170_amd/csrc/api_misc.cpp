// Status strings and shard geometry (Def. 1 / flattening theorem of arXiv 1805.04170, Sec. 4.1 and 4.4).
#include "tt_internal.h"

extern "C" const char *tt_strerror(tt_status s)
{
    switch (s) {
    case TT_OK: return "ok";
    case TT_EINVAL: return "invalid argument";
    case TT_EINFEASIBLE: return "infeasible: uneven cut or no feasible tiling";
    case TT_EUNSUPPORTED: return "unsupported request";
    case TT_ENOMEM: return "out of host memory";
    case TT_EDEVICE: return "HIP launch failed";
    case TT_EWORKSPACE: return "workspace missing, too small or misaligned";
    }
    return "unknown status";
}

extern "C" tt_status tt_shard_shape(int64_t rows, int64_t cols, tt_tiling t, int k, int64_t *srows, int64_t *scols)
{
    if (!tt::valid_k(k) || !tt::valid_tiling(t, k) || rows < 0 || cols < 0 || !srows || !scols) return TT_EINVAL;
    tt::Grid g;
    if (!tt::make_grid(t.cut, k, rows, cols, &g)) return TT_EINFEASIBLE;
    *srows = g.srows;
    *scols = g.scols;
    return TT_OK;
}
