// Launch parameters of the persistent engine (gemm_core3.h) and of the 256 x 128 engine (gemm_core4.h): what the
// kernels assume about a product is checked here, on the host, and the grid geometry is derived here.  Shared by the
// launchers and by the host build that checks the kernels' memory accesses, so that both see the same geometry.
#pragma once
#include <cstdint>
#include "gemm_core3.h"
#include "gemm_core4.h"
#include "tt_internal.h"

namespace tt {

// tile_m x tile_n output tiles, K tiles of k_tile; cus: compute units to fill (persistent engine; 0: one workgroup per
// output tile).  Returns TT_EUNSUPPORTED when the engine does not take the product.
inline tt_status fill_params3(core3::Params3 *p, int tile_m, int tile_n, int k_tile, int cus, int count, const void *const *A,
                              const void *const *B, void *const *C, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb,
                              int64_t ldc, bool a_kc, bool b_kc, int relu, int ksplit, int64_t kchunk)
{
    if (K <= 0 || K % k_tile || (ksplit > 1 && kchunk % k_tile) || M < 8 || N < 8) return TT_EUNSUPPORTED;
    if (count * ksplit > 64 || count < 1) return TT_EUNSUPPORTED;
    if ((!a_kc && M % 8) || (!b_kc && N % 8)) return TT_EUNSUPPORTED;
    if (M * K >= (int64_t(1) << 31) || K * N >= (int64_t(1) << 31)) return TT_EUNSUPPORTED; // 32-bit byte offsets
    for (int i = 0; i < 64; ++i) {
        p->A[i] = i < count ? A[i] : nullptr;
        p->B[i] = i < count ? B[i] : nullptr;
        p->C[i] = i < count * ksplit ? C[i] : nullptr;
    }
    p->M = (int32_t)M; p->N = (int32_t)N; p->K = (int32_t)K;
    p->lda = (int32_t)lda; p->ldb = (int32_t)ldb; p->ldc = (int32_t)ldc;
    p->tiles_m = (int32_t)((M + tile_m - 1) / tile_m);
    p->tiles_n = (int32_t)((N + tile_n - 1) / tile_n);
    const int64_t total = (int64_t)p->tiles_m * p->tiles_n * count * ksplit;
    if (total >= (int64_t(1) << 30)) return TT_EUNSUPPORTED;
    p->total = (int32_t)total;
    p->per_xcd = (int32_t)((total + core::kXcds - 1) / core::kXcds);
    p->wg_per_xcd = p->per_xcd;
    if (cus > 0) {
        const int per_xcd_cus = cus / core::kXcds > 0 ? cus / core::kXcds : 1;
        if (per_xcd_cus < p->wg_per_xcd) p->wg_per_xcd = per_xcd_cus;
    }
    p->relu = relu;
    p->ksplit = ksplit;
    p->kchunk = (int32_t)(ksplit > 1 ? kchunk : K);
    return TT_OK;
}

} // namespace tt
