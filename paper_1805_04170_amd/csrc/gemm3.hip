// Shard products on the persistent, software-pipelined MFMA engine (gemm_core3.h): kernels and launcher.
// One launch covers all shards (Sec. 5.2 step 2 of arXiv 1805.04170: every device runs the same sub-operator on its
// own tiles); the grid is one workgroup per CU and each workgroup walks its share of the 256 x 256 output tiles.
#include "tt_device.h"
#include <cstdint>
#include <cstdlib>
#include "gemm_core3.h"
#include "gemm_core4.h"
#include "gemm_core5.h"
#include "gemm_core6.h"
#include "gemm3_params.h"
#include "tt_internal.h"
#include "launch_util.h"

namespace tt {
namespace {

template <int BK, int NS, bool A_KC, bool B_KC, bool OUT_BF16, bool STAGED, bool ILV>
__global__ __launch_bounds__(core3::kThreads3, 2) void gemm_bf16_v3_kernel(const core3::Params3 p)
{
    extern __shared__ __attribute__((aligned(16))) char smem3[];
    core3::run_tiles<BK, NS, A_KC, B_KC, OUT_BF16, STAGED, ILV>(p, smem3);
}

// 256 x 128 tiles, four waves, two workgroups per CU (gemm_core4.h); one tile per workgroup
template <bool A_KC, bool B_KC, bool OUT_BF16, bool STAGED>
__global__ __launch_bounds__(core4::kThreads4, 2) void gemm_bf16_v4_kernel(const core3::Params3 p)
{
    extern __shared__ __attribute__((aligned(16))) char smem4[];
    const int logical = core::logical_block(p.per_xcd, p.total);
    if (logical < 0) return;
    const int tiles = p.tiles_m * p.tiles_n;
    const int vshard = logical / tiles;
    const int t = logical - vshard * tiles;
    int tm, tn;
    core::grouped_tile(t, p.tiles_m, p.tiles_n, &tm, &tn);
    const int shard = vshard / p.ksplit;
    const int kbeg = (vshard - shard * p.ksplit) * p.kchunk;
    const int klen = p.K - kbeg < p.kchunk ? p.K - kbeg : p.kchunk;
    const char *abase = reinterpret_cast<const char *>(p.A[shard]) + (size_t)kbeg * (A_KC ? 2 : 2 * (size_t)p.lda);
    const char *bbase = reinterpret_cast<const char *>(p.B[shard]) + (size_t)kbeg * (B_KC ? 2 : 2 * (size_t)p.ldb);
    core4::tile_product4<A_KC, B_KC, OUT_BF16, STAGED>(abase, p.lda, bbase, p.ldb, p.C[vshard], p.ldc, p.M, p.N, klen,
                                                       tm * core4::BM4, tn * core4::BN4, p.relu != 0, smem4);
}

template <bool A_KC, bool B_KC, bool OUT_BF16, bool STAGED> tt_status launch_cfg4(core3::Params3 &p, hipStream_t s)
{
    auto kern = gemm_bf16_v4_kernel<A_KC, B_KC, OUT_BF16, STAGED>;
    if (ensure_dynamic_lds(reinterpret_cast<const void *>(kern), core4::kSmem4) != TT_OK) return TT_EDEVICE;
    hipLaunchKernelGGL(kern, dim3((uint32_t)p.per_xcd * core::kXcds), dim3(core4::kThreads4), core4::kSmem4, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

template <bool A_KC, bool B_KC> tt_status launch_layout4(core3::Params3 &p, int out_dtype, bool vec, hipStream_t s)
{
    const bool bf = out_dtype == TT_BF16;
    if (vec) return bf ? launch_cfg4<A_KC, B_KC, true, true>(p, s) : launch_cfg4<A_KC, B_KC, false, true>(p, s);
    return bf ? launch_cfg4<A_KC, B_KC, true, false>(p, s) : launch_cfg4<A_KC, B_KC, false, false>(p, s);
}

// skinny products with both operands K-contiguous: 256 x 128 tiles, K tiles of 64, one workgroup per CU (gemm_core6.h)
template <bool B_KC, bool OUT_BF16, bool STAGED>
__global__ __launch_bounds__(core6::kThreads6, 1) void gemm_bf16_v6_kernel(const core3::Params3 p)
{
    extern __shared__ __attribute__((aligned(16))) char smem4[];
    const int logical = core::logical_block(p.per_xcd, p.total);
    if (logical < 0) return;
    const int tiles = p.tiles_m * p.tiles_n;
    const int vshard = logical / tiles;
    const int t = logical - vshard * tiles;
    int tm, tn;
    core::grouped_tile(t, p.tiles_m, p.tiles_n, &tm, &tn);
    const int shard = vshard / p.ksplit;
    const int kbeg = (vshard - shard * p.ksplit) * p.kchunk;
    const int klen = p.K - kbeg < p.kchunk ? p.K - kbeg : p.kchunk;
    const char *abase = reinterpret_cast<const char *>(p.A[shard]) + (size_t)kbeg * 2;
    const char *bbase = reinterpret_cast<const char *>(p.B[shard]) + (size_t)kbeg * (B_KC ? 2 : 2 * (size_t)p.ldb);
    core6::tile_product6<B_KC, OUT_BF16, STAGED>(abase, p.lda, bbase, p.ldb, p.C[vshard], p.ldc, p.M, p.N, klen, tm * core6::BM6,
                                           tn * core6::BN6, p.relu != 0, smem4);
}

template <bool B_KC, bool OUT_BF16, bool STAGED> tt_status launch_cfg6(core3::Params3 &p, hipStream_t s)
{
    auto kern = gemm_bf16_v6_kernel<B_KC, OUT_BF16, STAGED>;
    if (ensure_dynamic_lds(reinterpret_cast<const void *>(kern), core6::kSmem6) != TT_OK) return TT_EDEVICE;
    hipLaunchKernelGGL(kern, dim3((uint32_t)p.per_xcd * core::kXcds), dim3(core6::kThreads6), core6::kSmem6, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

// short-K products with the left operand's panel held in registers (gemm_core5.h); two workgroups per CU
template <int KT, bool NTS> __global__ __launch_bounds__(core5::kThreads5, KT <= 16 ? 2 : 1) void gemm_bf16_v5_kernel(const core5::Params5 p)
{
    extern __shared__ __attribute__((aligned(16))) char smem3[];
    core5::run_panels<KT, NTS>(p, smem3);
}

template <int KT, bool NTS> tt_status launch_cfg5(core5::Params5 &p, hipStream_t s)
{
    auto kern = gemm_bf16_v5_kernel<KT, NTS>;
    constexpr size_t smem = core5::smem_bytes5<KT>();
    if (ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem) != TT_OK) return TT_EDEVICE;
    hipLaunchKernelGGL(kern, dim3((uint32_t)p.grid), dim3(core5::kThreads5), smem, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

int cu_count()
{
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
        return cus;
    }();
    return n;
}

template <int BK, int NS, bool A_KC, bool B_KC, bool OUT_BF16, bool STAGED, bool ILV = false>
tt_status launch_cfg(core3::Params3 &p, hipStream_t s)
{
    auto kern = gemm_bf16_v3_kernel<BK, NS, A_KC, B_KC, OUT_BF16, STAGED, ILV>;
    constexpr size_t smem = core3::smem_bytes3<BK, NS, STAGED>();
    if (ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem) != TT_OK) return TT_EDEVICE;
    hipLaunchKernelGGL(kern, dim3((uint32_t)p.wg_per_xcd * core::kXcds), dim3(core3::kThreads3), smem, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

template <bool A_KC, bool B_KC> tt_status launch_layout(core3::Params3 &p, int out_dtype, bool vec, hipStream_t s)
{
    // results with 16-byte rows: staged epilogue (ring + 18 KB).  Odd pitches store element-wise from registers.  Ring: two stages of 64 (TT_V3_RING=324: four stages of 32; tuning aid).
    const int ring = tuning_int("TT_V3_RING", 642);
    const bool bf = out_dtype == TT_BF16;
    if (ring == 324) {
        if (bf && vec) return launch_cfg<32, 4, A_KC, B_KC, true, true>(p, s);
        return bf ? launch_cfg<32, 4, A_KC, B_KC, true, false>(p, s) : launch_cfg<32, 4, A_KC, B_KC, false, false>(p, s);
    }
    // short K loops (the weight gradients at batch 256): loads issued between the k-steps, see run_tiles
    // Loads issued between the k-steps (see run_tiles) measured faster for the products with bf16 results (the weight
    // gradients: short K loops) ...  (TT_V3_ILV=0: never; tuning aid.)
    const bool ilv = tuning_int("TT_V3_ILV", 1) != 0;
    if (bf && vec) return ilv ? launch_cfg<64, 2, A_KC, B_KC, true, true, true>(p, s) : launch_cfg<64, 2, A_KC, B_KC, true, true>(p, s);
    // ... and, among the products that write fp32 partial sums, for the NN layout (B read with LDS transpose reads)
    if constexpr (A_KC && !B_KC)
        if (!bf && ilv) return vec ? launch_cfg<64, 2, A_KC, B_KC, false, true, true>(p, s) : launch_cfg<64, 2, A_KC, B_KC, false, false, true>(p, s);
    if (!bf && vec) return launch_cfg<64, 2, A_KC, B_KC, false, true>(p, s); // fp32 partial sums with 16-byte rows: staged too
    return bf ? launch_cfg<64, 2, A_KC, B_KC, true, false>(p, s) : launch_cfg<64, 2, A_KC, B_KC, false, false>(p, s);
}

} // namespace

// C_s = A_s^T B_s, A_s stored K x M, B_s stored K x N, K = 128, 256 or 512, bf16 result with 16-byte rows.
// TT_EUNSUPPORTED when the engine does not take the product.
tt_status launch_gemm_v5(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                         int64_t K, int64_t lda, int64_t ldb, int64_t ldc, int relu, void *stream)
{
    if ((K != 128 && K != 256 && K != 512) || N < core5::NT5 || N % core5::NT5 || M < 8 || M % 8 || count < 1 || count > 64)
        return TT_EUNSUPPORTED;
    if (lda % 8 || ldb % 8 || ldc % 8 || lda < M || ldb < N || ldc < N) return TT_EUNSUPPORTED; // 16-byte chunks and rows
    if (K * lda >= (int64_t(1) << 30) || K * ldb >= (int64_t(1) << 30)) return TT_EUNSUPPORTED; // 32-bit byte offsets
    core5::Params5 p;
    for (int i = 0; i < 64; ++i) {
        p.A[i] = i < count ? A[i] : nullptr;
        p.B[i] = i < count ? B[i] : nullptr;
        p.C[i] = i < count ? C[i] : nullptr;
    }
    p.M = (int32_t)M; p.N = (int32_t)N;
    p.lda = (int32_t)lda; p.ldb = (int32_t)ldb; p.ldc = (int32_t)ldc;
    p.panels = (int32_t)((M + core5::PM5 - 1) / core5::PM5);
    p.ntiles = (int32_t)(N / core5::NT5);
    const int64_t total = (int64_t)count * p.panels * p.ntiles;
    if (total >= (int64_t(1) << 30)) return TT_EUNSUPPORTED;
    p.total = (int32_t)total;
    const int64_t resident = (K <= 256 ? 2 : 1) * (int64_t)cu_count(); // two workgroups per CU; one at K = 512
    p.grid = (int32_t)(total < resident ? total : resident);
    p.relu = relu;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const bool nts = tuning_int("TT_V5_NT", 1) != 0;
    if (K == 512) return nts ? launch_cfg5<32, true>(p, s) : launch_cfg5<32, false>(p, s);
    if (K == 256) return nts ? launch_cfg5<16, true>(p, s) : launch_cfg5<16, false>(p, s);
    return nts ? launch_cfg5<8, true>(p, s) : launch_cfg5<8, false>(p, s);
}

tt_status launch_gemm_v4(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                         int64_t K, int64_t lda, int64_t ldb, int64_t ldc, bool a_kc, bool b_kc, int out_dtype, int relu,
                         bool vec, int ksplit, int64_t kchunk, void *stream)
{
    core3::Params3 p;
    const tt_status st = fill_params3(&p, core4::BM4, core4::BN4, core4::BK4, 0, count, A, B, C, M, N, K, lda, ldb, ldc, a_kc,
                                      b_kc, relu, ksplit, kchunk);
    if (st != TT_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (a_kc && b_kc) return launch_layout4<true, true>(p, out_dtype, vec, s);
    if (a_kc && !b_kc) return launch_layout4<true, false>(p, out_dtype, vec, s);
    if (!a_kc && !b_kc) return launch_layout4<false, false>(p, out_dtype, vec, s);
    return launch_layout4<false, true>(p, out_dtype, vec, s);
}

// C_s = A_s B_s with A's rows K-contiguous (B either way), K (and a K chunk) a multiple of 64.
tt_status launch_gemm_v6(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                         int64_t K, int64_t lda, int64_t ldb, int64_t ldc, bool b_kc, int out_dtype, int relu, bool vec,
                         int ksplit, int64_t kchunk, void *stream)
{
    core3::Params3 p;
    const tt_status st = fill_params3(&p, core6::BM6, core6::BN6, core6::BK6, 0, count, A, B, C, M, N, K, lda, ldb, ldc, true, b_kc,
                                      relu, ksplit, kchunk);
    if (st != TT_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const bool bf = out_dtype == TT_BF16;
    if (b_kc) {
        if (vec) return bf ? launch_cfg6<true, true, true>(p, s) : launch_cfg6<true, false, true>(p, s);
        return bf ? launch_cfg6<true, true, false>(p, s) : launch_cfg6<true, false, false>(p, s);
    }
    if (vec) return bf ? launch_cfg6<false, true, true>(p, s) : launch_cfg6<false, false, true>(p, s);
    return bf ? launch_cfg6<false, true, false>(p, s) : launch_cfg6<false, false, false>(p, s);
}

tt_status launch_gemm_v3(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                         int64_t K, int64_t lda, int64_t ldb, int64_t ldc, bool a_kc, bool b_kc, int out_dtype, int relu,
                         bool vec, int ksplit, int64_t kchunk, void *stream)
{
    core3::Params3 p;
    const tt_status st = fill_params3(&p, core3::BM3, core3::BN3, 64, cu_count(), count, A, B, C, M, N, K, lda, ldb, ldc, a_kc,
                                      b_kc, relu, ksplit, kchunk);
    if (st != TT_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (a_kc && b_kc) return launch_layout<true, true>(p, out_dtype, vec, s);
    if (a_kc && !b_kc) return launch_layout<true, false>(p, out_dtype, vec, s);
    if (!a_kc && !b_kc) return launch_layout<false, false>(p, out_dtype, vec, s);
    return launch_layout<false, true>(p, out_dtype, vec, s);
}

} // namespace tt
