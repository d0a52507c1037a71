// Shard products: C_s = op(A_s) op(B_s) for all shards in one launch (Sec. 5.2 step 2 of arXiv 1805.04170:
// after input conversion every device runs the same sub-operator on its own tiles).
//
// bf16 path: the MFMA tile engine of gemm_core.h with dense-matrix loaders (NN, NT, TN, TT all share one main loop).
// fp32 path / shapes without 16-byte rows: a plain LDS-tiled FMA kernel with arbitrary strides.
#include "tt_device.h"
#include <cstdint>
#include <cstdlib>
#include <type_traits>
#include "gemm_core.h"
#include "gemm_core2.h"
#include "tt_internal.h"
#include "launch_util.h"

namespace tt {
namespace {

using core::kThreads;
using core::kXcds;
using core::f32_to_bf16_bits;

struct GemmParams {
    const void *A[kMaxShards];
    const void *B[kMaxShards];
    void *C[kMaxShards];
    int32_t M, N, K;
    int32_t lda, ldb, ldc;
    int32_t tiles_m, tiles_n;
    int32_t per_xcd;  // logical workgroups per XCD (grid = per_xcd * 8)
    int32_t total;    // tiles_m * tiles_n * count * ksplit
    int32_t relu;
    int32_t ksplit;   // each shard's K range is cut into ksplit chunks of kchunk (a multiple of 64); chunk c of shard s
    int32_t kchunk;   // writes its own output C[s * ksplit + c] (partial sums, added up by the reduction kernel)
};

template <int BM, int BN, int WM, int WN, int DEPTH, bool KMASK, bool A_KC, bool B_KC, bool OUT_BF16, bool VEC>
__global__ __launch_bounds__(WM * WN * 64, (WM * WN / 4) * (DEPTH == 0 ? (BM == 128 ? 3 : 2) : 1)) void gemm_bf16_kernel(const GemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
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

    constexpr int NT = WM * WN * 64;
    using LA = std::conditional_t<A_KC, core::DenseKC<core::Slots<BM, true, NT>::value>, core::DenseRC<core::Slots<BM, false, NT>::value>>;
    using LB = std::conditional_t<B_KC, core::DenseKC<core::Slots<BN, true, NT>::value>, core::DenseRC<core::Slots<BN, false, NT>::value>>;
    LA la;
    la.base = reinterpret_cast<const char *>(p.A[shard]) + (size_t)kbeg * (A_KC ? 2 : 2 * (size_t)p.lda);
    la.ld = p.lda; la.rows = p.M; la.K = klen;
    LB lb;
    lb.base = reinterpret_cast<const char *>(p.B[shard]) + (size_t)kbeg * (B_KC ? 2 : 2 * (size_t)p.ldb);
    lb.ld = p.ldb; lb.rows = p.N; lb.K = klen;
    core::tile_product<BM, BN, WM, WN, DEPTH, KMASK, OUT_BF16, VEC>(la, lb, p.C[vshard], p.ldc, p.M, p.N, klen, tm * BM, tn * BN, p.relu != 0, smem);
}

// second engine: operand tiles loaded straight into LDS, 256 x 256 tiles, eight waves
template <bool A_KC, bool B_KC, bool OUT_BF16, bool VEC>
__global__ __launch_bounds__(core2::kThreads2, 2) void gemm_bf16_v2_kernel(const GemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) char smem2[];
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
    using LA = std::conditional_t<A_KC, core2::DenseKC2, core2::DenseRC2>;
    using LB = std::conditional_t<B_KC, core2::DenseKC2, core2::DenseRC2>;
    LA la;
    la.base = reinterpret_cast<const char *>(p.A[shard]) + (size_t)kbeg * (A_KC ? 2 : 2 * (size_t)p.lda);
    la.ld = p.lda; la.rows = p.M; la.K = klen;
    LB lb;
    lb.base = reinterpret_cast<const char *>(p.B[shard]) + (size_t)kbeg * (B_KC ? 2 : 2 * (size_t)p.ldb);
    lb.ld = p.ldb; lb.rows = p.N; lb.K = klen;
    core2::tile_product2<OUT_BF16, VEC>(la, lb, p.C[vshard], p.ldc, p.M, p.N, klen, tm * 256, tn * 256, p.relu != 0, smem2);
}

template <bool A_KC, bool B_KC, bool OUT_BF16, bool VEC> tt_status launch_v2(GemmParams &p, int count, hipStream_t s)
{
    auto kern = gemm_bf16_v2_kernel<A_KC, B_KC, OUT_BF16, VEC>;
    if (ensure_dynamic_lds(reinterpret_cast<const void *>(kern), core2::kSmemBytes) != TT_OK) return TT_EDEVICE;
    p.tiles_m = (p.M + 255) / 256;
    p.tiles_n = (p.N + 255) / 256;
    int64_t total = (int64_t)p.tiles_m * p.tiles_n * count * p.ksplit;
    if (total >= (int64_t(1) << 30)) return TT_EUNSUPPORTED;
    p.total = (int32_t)total;
    p.per_xcd = (int32_t)((total + kXcds - 1) / kXcds);
    hipLaunchKernelGGL(kern, dim3((uint32_t)p.per_xcd * kXcds), dim3(core2::kThreads2), core2::kSmemBytes, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

// ---------------------------------------------------------------- generic kernel (fp32, or any unaligned shape)
// C[m][n] = sum_k A(m,k) B(k,n) with element strides; 64x64 tile, 16x16 threads, 4x4 outputs per thread.
struct GenericParams {
    const void *A[kMaxShards];
    const void *B[kMaxShards];
    void *C[kMaxShards];
    int32_t M, N, K;
    int64_t sam, sak, sbk, sbn;
    int32_t ldc;
    int32_t tiles_m, tiles_n;
    int32_t ksplit, kchunk;
};

template <bool IN_BF16> __device__ __forceinline__ float load_in(const void *p, int64_t off)
{
    if (IN_BF16) return __uint_as_float((uint32_t) reinterpret_cast<const uint16_t *>(p)[off] << 16);
    return reinterpret_cast<const float *>(p)[off];
}

template <bool IN_BF16, bool OUT_BF16, bool RELU>
__global__ __launch_bounds__(kThreads) void gemm_generic_kernel(const GenericParams p)
{
    constexpr int T = 64, KB = 16;
    __shared__ float As[KB][T + 1];
    __shared__ float Bs[KB][T + 1];
    int tiles = p.tiles_m * p.tiles_n;
    int vshard = blockIdx.x / tiles;
    int t = blockIdx.x - vshard * tiles;
    int m0 = (t % p.tiles_m) * T, n0 = (t / p.tiles_m) * T;
    const int shard = vshard / p.ksplit;
    const int kbeg = (vshard - shard * p.ksplit) * p.kchunk;
    const int kend = kbeg + p.kchunk < p.K ? kbeg + p.kchunk : p.K;
    const void *A = p.A[shard];
    const void *B = p.B[shard];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    // A tile's elements come into registers first (four of each operand per thread, all loads in flight together, from
    // clamped addresses with the out-of-range ones zeroed afterwards) and go to LDS when their step comes; the fetch
    // runs PD tiles ahead of the arithmetic.  These products are small and the chip is nearly idle while they run: what
    // a step costs is one trip to memory (about 2 us here), and PD of them are now under way at a time.
    constexpr int PT = T * KB / kThreads, PD = 4;
    float ra[PD][PT], rb[PD][PT];
    auto fetch = [&](int k0, float (&xa)[PT], float (&xb)[PT]) {
#pragma unroll
        for (int u = 0; u < PT; ++u) {
            const int i = threadIdx.x + u * kThreads;
            // pick the loop order that walks the contiguous stride
            int kk, mm;
            if (p.sak == 1) { kk = i % KB; mm = i / KB; } else { mm = i % T; kk = i / T; }
            const int gm = m0 + mm, gk = k0 + kk;
            const float va = load_in<IN_BF16>(A, (int64_t)(gm < p.M ? gm : p.M - 1) * p.sam + (int64_t)(gk < kend ? gk : kend - 1) * p.sak);
            xa[u] = (gm < p.M && gk < kend) ? va : 0.0f;
            int kb, nn;
            if (p.sbk == 1) { kb = i % KB; nn = i / KB; } else { nn = i % T; kb = i / T; }
            const int gn = n0 + nn, gkb = k0 + kb;
            const float vb = load_in<IN_BF16>(B, (int64_t)(gkb < kend ? gkb : kend - 1) * p.sbk + (int64_t)(gn < p.N ? gn : p.N - 1) * p.sbn);
            xb[u] = (gn < p.N && gkb < kend) ? vb : 0.0f;
        }
    };
#pragma unroll
    for (int d = 0; d < PD; ++d)
        if (kbeg + d * KB < kend) fetch(kbeg + d * KB, ra[d], rb[d]);
    for (int k0 = kbeg; k0 < kend; k0 += PD * KB) {
#pragma unroll
        for (int d = 0; d < PD; ++d) { // (unrolled: the register ring is indexed by constants)
            const int kd = k0 + d * KB;
            if (kd >= kend) break;
#pragma unroll
            for (int u = 0; u < PT; ++u) {
                const int i = threadIdx.x + u * kThreads;
                int kk, mm;
                if (p.sak == 1) { kk = i % KB; mm = i / KB; } else { mm = i % T; kk = i / T; }
                As[kk][mm] = ra[d][u];
                int kb, nn;
                if (p.sbk == 1) { kb = i % KB; nn = i / KB; } else { nn = i % T; kb = i / T; }
                Bs[kb][nn] = rb[d][u];
            }
            __syncthreads();
            if (kd + PD * KB < kend) fetch(kd + PD * KB, ra[d], rb[d]);
#pragma unroll
            for (int kk = 0; kk < KB; ++kk) {
                float a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int row = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
            if (row >= p.M || col >= p.N) continue;
            float v = acc[i][j];
            if (RELU) v = v > 0.0f ? v : 0.0f;
            if (OUT_BF16) reinterpret_cast<uint16_t *>(p.C[vshard])[(size_t)row * p.ldc + col] = (uint16_t)f32_to_bf16_bits(v);
            else reinterpret_cast<float *>(p.C[vshard])[(size_t)row * p.ldc + col] = v;
        }
}

template <int BM, int BN, int WM, int WN, int DEPTH, bool KMASK, bool A_KC, bool B_KC, bool OUT_BF16, bool VEC>
tt_status launch_mfma_cfg(GemmParams &p, int count, hipStream_t s)
{
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, DEPTH, KMASK, A_KC, B_KC, OUT_BF16, VEC>;
    constexpr size_t smem = core::smem_bytes<BM, BN, DEPTH>();
    if (ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem) != TT_OK) return TT_EDEVICE;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    int64_t total = (int64_t)p.tiles_m * p.tiles_n * count * p.ksplit;
    if (total >= (int64_t(1) << 30)) return TT_EUNSUPPORTED;
    p.total = (int32_t)total;
    p.per_xcd = (int32_t)((total + kXcds - 1) / kXcds);
    hipLaunchKernelGGL(kern, dim3((uint32_t)p.per_xcd * kXcds), dim3(WM * WN * 64), smem, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

// Tile choice (TT_GEMM_TILE=0..5 overrides; tuning aid).
//   5: 256 x 256, eight waves (two per SIMD, 128 x 64 each): the default whenever the launch has enough tiles to put
//      work on at least half the CUs; two resident waves per SIMD cover each other's LDS / memory waits and the large
//      tile halves operand traffic per flop.
//   0: 256 x 128, four waves, two K tiles prefetched in registers: long K loops with few column tiles.
//   1: 128 x 128, four waves, up to two workgroups per CU: small products and short K loops.
//   2, 3, 4: 256 x 256 four-wave, 256 x 128 and 128 x 128 single-LDS-buffer variants kept for experiments.
//   8: 256 x 256, eight waves, second engine (gemm_core2.h): tiles loaded straight into LDS.
int pick_tile(int64_t M, int64_t N, int64_t K, int count)
{
    const int forced = tuning_int("TT_GEMM_TILE", -1);
    if ((forced >= 0 && forced <= 5) || forced == 8) return forced;
    const int64_t big = ((M + 255) / 256) * ((N + 255) / 256) * count;
    if (M > 128 && N > 128 && big >= 128) return 5;
    return (M > 128 && K >= 1024) ? 0 : 1;
}

template <bool KMASK, bool A_KC, bool B_KC, bool OUT_BF16, bool VEC> tt_status launch_mfma_tile(GemmParams &p, int count, hipStream_t s)
{
    const int tile = pick_tile(p.M, p.N, p.ksplit > 1 ? p.kchunk : p.K, count * p.ksplit);
    if (tile == 5) return launch_mfma_cfg<256, 256, 2, 4, 1, KMASK, A_KC, B_KC, OUT_BF16, VEC>(p, count, s);
    if (tile == 4) return launch_mfma_cfg<128, 128, 2, 2, 0, KMASK, A_KC, B_KC, OUT_BF16, VEC>(p, count, s);
    if (tile == 3) return launch_mfma_cfg<256, 128, 2, 2, 0, KMASK, A_KC, B_KC, OUT_BF16, VEC>(p, count, s);
    if (tile == 2) return launch_mfma_cfg<256, 256, 2, 2, 1, KMASK, A_KC, B_KC, OUT_BF16, VEC>(p, count, s);
    if (tile == 0) return launch_mfma_cfg<256, 128, 2, 2, 2, KMASK, A_KC, B_KC, OUT_BF16, VEC>(p, count, s);
    return launch_mfma_cfg<128, 128, 2, 2, 1, KMASK, A_KC, B_KC, OUT_BF16, VEC>(p, count, s);
}

template <bool A_KC, bool B_KC, bool OUT_BF16, bool VEC> tt_status launch_mfma_kmask(GemmParams &p, int count, hipStream_t s)
{
    // Where the eight-wave 256 x 256 tile is chosen, the engine that loads tiles straight into LDS measured faster for
    // every layout but NN (A K-contiguous, B row-contiguous), which stays on the register-staged engine.
    const int tile = pick_tile(p.M, p.N, p.ksplit > 1 ? p.kchunk : p.K, count * p.ksplit);
    const bool nn = A_KC && !B_KC;
    if ((tile == 8 || (tile == 5 && !nn && tuning_int("TT_GEMM_TILE", -1) < 0)) && p.M >= 8 && p.N >= 8)
        return launch_v2<A_KC, B_KC, OUT_BF16, VEC>(p, count, s);
    return p.K % core::BK ? launch_mfma_tile<true, A_KC, B_KC, OUT_BF16, VEC>(p, count, s)
                          : launch_mfma_tile<false, A_KC, B_KC, OUT_BF16, VEC>(p, count, s);
}

template <bool A_KC, bool B_KC> tt_status launch_mfma_out(GemmParams &p, int count, int out_dtype, int act, bool vec, hipStream_t s)
{
    p.relu = act == TT_ACT_RELU;
    if (out_dtype == TT_BF16)
        return vec ? launch_mfma_kmask<A_KC, B_KC, true, true>(p, count, s) : launch_mfma_kmask<A_KC, B_KC, true, false>(p, count, s);
    return vec ? launch_mfma_kmask<A_KC, B_KC, false, true>(p, count, s) : launch_mfma_kmask<A_KC, B_KC, false, false>(p, count, s);
}

template <bool IN_BF16> tt_status launch_generic_in(const GenericParams &p, int count, int out_dtype, int act, hipStream_t s)
{
    const bool relu = act == TT_ACT_RELU;
    dim3 grid((uint32_t)(p.tiles_m * p.tiles_n * count * p.ksplit)), block(kThreads);
    if (out_dtype == TT_BF16) {
        if (relu) hipLaunchKernelGGL((gemm_generic_kernel<IN_BF16, true, true>), grid, block, 0, s, p);
        else hipLaunchKernelGGL((gemm_generic_kernel<IN_BF16, true, false>), grid, block, 0, s, p);
    } else {
        if (relu) hipLaunchKernelGGL((gemm_generic_kernel<IN_BF16, false, true>), grid, block, 0, s, p);
        else hipLaunchKernelGGL((gemm_generic_kernel<IN_BF16, false, false>), grid, block, 0, s, p);
    }
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

bool all_aligned16(const void *const *ptrs, int n)
{
    for (int i = 0; i < n; ++i)
        if (reinterpret_cast<uintptr_t>(ptrs[i]) & 15) return false;
    return true;
}

} // namespace

tt_status launch_gemm(int count, const void *const *A, const void *const *B, void *const *C, int64_t M, int64_t N,
                      int64_t K, int trans_a, int trans_b, int in_dtype, int out_dtype, int act, int ksplit, void *stream)
{
    if (!A || !B || !C || count < 0 || count > kMaxShards || M < 0 || N < 0 || K < 0) return TT_EINVAL;
    if ((in_dtype != TT_BF16 && in_dtype != TT_F32) || (out_dtype != TT_BF16 && out_dtype != TT_F32)) return TT_EINVAL;
    if (act != TT_ACT_NONE && act != TT_ACT_RELU) return TT_EINVAL;
    if (ksplit < 1 || count * ksplit > kMaxShards) return TT_EINVAL;
    if (count == 0 || M == 0 || N == 0) return TT_OK;
    if (M >= (int64_t(1) << 31) || N >= (int64_t(1) << 31) || K >= (int64_t(1) << 31)) return TT_EUNSUPPORTED;
    for (int s = 0; s < count; ++s)
        if (!A[s] || !B[s]) return TT_EINVAL;
    for (int s = 0; s < count * ksplit; ++s)
        if (!C[s]) return TT_EINVAL;
    // K chunk per split: a multiple of the tile depth; every chunk must be non-empty
    const int64_t kchunk = ksplit == 1 ? (K > 0 ? K : 1) : ((K + ksplit - 1) / ksplit + 63) / 64 * 64;
    if (ksplit > 1 && kchunk * (ksplit - 1) >= K) return TT_EINVAL;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    // MFMA path needs 16-byte vectors along each operand's contiguous dimension
    const int64_t a_contig = trans_a ? M : K, b_contig = trans_b ? K : N;
    // (operand byte offsets are kept in 32 bits inside the kernel)
    const bool mfma_ok = in_dtype == TT_BF16 && K > 0 && a_contig % 8 == 0 && b_contig % 8 == 0 &&
                         M * K < (int64_t(1) << 31) && K * N < (int64_t(1) << 31) &&
                         all_aligned16(A, count) && all_aligned16(B, count);
    const uint64_t in_b = in_dtype == TT_BF16 ? 2 : 4, out_b = out_dtype == TT_BF16 ? 2 : 4;
    const int kclass = !mfma_ok ? TT_K_GEMM_GENERIC
                                : (trans_a ? (trans_b ? TT_K_GEMM_TT : TT_K_GEMM_TN) : (trans_b ? TT_K_GEMM_NT : TT_K_GEMM_NN));
    ProfileScope scope(stream, kclass, count, M, N, K,
                       (uint64_t)count * (in_b * ((uint64_t)M * K + (uint64_t)K * N) + out_b * (uint64_t)M * N),
                       2ull * (uint64_t)M * (uint64_t)N * (uint64_t)K * (uint64_t)count);
    if (mfma_ok) {
        GemmParams p;
        for (int i = 0; i < kMaxShards; ++i) {
            p.A[i] = i < count ? A[i] : nullptr;
            p.B[i] = i < count ? B[i] : nullptr;
            p.C[i] = i < count * ksplit ? C[i] : nullptr;
        }
        p.M = (int32_t)M; p.N = (int32_t)N; p.K = (int32_t)K;
        p.lda = (int32_t)a_contig;
        p.ldb = (int32_t)b_contig;
        p.ldc = (int32_t)N;
        p.ksplit = ksplit;
        p.kchunk = (int32_t)kchunk;
        const bool a_kc = !trans_a, b_kc = trans_b != 0;
        // 16-byte stores along C's rows need 16-byte row pitch and base addresses
        const bool vec = N % (out_dtype == TT_BF16 ? 8 : 4) == 0 && all_aligned16(const_cast<const void *const *>(C), count * ksplit);
        // Engine choice (TT_GEMM_ENGINE=1: the two older engines only, =3 / =4: that engine wherever it applies; tuning aid):
        //  - launches with too few 256 x 256 tiles to occupy the chip (the hidden-layer products at batch 256): the
        //    256 x 128 engine with two workgroups per CU, which doubles the number of workgroups;
        //  - large launches with more than one row of tiles: the persistent pipelined engine;
        //  - of the skinny batch-256 products of the wide layers (one row of tiles, bound by the weight stream) the NN
        //    layout measured 6 % faster on the persistent engine, the others equal or faster on the direct-to-LDS engine.
        const int engine = tuning_int("TT_GEMM_ENGINE", 0);
        const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256) * count * ksplit;
        //  - weight-gradient shaped products (both operands stored with K as the slow dimension, K = 128, 256 or 512, a bf16
        //    result large enough to give every resident workgroup at least two 256 x 64 units; measured down to the second
        //    VGG-16 weight gradient, 8 x 1024 x 2048 x 256: 16 us against 20 us on the persistent engine): the engine that
        //    keeps the left operand's panel in registers and is bound by writing the result (gemm_core5.h)
        if ((engine == 5 || engine == 0) && !a_kc && !b_kc && ksplit == 1 && out_dtype == TT_BF16 && vec && in_dtype == TT_BF16 &&
            (engine == 5 || ((M + 255) / 256) * (N / 64) * count >= 2 * 512)) {
            const tt_status st = launch_gemm_v5(count, A, B, C, M, N, K, a_contig, b_contig, N, act == TT_ACT_RELU, stream);
            if (st != TT_EUNSUPPORTED) return st;
        }
        //  - of those, the products A B^T with both operands K-contiguous (the data gradients) that give between half a
        //    tile and one 256 x 128 tile per CU: the same tile with K tiles of 64, which fetches whole 128-byte lines of the
        //    streamed weights (gemm_core6.h says what that is worth: 74 -> 66 us for the first VGG-16 data gradient; with
        //    more tiles than CUs, with fewer than half as many, and for the NN layout it measured equal or slower)
        const int64_t tiles128 = ((M + 255) / 256) * ((N + 127) / 128) * count * ksplit;
        if (a_kc && (engine == 6 || (engine == 0 && b_kc && big_tiles < 200 && M > 128 && N >= 256 && tiles128 >= 128 &&
                                     tiles128 <= 256 && (ksplit > 1 ? kchunk : K) >= 256))) {
            const tt_status st = launch_gemm_v6(count, A, B, C, M, N, K, a_contig, b_contig, N, b_kc, out_dtype, act == TT_ACT_RELU,
                                                vec, ksplit, kchunk, stream);
            if (st != TT_EUNSUPPORTED) return st;
        }
        if (engine == 4 || (engine == 0 && big_tiles < 200 && M > 128 && N >= 256)) {
            const tt_status st = launch_gemm_v4(count, A, B, C, M, N, K, a_contig, b_contig, N, a_kc, b_kc, out_dtype,
                                                act == TT_ACT_RELU, vec, ksplit, kchunk, stream);
            if (st != TT_EUNSUPPORTED) return st;
        }
        if (engine != 1 && engine != 4 && (engine == 3 || M > 256 || (a_kc && !b_kc)) && pick_tile(M, N, ksplit > 1 ? kchunk : K, count * ksplit) == 5) {
            const tt_status st = launch_gemm_v3(count, A, B, C, M, N, K, a_contig, b_contig, N, a_kc, b_kc, out_dtype,
                                                act == TT_ACT_RELU, vec, ksplit, kchunk, stream);
            if (st != TT_EUNSUPPORTED) return st;
        }
        if (a_kc && b_kc) return launch_mfma_out<true, true>(p, count, out_dtype, act, vec, s);
        if (a_kc && !b_kc) return launch_mfma_out<true, false>(p, count, out_dtype, act, vec, s);
        if (!a_kc && !b_kc) return launch_mfma_out<false, false>(p, count, out_dtype, act, vec, s);
        return launch_mfma_out<false, true>(p, count, out_dtype, act, vec, s);
    }
    GenericParams g;
    for (int i = 0; i < kMaxShards; ++i) {
        g.A[i] = i < count ? A[i] : nullptr;
        g.B[i] = i < count ? B[i] : nullptr;
        g.C[i] = i < count * ksplit ? C[i] : nullptr;
    }
    g.M = (int32_t)M; g.N = (int32_t)N; g.K = (int32_t)K;
    g.sam = trans_a ? 1 : K; g.sak = trans_a ? M : 1;
    g.sbk = trans_b ? 1 : N; g.sbn = trans_b ? K : 1;
    g.ldc = (int32_t)N;
    g.tiles_m = (int32_t)((M + 63) / 64);
    g.tiles_n = (int32_t)((N + 63) / 64);
    g.ksplit = ksplit;
    g.kchunk = (int32_t)kchunk;
    if ((int64_t)g.tiles_m * g.tiles_n * count * ksplit >= (int64_t(1) << 31)) return TT_EUNSUPPORTED;
    return in_dtype == TT_BF16 ? launch_generic_in<true>(g, count, out_dtype, act, s)
                               : launch_generic_in<false>(g, count, out_dtype, act, s);
}

} // namespace tt

extern "C" tt_status tt_shard_gemm(int count, const void *const *A, const void *const *B, void *const *C, int64_t M,
                                   int64_t N, int64_t K, int trans_a, int trans_b, int in_dtype, int out_dtype, int act,
                                   void *stream)
{
    return tt::launch_gemm(count, A, B, C, M, N, K, trans_a, trans_b, in_dtype, out_dtype, act, 1, stream);
}
