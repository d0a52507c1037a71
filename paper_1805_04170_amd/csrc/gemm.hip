// Shard products: C_s = op(A_s) op(B_s) for all shards in one launch (Sec. 5.2 step 2 of arXiv 1805.04170:
// after input conversion every device runs the same sub-operator on its own tiles).
//
// bf16 path: CDNA4 MFMA (v_mfma_f32_32x32x16_bf16), 256-thread workgroups of four 64-lane waves, operand tiles
// staged through LDS in K-contiguous rows, fp32 accumulators in registers, double-buffered LDS with the next
// tile's global loads in flight during the MFMA loop.  Operands whose contiguous dimension is not K (W in the
// forward product, both operands of the weight gradient) are transposed in registers (4x8 blocks) on their way
// into LDS, so the MFMA loop is the same for NN, NT and TN products.
// fp32 path / unaligned shapes: a plain LDS-tiled FMA kernel with arbitrary strides.
#include <hip/hip_runtime.h>
#include <cstdint>
#include "tt_internal.h"

namespace tt {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int BK = 64;        // K extent of an LDS tile
constexpr int LDK = BK + 8;   // padded LDS row (elements): 144-byte rows make the 16-byte fragment reads conflict-free
constexpr int kXcds = 8;

struct GemmParams {
    const void *A[kMaxShards];
    const void *B[kMaxShards];
    void *C[kMaxShards];
    int32_t M, N, K;
    int32_t lda, ldb, ldc;
    int32_t tiles_m, tiles_n;
    int32_t per_xcd;  // logical workgroups per XCD (grid = per_xcd * 8)
    int32_t total;    // tiles_m * tiles_n * count
};

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Global -> register staging of one operand tile.
// KC = true : operand stored [rows][K] (K contiguous).  Tile = ROWS x BK, 16-byte vectors along K.
// KC = false: operand stored [K][rows] (rows contiguous).  Tile = BK x ROWS, handled as 4(k) x 8(row) blocks that
//             are transposed in registers so that LDS always holds K-contiguous rows.
template <int ROWS, bool KC> struct Stage {
    static constexpr int NV = KC ? ROWS * (BK / 8) / kThreads : (BK / 4) * (ROWS / 8) / kThreads * 4;
    u32x4 r[NV];

    __device__ __forceinline__ void load(const uint16_t *__restrict__ base, int ld, int row0, int nrows, int k0, int K)
    {
        const int tid = threadIdx.x;
        if constexpr (KC) {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                int v = tid + i * kThreads;
                int row = row0 + (v >> 3), k = k0 + ((v & 7) << 3);
                u32x4 z = {0, 0, 0, 0};
                r[i] = (row < nrows && k < K) ? *reinterpret_cast<const u32x4 *>(base + (size_t)row * ld + k) : z;
            }
        } else {
            constexpr int RV = ROWS / 8; // 16-byte vectors per k-row
#pragma unroll
            for (int i = 0; i < NV / 4; ++i) {
                int b = tid + i * kThreads;
                int rv = b % RV, kg = b / RV;
                int row = row0 + rv * 8;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    int k = k0 + kg * 4 + q;
                    u32x4 z = {0, 0, 0, 0};
                    r[i * 4 + q] = (row < nrows && k < K) ? *reinterpret_cast<const u32x4 *>(base + (size_t)k * ld + row) : z;
                }
            }
        }
    }

    __device__ __forceinline__ void store(uint16_t *lds) const
    {
        const int tid = threadIdx.x;
        if constexpr (KC) {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                int v = tid + i * kThreads;
                *reinterpret_cast<u32x4 *>(lds + (v >> 3) * LDK + ((v & 7) << 3)) = r[i];
            }
        } else {
            constexpr int RV = ROWS / 8;
#pragma unroll
            for (int i = 0; i < NV / 4; ++i) {
                int b = tid + i * kThreads;
                int rv = b % RV, kg = b / RV;
                uint16_t *dst = lds + (rv * 8) * LDK + kg * 4;
                const u32x4 &a = r[i * 4 + 0], &bq = r[i * 4 + 1], &c = r[i * 4 + 2], &d = r[i * 4 + 3];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // word j of each k-row holds rows (2j, 2j+1); gather the four k values of each row
                    u32x2 lo = {(a[j] & 0xffffu) | (bq[j] << 16), (c[j] & 0xffffu) | (d[j] << 16)};
                    u32x2 hi = {(a[j] >> 16) | (bq[j] & 0xffff0000u), (c[j] >> 16) | (d[j] & 0xffff0000u)};
                    *reinterpret_cast<u32x2 *>(dst + (2 * j) * LDK) = lo;
                    *reinterpret_cast<u32x2 *>(dst + (2 * j + 1) * LDK) = hi;
                }
            }
        }
    }
};

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, bool OUT_BF16, bool RELU>
__global__ __launch_bounds__(kThreads) void gemm_bf16_kernel(const GemmParams p)
{
    static_assert(WM * WN == 4, "four waves");
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    constexpr int A_ELEMS = BM * LDK, B_ELEMS = BN * LDK;

    // XCD-aware order: consecutive hardware workgroup numbers go round-robin over the 8 XCDs, so give every XCD a
    // contiguous range of logical workgroups (shard-major): tiles of one shard share that XCD's L2.
    int bid = blockIdx.x;
    int logical = (bid % kXcds) * p.per_xcd + bid / kXcds;
    if (logical >= p.total) return;
    int tiles = p.tiles_m * p.tiles_n;
    int shard = logical / tiles;
    int t = logical - shard * tiles;
    int tm = t % p.tiles_m, tn = t / p.tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;

    const uint16_t *A = reinterpret_cast<const uint16_t *>(p.A[shard]);
    const uint16_t *B = reinterpret_cast<const uint16_t *>(p.B[shard]);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave / WN) * (TM * 32), wn0 = (wave % WN) * (TN * 32);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    Stage<BM, A_KC> sa;
    Stage<BN, B_KC> sb;
    const int nk = (p.K + BK - 1) / BK;

    sa.load(A, p.lda, m0, p.M, 0, p.K);
    sb.load(B, p.ldb, n0, p.N, 0, p.K);
    sa.store(smem);
    sb.store(smem + A_ELEMS);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const uint16_t *As = smem + cur * (A_ELEMS + B_ELEMS);
        const uint16_t *Bs = As + A_ELEMS;
        const bool more = kt + 1 < nk;
        if (more) {
            sa.load(A, p.lda, m0, p.M, (kt + 1) * BK, p.K);
            sb.load(B, p.ldb, n0, p.N, (kt + 1) * BK, p.K);
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[TM], bf[TN];
            const int koff = ks * 16 + (lane >> 5) * 8;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8 *>(As + (wm0 + i * 32 + (lane & 31)) * LDK + koff);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bf[j] = *reinterpret_cast<const bf16x8 *>(Bs + (wn0 + j * 32 + (lane & 31)) * LDK + koff);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            uint16_t *nxt = smem + (cur ^ 1) * (A_ELEMS + B_ELEMS);
            sa.store(nxt);
            sb.store(nxt + A_ELEMS);
        }
        __syncthreads();
    }

    // epilogue: lane holds column (lane & 31) and rows 8*(e/4) + 4*(lane/32) + e%4 of each 32x32 tile
    const int col_l = lane & 31, row_l = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn0 + j * 32 + col_l;
            if (col >= p.N) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + wm0 + i * 32 + 8 * (e >> 2) + row_l + (e & 3);
                if (row >= p.M) continue;
                float v = acc[i][j][e];
                if (RELU) v = v > 0.0f ? v : 0.0f;
                if (OUT_BF16)
                    reinterpret_cast<uint16_t *>(p.C[shard])[(size_t)row * p.ldc + col] = (uint16_t)f32_to_bf16_bits(v);
                else
                    reinterpret_cast<float *>(p.C[shard])[(size_t)row * p.ldc + col] = v;
            }
        }
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
    int shard = blockIdx.x / tiles;
    int t = blockIdx.x - shard * tiles;
    int m0 = (t % p.tiles_m) * T, n0 = (t / p.tiles_m) * T;
    const void *A = p.A[shard];
    const void *B = p.B[shard];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < p.K; k0 += KB) {
        for (int i = threadIdx.x; i < T * KB; i += kThreads) {
            // A tile: pick the loop order that walks the contiguous stride
            int kk, mm;
            if (p.sak == 1) { kk = i % KB; mm = i / KB; } else { mm = i % T; kk = i / T; }
            int gm = m0 + mm, gk = k0 + kk;
            As[kk][mm] = (gm < p.M && gk < p.K) ? load_in<IN_BF16>(A, gm * p.sam + gk * p.sak) : 0.0f;
            int kb, nn;
            if (p.sbk == 1) { kb = i % KB; nn = i / KB; } else { nn = i % T; kb = i / T; }
            int gn = n0 + nn, gkb = k0 + kb;
            Bs[kb][nn] = (gn < p.N && gkb < p.K) ? load_in<IN_BF16>(B, gkb * p.sbk + gn * p.sbn) : 0.0f;
        }
        __syncthreads();
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
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int row = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
            if (row >= p.M || col >= p.N) continue;
            float v = acc[i][j];
            if (RELU) v = v > 0.0f ? v : 0.0f;
            if (OUT_BF16) reinterpret_cast<uint16_t *>(p.C[shard])[(size_t)row * p.ldc + col] = (uint16_t)f32_to_bf16_bits(v);
            else reinterpret_cast<float *>(p.C[shard])[(size_t)row * p.ldc + col] = v;
        }
}

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, bool OUT_BF16, bool RELU>
tt_status launch_mfma_cfg(GemmParams &p, int count, hipStream_t s)
{
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, A_KC, B_KC, OUT_BF16, RELU>;
    constexpr size_t smem = 2 * (size_t)(BM + BN) * LDK * sizeof(uint16_t);
    static bool configured = false; // attribute is per function; setting it twice is harmless
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return TT_EDEVICE;
        configured = true;
    }
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    int64_t total = (int64_t)p.tiles_m * p.tiles_n * count;
    if (total >= (int64_t(1) << 30)) return TT_EUNSUPPORTED;
    p.total = (int32_t)total;
    p.per_xcd = (int32_t)((total + kXcds - 1) / kXcds);
    hipLaunchKernelGGL(kern, dim3((uint32_t)p.per_xcd * kXcds), dim3(kThreads), smem, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

template <bool A_KC, bool B_KC, bool OUT_BF16, bool RELU> tt_status launch_mfma_tile(GemmParams &p, int count, hipStream_t s)
{
    // Tall tile when there are at least 256 rows (weights stream through once per 256 batch rows), else square.
    if (p.M > 128) return launch_mfma_cfg<256, 128, 2, 2, A_KC, B_KC, OUT_BF16, RELU>(p, count, s);
    return launch_mfma_cfg<128, 128, 2, 2, A_KC, B_KC, OUT_BF16, RELU>(p, count, s);
}

template <bool A_KC, bool B_KC> tt_status launch_mfma_out(GemmParams &p, int count, int out_dtype, int act, hipStream_t s)
{
    const bool relu = act == TT_ACT_RELU;
    if (out_dtype == TT_BF16)
        return relu ? launch_mfma_tile<A_KC, B_KC, true, true>(p, count, s) : launch_mfma_tile<A_KC, B_KC, true, false>(p, count, s);
    return relu ? launch_mfma_tile<A_KC, B_KC, false, true>(p, count, s) : launch_mfma_tile<A_KC, B_KC, false, false>(p, count, s);
}

template <bool IN_BF16> tt_status launch_generic_in(const GenericParams &p, int count, int out_dtype, int act, hipStream_t s)
{
    const bool relu = act == TT_ACT_RELU;
    dim3 grid((uint32_t)(p.tiles_m * p.tiles_n * count)), block(kThreads);
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
                      int64_t K, int trans_a, int trans_b, int in_dtype, int out_dtype, int act, void *stream)
{
    if (!A || !B || !C || count < 0 || count > kMaxShards || M < 0 || N < 0 || K < 0) return TT_EINVAL;
    if ((in_dtype != TT_BF16 && in_dtype != TT_F32) || (out_dtype != TT_BF16 && out_dtype != TT_F32)) return TT_EINVAL;
    if (act != TT_ACT_NONE && act != TT_ACT_RELU) return TT_EINVAL;
    if (count == 0 || M == 0 || N == 0) return TT_OK;
    if (M >= (int64_t(1) << 31) || N >= (int64_t(1) << 31) || K >= (int64_t(1) << 31)) return TT_EUNSUPPORTED;
    for (int s = 0; s < count; ++s)
        if (!A[s] || !B[s] || !C[s]) return TT_EINVAL;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    // MFMA path needs 16-byte vectors along each operand's contiguous dimension
    const int64_t a_contig = trans_a ? M : K, b_contig = trans_b ? K : N;
    const bool mfma_ok = in_dtype == TT_BF16 && K > 0 && a_contig % 8 == 0 && b_contig % 8 == 0 &&
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
            p.C[i] = i < count ? C[i] : nullptr;
        }
        p.M = (int32_t)M; p.N = (int32_t)N; p.K = (int32_t)K;
        p.lda = (int32_t)a_contig;
        p.ldb = (int32_t)b_contig;
        p.ldc = (int32_t)N;
        const bool a_kc = !trans_a, b_kc = trans_b != 0;
        if (a_kc && b_kc) return launch_mfma_out<true, true>(p, count, out_dtype, act, s);
        if (a_kc && !b_kc) return launch_mfma_out<true, false>(p, count, out_dtype, act, s);
        if (!a_kc && !b_kc) return launch_mfma_out<false, false>(p, count, out_dtype, act, s);
        return launch_mfma_out<false, true>(p, count, out_dtype, act, s);
    }
    GenericParams g;
    for (int i = 0; i < kMaxShards; ++i) {
        g.A[i] = i < count ? A[i] : nullptr;
        g.B[i] = i < count ? B[i] : nullptr;
        g.C[i] = i < count ? C[i] : nullptr;
    }
    g.M = (int32_t)M; g.N = (int32_t)N; g.K = (int32_t)K;
    g.sam = trans_a ? 1 : K; g.sak = trans_a ? M : 1;
    g.sbk = trans_b ? 1 : N; g.sbn = trans_b ? K : 1;
    g.ldc = (int32_t)N;
    g.tiles_m = (int32_t)((M + 63) / 64);
    g.tiles_n = (int32_t)((N + 63) / 64);
    if ((int64_t)g.tiles_m * g.tiles_n * count >= (int64_t(1) << 31)) return TT_EUNSUPPORTED;
    return in_dtype == TT_BF16 ? launch_generic_in<true>(g, count, out_dtype, act, s)
                               : launch_generic_in<false>(g, count, out_dtype, act, s);
}

} // namespace tt

extern "C" tt_status tt_shard_gemm(int count, const void *const *A, const void *const *B, void *const *C, int64_t M,
                                   int64_t N, int64_t K, int trans_a, int trans_b, int in_dtype, int out_dtype, int act,
                                   void *stream)
{
    return tt::launch_gemm(count, A, B, C, M, N, K, trans_a, trans_b, in_dtype, out_dtype, act, stream);
}
