// Second bf16 MFMA tile engine: operand tiles go from global memory straight into LDS (global_load_lds_dwordx4, no
// register hop and no LDS store instructions), eight waves per workgroup (two per SIMD), 256 x 256 tiles, two LDS stages.
//
// LDS layouts (no padding is possible: a wave-wide direct load writes 64 x 16 contiguous bytes, lane by lane; instead
// each lane chooses WHICH global chunk it fetches, which gives an XOR swizzle for free):
//   K-contiguous operand  tile[row][8 chunks of 8 k]   chunk position p of row r holds k-chunk p ^ ((r >> 1) & 7);
//                         fragments are plain 16-byte reads.
//   row-contiguous operand tile[k][ROWS / 8 chunks of 8 rows]  chunk position p of k-row k holds row-chunk p ^ ((k & 3) << 1);
//                         fragments are two ds_read_b64_tr_b16 (LDS transpose reads): within 16 lanes, lane i receives
//                         element i % 4 of the 4-element rows addressed by lanes 4e + i / 4, e = 0..3, so addressing
//                         row (k0 + j / 4, rows 4 (j % 4) ..) from lane j hands lane i the values (k0 + e, row i).
// Out-of-range chunks (K tails, image padding) are fetched from a 16-byte block of zeros instead of being masked.
#pragma once
#include <cstdint>
#include "tt_device.h"
#include "gemm_core.h"

namespace tt {
namespace core2 {

using core::bf16x8;
using core::f32x16;
using core::f32x4;
using core::u32x4;
using core::BK;

constexpr int kThreads2 = 512;
constexpr int BM2 = 256, BN2 = 256;
constexpr int kStageBytes = (BM2 + BN2) * BK * 2; // 64 KB
constexpr size_t kSmemBytes = 2 * (size_t)kStageBytes;

using dev::s16x4;

__device__ __attribute__((aligned(16))) const uint32_t g_zero_chunk[4] = {0, 0, 0, 0};

template <int ROWS, class L> __device__ __forceinline__ void issue_tile(const L &ld, int row0, int k0, char *lds);

// ---- loaders.  A loader issues the global -> LDS loads of one operand tile through issue<ROWS>(row0, k0, lds); the dense
// ---- ones below name the address of one 16-byte chunk and leave the walk over the tile to issue_tile ----
// KC: rows of the operand have K contiguous.  chunk(row, k): 8 consecutive k of one row.
struct DenseKC2 {
    static constexpr bool KC = true;
    const char *base;
    int ld, rows, K;
    __device__ __forceinline__ const void *chunk(int row, int k) const
    {
        row = row < rows ? row : rows - 1; // rows past the end only feed C rows that are never stored
        const char *p = base + ((size_t)row * ld + k) * 2;
        return k < K ? (const void *)p : (const void *)g_zero_chunk;
    }
    template <int ROWS> __device__ __forceinline__ void issue(int row0, int k0, char *lds) const { issue_tile<ROWS>(*this, row0, k0, lds); }
};
// RC: rows contiguous, K strides.  chunk(k, row0): rows row0..row0+7 at one k.
struct DenseRC2 {
    static constexpr bool KC = false;
    const char *base;
    int ld, rows, K;
    __device__ __forceinline__ const void *chunk(int k, int row0) const
    {
        row0 = row0 < rows ? row0 : rows - 8;
        const char *p = base + ((size_t)k * ld + row0) * 2;
        return k < K ? (const void *)p : (const void *)g_zero_chunk;
    }
    template <int ROWS> __device__ __forceinline__ void issue(int row0, int k0, char *lds) const { issue_tile<ROWS>(*this, row0, k0, lds); }
};

__device__ __forceinline__ void load_chunk_to_lds(const void *g, char *lds_wave_base)
{
    // every lane supplies its own global address; the 64 chunks land at lds_wave_base + lane * 16 (see tt_device.h)
    dev::lds_dma16(g, __builtin_amdgcn_readfirstlane(dev::lds_addr(lds_wave_base)));
}

// issue the loads of one operand tile (ROWS x 64) into lds
template <int ROWS, class L> __device__ __forceinline__ void issue_tile(const L &ld, int row0, int k0, char *lds)
{
    const int tid = threadIdx.x, wave = tid >> 6;
    constexpr int NI = ROWS * 8 / kThreads2;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int v = tid + i * kThreads2; // chunk position in the tile
        char *dst = lds + (size_t)(wave * 64 + i * kThreads2) * 16;
        if constexpr (L::KC) {
            const int r = v >> 3, p = v & 7;
            load_chunk_to_lds(ld.chunk(row0 + r, k0 + ((p ^ ((r >> 1) & 7)) << 3)), dst);
        } else {
            constexpr int CPR = ROWS / 8;
            const int k = v / CPR, p = v % CPR;
            load_chunk_to_lds(ld.chunk(k0 + k, row0 + ((p ^ ((k & 3) << 1)) << 3)), dst);
        }
    }
}

// fragment (32 rows x 16 k) of an operand tile for the MFMA: rows rbase .. rbase+31 of the tile, k-step ks
template <int ROWS, bool KC> __device__ __forceinline__ bf16x8 read_frag(const char *lds, int rbase, int ks, int lane)
{
    if constexpr (KC) {
        const int r = rbase + (lane & 31), q = ks * 2 + (lane >> 5);
        return *reinterpret_cast<const bf16x8 *>(lds + r * 128 + ((q ^ ((r >> 1) & 7)) << 4));
    } else {
        const int g16 = lane >> 4, j = lane & 15;
        const int n0 = rbase + (g16 & 1) * 16 + 4 * (j & 3); // first of this lane's 4 addressed rows
        const int c = n0 >> 3, byte = (n0 & 7) * 2;
        union { s16x4 h[2]; bf16x8 v; } u;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int k = ks * 16 + (g16 >> 1) * 8 + h * 4 + (j >> 2);
            const char *a = lds + k * (ROWS * 2) + ((c ^ ((k & 3) << 1)) << 4) + byte;
            u.h[h] = dev::lds_read_tr16_b64(a);
        }
        return u.v;
    }
}

// C tile (m0, n0) of C = A B; 512 threads; smem: kSmemBytes, 16-byte aligned.
template <bool OUT_BF16, bool VEC_STORE, class LA, class LB>
__device__ __forceinline__ void tile_product2(const LA &la, const LB &lb, void *Cv, int ldc, int M, int N, int K, int m0,
                                              int n0, bool relu, char *smem)
{
    constexpr int TM = 4, TN = 2, WN = 4; // 2 x 4 waves, 128 x 64 per wave
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave / WN) * (TM * 32), wn0 = (wave % WN) * (TN * 32);
    constexpr int A_BYTES = BM2 * BK * 2;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    const int nk = (K + BK - 1) / BK;
    la.template issue<BM2>(m0, 0, smem);
    lb.template issue<BN2>(n0, 0, smem + A_BYTES);

    for (int kt = 0; kt < nk; ++kt) {
        char *cur = smem + (kt & 1) * kStageBytes, *nxt = smem + ((kt & 1) ^ 1) * kStageBytes;
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's chunks of tile kt have landed
        __syncthreads();                     // everyone's have; and everyone is done reading the other stage
        if (kt + 1 < nk) {
            la.template issue<BM2>(m0, (kt + 1) * BK, nxt);
            lb.template issue<BN2>(n0, (kt + 1) * BK, nxt + A_BYTES);
        }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_iglp_opt(1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = read_frag<BM2, LA::KC>(cur, wm0 + i * 32, ks, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = read_frag<BN2, LB::KC>(cur + A_BYTES, wn0 + j * 32, ks, lane);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads(); // all fragment reads done before the staging area is reused

    const int col_l = lane & 31, row_l = (lane >> 5) * 4;
    if constexpr (!VEC_STORE) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn0 + j * 32 + col_l;
                if (col >= N) continue;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wm0 + i * 32 + 8 * (e >> 2) + row_l + (e & 3);
                    if (row >= M) continue;
                    float v = acc[i][j][e];
                    if (relu) v = fmaxf(v, 0.0f);
                    if (OUT_BF16) reinterpret_cast<uint16_t *>(Cv)[(size_t)row * ldc + col] = (uint16_t)core::f32_to_bf16_bits(v);
                    else reinterpret_cast<float *>(Cv)[(size_t)row * ldc + col] = v;
                }
            }
    } else {
        constexpr int SW = TN * 32, SLD = SW + 4;
        float *strip = reinterpret_cast<float *>(smem) + wave * (32 * SLD);
        static_assert(8 * 32 * SLD * sizeof(float) <= kSmemBytes, "strip staging fits");
        constexpr int EPV = OUT_BF16 ? 8 : 4, VPR = SW / EPV, RPI = 64 / VPR;
        const int vr = lane / VPR, vc = (lane % VPR) * EPV;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float v = acc[i][j][e];
                    if (relu) v = fmaxf(v, 0.0f);
                    strip[(8 * (e >> 2) + row_l + (e & 3)) * SLD + j * 32 + col_l] = v;
                }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int rr = 0; rr < 32; rr += RPI) {
                const int srow = rr + vr;
                const int row = m0 + wm0 + i * 32 + srow, col = n0 + wn0 + vc;
                const float *sp = strip + srow * SLD + vc;
                if (row < M && col < N) {
                    if constexpr (OUT_BF16) {
                        f32x4 x = *reinterpret_cast<const f32x4 *>(sp), y = *reinterpret_cast<const f32x4 *>(sp + 4);
                        u32x4 o = {core::pack_bf16x2(x[0], x[1]), core::pack_bf16x2(x[2], x[3]), core::pack_bf16x2(y[0], y[1]),
                                   core::pack_bf16x2(y[2], y[3])};
                        __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(reinterpret_cast<uint16_t *>(Cv) + (size_t)row * ldc + col));
                    } else {
                        __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(sp),
                                                    reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(Cv) + (size_t)row * ldc + col));
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

} // namespace core2
} // namespace tt
