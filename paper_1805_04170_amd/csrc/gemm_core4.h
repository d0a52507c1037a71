// Fourth bf16 MFMA tile engine: 256 x 128 output tiles, four waves, TWO workgroups resident per CU.
//
// The engines with one 256 x 256 workgroup per CU run their phases one after the other on a CU: fill the pipeline,
// multiply, write the tile out.  For products with a short K loop and a large output (the weight gradients at batch
// 256: four 64-deep K tiles per 128 KB output tile) the write-out is as long as the multiplication.  Here a workgroup
// needs half the registers and less than half the LDS of a CU, so two of them share it and the hardware interleaves
// them: while one stores its tile the other one multiplies.
//
//   - four waves as 2 x 2, 128 x 64 per wave (the same wave tile as the 256 x 256 engines);
//   - K tiles of 32; a stage is 16 KB of A and 8 KB of B; three stages (72 KB) fetched global -> LDS with
//     global_load_lds_dwordx4 two tiles ahead (inline assembly, see gemm_core2.h for why);
//   - LDS layouts: K-contiguous operands as [row][4 chunks of 8 k], chunk position p of row r holds k-chunk
//     p ^ ((r >> 2) & 3); row-contiguous operands as [k][ROWS / 8 chunks of 8 rows], swizzled and read with LDS
//     transpose reads as in gemm_core2.h;
//   - K must be a multiple of 32; a workgroup computes one tile and ends (the other resident workgroup and the next
//     one queued cover its start-up and wind-down);
//   - epilogue: bf16 results with 16-byte rows are turned around in a wave-private strip of the (drained) ring, 16 rows
//     at a time; everything else is stored element-wise from the accumulators.
#pragma once
#include <cstdint>
#include "tt_device.h"
#include "gemm_core.h"
#include "gemm_core2.h"
#include "gemm_core3.h"

namespace tt {
namespace core4 {

using core::bf16x8;
using core::f32x16;
using core::u32x4;
using core2::s16x4;

constexpr int kThreads4 = 256;
constexpr int BM4 = 256, BN4 = 128, BK4 = 32, NS4 = 3;
constexpr int kABytes = BM4 * BK4 * 2, kBBytes = BN4 * BK4 * 2, kStage4 = kABytes + kBBytes; // 16 KB + 8 KB
constexpr size_t kSmem4 = (size_t)NS4 * kStage4;                                              // 72 KB
constexpr int kLoadsA = kABytes / 16 / kThreads4, kLoadsB = kBBytes / 16 / kThreads4;        // 4 and 2 per thread

// lane offsets of this thread's 16-byte chunks of one operand tile (ROWS x 32), see the layouts above
template <int ROWS, bool KC> __device__ __forceinline__ void chunk_offsets(int row0, int rows, int ld, uint32_t *voff)
{
    const int tid = threadIdx.x;
    constexpr int NL = ROWS * BK4 * 2 / 16 / kThreads4;
    if constexpr (KC) {
        // chunk c = tid + 256 i: row c / 4 = tid / 4 + 64 i, position c % 4
        const int rl = tid >> 2;
        const int kc = (tid & 3) ^ ((rl >> 2) & 3);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            int r = row0 + rl + 64 * i;
            r = r < rows ? r : rows - 1; // rows past the end only feed C rows / columns that are never stored
            voff[i] = (uint32_t)r * (uint32_t)ld * 2u + (uint32_t)kc * 16u;
        }
    } else {
        // chunk c = tid + 256 i: k-row c / CPR, position c % CPR holds row-chunk position ^ ((k & 3) << 1)
        constexpr int CPR = ROWS / 8;           // 32 or 16 chunks per k-row
        constexpr int KPI = kThreads4 / CPR;    // k-rows covered per i: 8 or 16 (multiples of 4: k & 3 does not depend on i)
        const int kl = tid / CPR;
        const int rc = (tid % CPR) ^ ((kl & 3) << 1);
        int r = row0 + rc * 8;
        r = r < rows ? r : rows - 8;
#pragma unroll
        for (int i = 0; i < NL; ++i) voff[i] = (uint32_t)(kl + KPI * i) * (uint32_t)ld * 2u + (uint32_t)r * 2u;
    }
}

template <int NL> __device__ __forceinline__ void issue_chunks(const char *base, const uint32_t *voff, uint32_t lds)
{
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // the base is wave-uniform by construction; say so, or the "s" operand may be handed a vector register pair
    // (readfirstlane returns a signed int: go through uint32_t so the low half is not sign-extended)
    const uint64_t b64 = reinterpret_cast<uint64_t>(base);
    const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b64);
    const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b64 >> 32));
    const uint64_t sbase = ((uint64_t)b_hi << 32) | (uint64_t)b_lo;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const uint32_t dst = lds + (wave * 64u + (uint32_t)i * kThreads4) * 16u;
        dev::lds_dma16(voff[i], sbase, dst);
    }
}

// fragment (32 rows x 16 k) of an operand stage: rows rbase .. rbase+31 of the tile, k-step ks (0 or 1)
template <int ROWS, bool KC> __device__ __forceinline__ bf16x8 read_frag4(const char *lds, int rbase, int ks, int lane)
{
    if constexpr (KC) {
        const int r = rbase + (lane & 31), q = ks * 2 + (lane >> 5);
        return *reinterpret_cast<const bf16x8 *>(lds + r * 64 + ((q ^ ((r >> 2) & 3)) << 4));
    } else {
        return core2::read_frag<ROWS, false>(lds, rbase, ks, lane);
    }
}

// Write-out of a workgroup's 256 x 128 accumulator tile (four waves as 2 x 2, 128 x 64 per wave: the wave tile of this
// engine and of gemm_core6.h).  The ring must be drained and idle: STAGED turns the results round in a wave-private
// strip at the start of smem (at least 4 * 16 * 72 * 2 bytes; bf16 16 rows at a time, fp32 8) so that they leave as
// 16-byte vectors of whole row segments; without it they are stored element by element.
template <bool OUT_BF16, bool STAGED>
__device__ __forceinline__ void write_tile4(f32x16 (&acc)[4][2], void *Cv, int ldc, int M, int N, int m0, int n0, bool relu,
                                            char *smem)
{
    constexpr int TM = 4, TN = 2, WN = 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave / WN) * (TM * 32), wn0 = (wave % WN) * (TN * 32);
    // ---- epilogue.  A lane holds column (lane & 31) and rows 8*(e/4) + 4*(lane/32) + e%4 of each 32 x 32 block.
    const int col_l = lane & 31, row_l = (lane >> 5) * 4;
    if constexpr (STAGED && !OUT_BF16) {
        static_assert(4 * core3::kEpiRowsF * core3::kEpiLdF * 4 <= kSmem4, "strips fit in the ring");
        float *strip = reinterpret_cast<float *>(smem) + wave * (core3::kEpiRowsF * core3::kEpiLdF);
        core3::store_wave_tile_f32(acc, strip, reinterpret_cast<float *>(Cv), ldc, m0 + wm0, n0 + wn0, M, N, relu, lane);
    } else if constexpr (!STAGED) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn0 + j * 32 + col_l;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + wm0 + i * 32 + 8 * (e >> 2) + row_l + (e & 3);
                    float v = acc[i][j][e];
                    if (relu) v = fmaxf(v, 0.0f);
                    if (row < M && col < N) {
                        if constexpr (OUT_BF16)
                            reinterpret_cast<uint16_t *>(Cv)[(size_t)row * ldc + col] = (uint16_t)core::f32_to_bf16_bits(v);
                        else
                            __builtin_nontemporal_store(v, reinterpret_cast<float *>(Cv) + (size_t)row * ldc + col);
                    }
                }
            }
    } else {
        constexpr int ER = 16, ELD = 64 + 8; // strip of one wave: 16 rows x 64 columns of bf16, padded
        static_assert(4 * ER * ELD * 2 <= kSmem4, "strips fit in the ring");
        uint16_t *strip = reinterpret_cast<uint16_t *>(smem) + wave * (ER * ELD);
        uint16_t *Cs = reinterpret_cast<uint16_t *>(Cv);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int eg = 0; eg < 2; ++eg)
#pragma unroll
                        for (int ee = 0; ee < 4; ee += 2) {
                            float v0 = acc[i][j][(2 * h + eg) * 4 + ee], v1 = acc[i][j][(2 * h + eg) * 4 + ee + 1];
                            if (relu) { v0 = fmaxf(v0, 0.0f); v1 = fmaxf(v1, 0.0f); }
                            const uint32_t pk = core::pack_bf16x2(v0, v1);
                            uint16_t *d = strip + (8 * eg + row_l + ee) * ELD + j * 32 + col_l;
                            d[0] = (uint16_t)(pk & 0xffffu);
                            d[ELD] = (uint16_t)(pk >> 16);
                        }
                // Wave-private data: LDS operations of one wave execute in order, so the reads below see the writes above and the
                // next strip's writes cannot overtake them; no wait is needed, only a fence for the compiler's scheduler.
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int v = 0; v < 2; ++v) {
                    const int idx = lane + 64 * v, lrow = idx >> 3, vc = (idx & 7) * 8;
                    const int row = m0 + wm0 + i * 32 + 16 * h + lrow, col = n0 + wn0 + vc;
                    const u32x4 o = *reinterpret_cast<const u32x4 *>(strip + lrow * ELD + vc);
                    if (row < M && col < N) // N is a multiple of 8 on this path: a vector is all in or all out
                        __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(Cs + (size_t)row * ldc + col));
                }
                __builtin_amdgcn_wave_barrier();
            }
    }
}

// C tile (m0, n0) of C = A B over K = klen (a multiple of 32) starting at the operands' k = 0 as given by abase / bbase.
// 256 threads; smem: kSmem4 bytes, 16-byte aligned.  STAGED: bf16 result, 16-byte stores legal.
template <bool A_KC, bool B_KC, bool OUT_BF16, bool STAGED>
__device__ __forceinline__ void tile_product4(const char *abase, int lda, const char *bbase, int ldb, void *Cv, int ldc, int M,
                                              int N, int klen, int m0, int n0, bool relu, char *smem)
{
    constexpr int TM = 4, TN = 2, WN = 2; // 2 x 2 waves, 128 x 64 per wave
    constexpr int D = NS4 - 1;
    constexpr int W = (D - 1) * (kLoadsA + kLoadsB); // loads that may still be in flight at the top of an item
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave / WN) * (TM * 32), wn0 = (wave % WN) * (TN * 32);
    const uint32_t lds0 = dev::lds_addr(smem);

    uint32_t voa[kLoadsA], vob[kLoadsB];
    chunk_offsets<BM4, A_KC>(m0, M, lda, voa);
    chunk_offsets<BN4, B_KC>(n0, N, ldb, vob);
    const uint32_t astep = A_KC ? BK4 * 2u : (uint32_t)BK4 * (uint32_t)lda * 2u;
    const uint32_t bstep = B_KC ? BK4 * 2u : (uint32_t)BK4 * (uint32_t)ldb * 2u;
    const int nk = klen / BK4;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Every item issues the same number of loads so that the wait count stays constant: past the end of K the last
    // tile is fetched again into a stage nobody reads any more.
    int it_issue = 0, is = 0;
    auto issue = [&]() {
        const int kt = it_issue < nk ? it_issue : nk - 1;
        issue_chunks<kLoadsA>(abase + (size_t)kt * astep, voa, lds0 + (uint32_t)is * kStage4);
        issue_chunks<kLoadsB>(bbase + (size_t)kt * bstep, vob, lds0 + (uint32_t)is * kStage4 + kABytes);
        ++it_issue;
        is = is + 1 == NS4 ? 0 : is + 1;
    };
#pragma unroll
    for (int s = 0; s < D; ++s) issue();

    int cs = 0;
    for (int kt = 0; kt < nk; ++kt) {
        __builtin_amdgcn_s_waitcnt(core3::waitcnt_vm(W)); // this wave's chunks of the item have landed
        __syncthreads();                                  // everyone's have; everyone has finished reading the previous item
        issue();                                          // into the stage of the previous item
        const char *As = smem + cs * kStage4, *Bs = As + kABytes;
        cs = cs + 1 == NS4 ? 0 : cs + 1;
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_iglp_opt(1);
#pragma unroll
        for (int ks = 0; ks < BK4 / 16; ++ks) {
            bf16x8 af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = read_frag4<BM4, A_KC>(As, wm0 + i * 32, ks, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = read_frag4<BN4, B_KC>(Bs, wn0 + j * 32, ks, lane);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    // the re-fetches issued past the end have landed and every wave is done with the ring: it can be reused / given up
    __builtin_amdgcn_s_waitcnt(core3::waitcnt_vm(0));
    __syncthreads();
    write_tile4<OUT_BF16, STAGED>(acc, Cv, ldc, M, N, m0, n0, relu, smem);
}

} // namespace core4
} // namespace tt
