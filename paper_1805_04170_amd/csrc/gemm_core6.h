// Sixth bf16 MFMA tile engine: skinny products C_s = A_s B_s^T whose two operands both have K contiguous (the data
// gradients dC/dx_{l-1} = df(dC/dx_l) W_l^T of Sec. 2.1 of arXiv 1805.04170 at batch 256: one row of 256 x 128 tiles,
// bound by streaming the weights once from HBM next to a small operand that every workgroup takes in from L2).
//
// What the 256 x 128 engine of gemm_core4.h leaves on the table there: with K tiles of 32 every load takes 64 bytes out
// of each weight row, and the next 64 bytes of the same rows are asked for one K step later.  Measured on MI355X with
// the memory skeleton of that K loop (same loads, no arithmetic): a streamed operand fetched in 64-byte pieces at an
// 8 KB pitch arrives at 2.8 TB/s over the chip beside the shared operand, in 128-byte pieces (whole cache lines) at
// 3.5 TB/s, and the engine itself runs exactly at its skeleton's rate; ring depth beyond two tiles in flight changes
// neither.  So this engine differs from gemm_core4.h in the shape of its K tiles, not in its tile or wave layout:
//   - 256 x 128 output tiles, four waves as 2 x 2, 128 x 64 per wave, one workgroup per CU (the launches it is used for
//     have at most one workgroup per CU anyway);
//   - K tiles of 64: a lane group of eight fetches one whole 128-byte line of a row;
//   - the streamed operand B (16 KB per K tile) has three stages, two tiles in flight; the L2-resident operand A (32 KB
//     per K tile) has two stages, one tile in flight: 112 KB of LDS, all of it below 128 KB;
//   - LDS layout of both operands: [row][8 chunks of 8 k], chunk position p of row r holds k-chunk p ^ ((r >> 1) & 7),
//     fragments are plain 16-byte reads (the K-contiguous layout of gemm_core2.h).  (B may also be given with its rows
//     contiguous, K x N: the [k][16 chunks of 8 columns] layout and the LDS transpose reads of gemm_core2.h; built to
//     measure the forward products with it, which came out no faster than on gemm_core4.h, so the launch code only
//     takes that form when the engine is forced;)
//   - waits count operations: the loads are issued in the order B(0) A(0) B(1) | A(1) B(2) | A(2) B(3) | ..., so at the
//     top of step kt everything but the newest B tile (four loads per lane) has to be complete: s_waitcnt vmcnt(4)
//     (a wave's loads retire in order on that counter).  Past the end of K the last tile is fetched again into stages
//     nobody reads any more, so the count stays constant;
//   - K must be a multiple of 64.  Write-out: gemm_core4.h's.
#pragma once
#include <cstdint>
#include "tt_device.h"
#include "gemm_core.h"
#include "gemm_core2.h"
#include "gemm_core3.h"
#include "gemm_core4.h"

namespace tt {
namespace core6 {

using core::bf16x8;
using core::f32x16;

constexpr int kThreads6 = 256;
constexpr int BM6 = 256, BN6 = 128, BK6 = 64, NSA6 = 2, NSB6 = 3;
constexpr int kABytes6 = BM6 * BK6 * 2, kBBytes6 = BN6 * BK6 * 2;                    // 32 KB and 16 KB
constexpr size_t kSmem6 = (size_t)NSA6 * kABytes6 + (size_t)NSB6 * kBBytes6;          // 112 KB
constexpr int kLoadsA6 = kABytes6 / 16 / kThreads6, kLoadsB6 = kBBytes6 / 16 / kThreads6; // 8 and 4 per thread
static_assert(kSmem6 <= 128 * 1024, "every global -> LDS landing address stays below 128 KB");

// lane offsets of this thread's 16-byte chunks of one operand tile (ROWS x 64).  K contiguous: chunk c = tid + 256 i lies
// in row c / 8 = tid / 8 + 32 i at position c % 8 and holds k-chunk position ^ ((row >> 1) & 7), which does not depend on
// i.  Rows contiguous (the layout of gemm_core2.h / gemm_core4.h): chunk c lies in k-row c / CPR = tid / CPR + KPI i at
// position c % CPR and holds row-chunk position ^ ((k & 3) << 1); KPI is a multiple of 4, so that does not depend on i.
template <int ROWS, bool KC> __device__ __forceinline__ void chunk_offsets6(int row0, int rows, int ld, uint32_t *voff)
{
    const int tid = threadIdx.x;
    constexpr int NL = ROWS * BK6 * 2 / 16 / kThreads6;
    if constexpr (KC) {
        const int rl = tid >> 3;
        const int kc = (tid & 7) ^ ((rl >> 1) & 7);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            int r = row0 + rl + 32 * i;
            r = r < rows ? r : rows - 1; // rows past the end only feed C rows / columns that are never stored
            voff[i] = (uint32_t)r * (uint32_t)ld * 2u + (uint32_t)kc * 16u;
        }
    } else {
        constexpr int CPR = ROWS / 8;
        constexpr int KPI = kThreads6 / CPR;
        static_assert(KPI % 4 == 0 && KPI * NL == BK6, "k-rows per load");
        const int kl = tid / CPR;
        const int rc = (tid % CPR) ^ ((kl & 3) << 1);
        int r = row0 + rc * 8;
        r = r < rows ? r : rows - 8;
#pragma unroll
        for (int i = 0; i < NL; ++i) voff[i] = (uint32_t)(kl + KPI * i) * (uint32_t)ld * 2u + (uint32_t)r * 2u;
    }
}

// C tile (m0, n0) of C = A B over K = klen (a multiple of 64) starting at the operands' k = 0 as given by abase / bbase;
// A is M x K with pitch lda; B is N x K with pitch ldb (B_KC) or K x N with pitch ldb (fragments through LDS transpose
// reads).  256 threads; smem: kSmem6 bytes, 16-byte aligned.  STAGED: bf16 result, 16-byte stores legal.
template <bool B_KC, bool OUT_BF16, bool STAGED>
__device__ __forceinline__ void tile_product6(const char *abase, int lda, const char *bbase, int ldb, void *Cv, int ldc, int M,
                                              int N, int klen, int m0, int n0, bool relu, char *smem)
{
    constexpr int TM = 4, TN = 2, WN = 2; // 2 x 2 waves, 128 x 64 per wave
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave / WN) * (TM * 32), wn0 = (wave % WN) * (TN * 32);
    const uint32_t lds0 = dev::lds_addr(smem);
    constexpr uint32_t kBRing = (uint32_t)NSA6 * kABytes6; // the B stages follow the A stages

    uint32_t voa[kLoadsA6], vob[kLoadsB6];
    chunk_offsets6<BM6, true>(m0, M, lda, voa);
    chunk_offsets6<BN6, B_KC>(n0, N, ldb, vob);
    const size_t bstep = B_KC ? (size_t)BK6 * 2 : (size_t)BK6 * (size_t)ldb * 2;
    const int nk = klen / BK6;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    int ia = 0, sa = 0, ib = 0, sb = 0; // next tile to ask for and the stage it goes to, per operand
    auto issue_a = [&]() {
        const int kt = ia < nk ? ia : nk - 1;
        core4::issue_chunks<kLoadsA6>(abase + (size_t)kt * (BK6 * 2), voa, lds0 + (uint32_t)sa * kABytes6);
        ++ia;
        sa ^= 1;
    };
    auto issue_b = [&]() {
        const int kt = ib < nk ? ib : nk - 1;
        core4::issue_chunks<kLoadsB6>(bbase + (size_t)kt * bstep, vob, lds0 + kBRing + (uint32_t)sb * kBBytes6);
        ++ib;
        sb = sb + 1 == NSB6 ? 0 : sb + 1;
    };
    issue_b();
    issue_a();
    issue_b();

    int ca = 0, cb = 0;
    for (int kt = 0; kt < nk; ++kt) {
        __builtin_amdgcn_s_waitcnt(core3::waitcnt_vm(kLoadsB6)); // all but the newest B tile: this step's A and B have landed
        __syncthreads();                                         // everyone's have; everyone has finished reading step kt - 1
        issue_a();                                               // A(kt + 1) into the stage of A(kt - 1)
        issue_b();                                               // B(kt + 2) into the stage of B(kt - 1)
        const char *As = smem + ca * kABytes6, *Bs = smem + kBRing + cb * kBBytes6;
        ca ^= 1;
        cb = cb + 1 == NSB6 ? 0 : cb + 1;
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_iglp_opt(1);
#pragma unroll
        for (int ks = 0; ks < BK6 / 16; ++ks) {
            bf16x8 af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = core2::read_frag<BM6, true>(As, wm0 + i * 32, ks, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = core2::read_frag<BN6, B_KC>(Bs, wn0 + j * 32, ks, lane);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    // the re-fetches issued past the end have landed and every wave is done with the rings: they can be reused / given up
    __builtin_amdgcn_s_waitcnt(core3::waitcnt_vm(0));
    __syncthreads();
    core4::write_tile4<OUT_BF16, STAGED>(acc, Cv, ldc, M, N, m0, n0, relu, smem);
}

} // namespace core6
} // namespace tt
