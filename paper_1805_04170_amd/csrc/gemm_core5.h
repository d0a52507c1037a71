// Fifth bf16 MFMA engine: products with a SHORT contraction and a LARGE result, C_s = A_s^T B_s with A_s stored K x M and
// B_s stored K x N (both with K as the slow dimension) and K = 128, 256 or 512.  These are the weight gradients
// dC/dW_l = x_l^T df(dC/dx_{l+1}) of Sec. 2.1 of arXiv 1805.04170 at a per-shard batch of 128 / 256: 2 K flops per result
// element, so the product is bound by writing C, and the job of the kernel is to keep the chip writing.
//
// What keeps the other engines from that: they walk K in tiles, so the loads of a tile's later K steps are issued after the
// stores of the previous tile and queue behind them in the CU's memory pipeline; multiplication and write-out of a CU then
// take turns instead of overlapping.  Here K is so short that one operand stays in registers for its whole length:
//   - a workgroup of four waves owns a PANEL of 256 rows of C (64 per wave).  Each wave keeps its 64 x K slice of A^T in
//     registers (2 x K/16 MFMA fragments, 128 VGPRs at K = 256), loaded once per panel through LDS with transpose reads;
//   - the workgroup then walks UNITS of 64 columns of C.  A unit needs one B tile (K x 64, 32 KB at K = 256), fetched
//     global -> LDS one unit ahead into a two-stage ring: every load a unit needs is issued BEFORE the previous unit's
//     stores, so nothing a unit waits for queues behind stores, and the stores of unit u drain while unit u + 1 multiplies;
//   - waits count operations instead of draining: at the top of a unit the wave's outstanding vector-memory operations
//     are, oldest first, this unit's B loads and the previous unit's 8 stores, so s_waitcnt vmcnt(8) is exactly "my B
//     chunks have landed" (loads and stores of a wave retire in order on this counter).  Waves whose panel rows are
//     partly past M store under a row mask, where the number of issued stores is not fixed: they wait for zero instead;
//   - 80 KB of LDS and at most 256 registers per lane, so TWO workgroups share a CU and cover each other's panel
//     changes, barriers and epilogues;
//   - K = 512 (weight gradients at a per-shard batch of 512: compute-bound, 4 K flops per result element) runs the same
//     way with ONE workgroup per CU: the panel takes 256 registers per lane and the two B stages 128 KB.  What it buys
//     there is LDS traffic: only B goes through LDS (two fragment reads per four products instead of six per eight),
//     where the tile engines that read both operands through LDS transpose reads are bound by LDS;
//   - the grid is persistent: each workgroup takes a contiguous run of units (shard-major, panel, column tile).
//
// LDS layouts (XOR-swizzled by the choice of which global chunk a lane fetches, as in gemm_core2.h):
//   A staging  [k][32 chunks of 8 rows], half a panel's K at a time: the layout and fragment read of gemm_core2.h
//              (row-contiguous operand, 256 rows);
//   B stage    [k][8 chunks of 8 columns]: chunk position p of k-row k holds column chunk p ^ (((k >> 1) & 1) << 1);
//              fragments are two ds_read_b64_tr_b16 as in gemm_core2.h (with 128-byte k-rows, rows k and k + 2 share
//              banks, hence the different swizzle).
#pragma once
#include <cstdint>
#include "tt_device.h"
#include "gemm_core.h"
#include "gemm_core2.h"
#include "gemm_core3.h"

namespace tt {
namespace core5 {

using core::bf16x8;
using core::f32x16;
using core::u32x4;
using core2::s16x4;

constexpr int kThreads5 = 256;
constexpr int PM5 = 256; // rows of C per panel (64 per wave)
constexpr int NT5 = 64;  // columns of C per unit
constexpr int kEpiRows5 = 32;                                                 // rows of a wave's result strip
constexpr int kEpiBytes5 = 4 * kEpiRows5 * NT5 * 2;                           // 16 KB: one 32 x 64 bf16 strip per wave
constexpr int kStoresPerUnit5 = 64 * NT5 * 2 / (64 * 16);                     // 16-byte stores per wave and unit: 8
template <int KT> constexpr int stage_bytes5() { return KT * 16 * NT5 * 2; }  // one B tile: K x 64
template <int KT> constexpr size_t smem_bytes5() { return 2 * (size_t)stage_bytes5<KT>() + kEpiBytes5; }

struct Params5 {
    const void *A[64]; // K x M row-major (A^T is the left operand)
    const void *B[64]; // K x N row-major
    void *C[64];       // M x N row-major, bf16
    int32_t M, N;
    int32_t lda, ldb, ldc;
    int32_t panels, ntiles; // per shard
    int32_t total;          // count * panels * ntiles
    int32_t grid;           // workgroups launched
    int32_t relu;
};

// B fragment (32 columns x 16 k) of a stage: columns cbase .. cbase + 31 of the unit, k-step ks
__device__ __forceinline__ bf16x8 read_frag_b5(const char *lds, int cbase, int ks, int lane)
{
    const int g16 = lane >> 4, j = lane & 15;
    const int n0 = cbase + (g16 & 1) * 16 + 4 * (j & 3); // first of this lane's 4 addressed columns
    const int c = n0 >> 3, byte = (n0 & 7) * 2;
    union { s16x4 h[2]; bf16x8 v; } u;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int k = ks * 16 + (g16 >> 1) * 8 + h * 4 + (j >> 2);
        const char *a = lds + k * (NT5 * 2) + ((c ^ (((k >> 1) & 1) << 1)) << 4) + byte;
        u.h[h] = dev::lds_read_tr16_b64(a);
    }
    return u.v;
}

__device__ __forceinline__ uint64_t uniform64(const char *p)
{
    // wave-uniform by construction; say so, or an "s" operand may be handed a vector register pair (readfirstlane
    // returns a signed int: go through uint32_t so the low half is not sign-extended)
    const uint64_t b64 = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b64);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b64 >> 32));
    return ((uint64_t)hi << 32) | (uint64_t)lo;
}

// KT = K / 16 (8, 16 or 32).  NTS: non-temporal stores.  256 threads; smem: smem_bytes5<KT>() bytes, 16-byte aligned.
template <int KT, bool NTS> __device__ __forceinline__ void run_panels(const Params5 &p, char *smem)
{
    static_assert(KT == 8 || KT == 16 || KT == 32, "K = 128, 256 or 512");
    constexpr int STB = stage_bytes5<KT>();
    constexpr int NLB = KT / 2; // B loads per thread and unit: k-rows tid / 8 + 32 i
    constexpr int ACH = KT * 8; // k-rows per A staging step (half of K): fills both stages
    constexpr int NLA = KT;     // A loads per thread and staging step: k-rows tid / 32 + 8 i
    constexpr int S = kStoresPerUnit5;
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (int)wave * 64;
    const uint32_t lds0 = dev::lds_addr(smem);
    const int M = p.M, ldc = p.ldc;

    // contiguous run of units; workgroup numbers go round-robin over the XCDs, so give every XCD a contiguous range
    const uint32_t bid = blockIdx.x, grid = (uint32_t)p.grid;
    const uint32_t lw = grid % core::kXcds == 0 ? (bid % core::kXcds) * (grid / core::kXcds) + bid / core::kXcds : bid;
    int64_t u = (int64_t)lw * p.total / grid;
    const int64_t end = (int64_t)(lw + 1) * p.total / grid;

    // lane parts of the load addresses
    const uint32_t bkl = (uint32_t)tid >> 3, bpc = (uint32_t)tid & 7u;
    const uint32_t voff_b = bkl * (uint32_t)p.ldb * 2u + ((bpc ^ (((bkl >> 1) & 1u) << 1)) << 4);
    const uint32_t akl = (uint32_t)tid >> 5, apc = (uint32_t)tid & 31u;
    const int a_chunk = (int)(apc ^ ((akl & 3u) << 1));

    // Result strip of the wave: 32 rows of 128 bytes.  The products are formed as (B tile) x (A panel)^T, so a lane
    // holds row (lane & 31) of a 32 x 32 block of C and, per register group g, the four consecutive columns
    // 8 g + 4 (lane / 32) + 0..3: eight bytes, written with one LDS store.  Row r keeps its 16-byte piece c at position
    // c ^ ((r >> 1) & 7) and, for r >= 16, the two halves of a piece exchanged: the 32 rows written together then fall
    // into 32 different bank pairs, and the 16-byte reads of the row-contiguous write-out stay conflict-free.
    char *strip = smem + 2 * STB + wave * (kEpiRows5 * NT5 * 2);
    const int srow = lane & 31;
    char *swr = strip + srow * (NT5 * 2) + ((((lane >> 5) ^ (srow >> 4)) & 1) << 3);
    const int sswz = (srow >> 1) & 7;
    // write-out: lane l takes piece l % 8 of strip row l / 8 + 8 v (v = 0..3); (row >> 1) & 7 = ((l >> 4) + 4 v) & 7, so
    // the swizzled position is that of v = 0 with bit 2 flipped for odd v; rows 16.. have their halves exchanged
    const char *srd[2];
    srd[0] = strip + (lane >> 3) * (NT5 * 2) + (((lane & 7) ^ ((lane >> 4) & 7)) << 4);
    srd[1] = strip + (lane >> 3) * (NT5 * 2) + (((lane & 7) ^ ((lane >> 4) & 7) ^ 4) << 4);
    const uint32_t st_off = (uint32_t)((lane >> 3) * ldc + (lane & 7) * 8) * 2u; // lane part of the store address
    const float floor_v = p.relu ? 0.0f : -__builtin_inff(); // the element-wise function as one maximum, no branch
    const int per_shard = p.panels * p.ntiles;

    while (u < end) {
        const int shard = (int)(u / per_shard);
        const int r = (int)(u - (int64_t)shard * per_shard);
        const int panel = r / p.ntiles, nt0 = r - panel * p.ntiles;
        const int run = (int)(end - u < (int64_t)(p.ntiles - nt0) ? end - u : (int64_t)(p.ntiles - nt0));
        const int m0 = panel * PM5;

        // ---- the panel's slice of A^T into registers, half of K at a time through the (idle) B stages
        __builtin_amdgcn_s_waitcnt(core3::waitcnt_vm(0));
        __syncthreads(); // nobody still reads a stage
        bf16x8 af[2][KT];
        {
            int col = m0 + a_chunk * 8;
            col = col < M ? col : M - 8; // columns past M only feed rows of C that are never stored
            const uint32_t voff_a = akl * (uint32_t)p.lda * 2u + (uint32_t)col * 2u;
            const char *abase = reinterpret_cast<const char *>(p.A[shard]);
#pragma unroll
            for (int c = 0; c < 2; ++c) {
#pragma unroll
                for (int i = 0; i < NLA; ++i) {
                    const uint64_t sb = uniform64(abase + (size_t)(c * ACH + 8 * i) * (size_t)p.lda * 2);
                    dev::lds_dma16(voff_a, sb, lds0 + (wave * 64u + (uint32_t)i * kThreads5) * 16u);
                }
                __builtin_amdgcn_s_waitcnt(core3::waitcnt_vm(0));
                __syncthreads();
#pragma unroll
                for (int ks = 0; ks < KT / 2; ++ks)
#pragma unroll
                    for (int i = 0; i < 2; ++i) af[i][c * (KT / 2) + ks] = core2::read_frag<256, false>(smem, wm0 + i * 32, ks, lane);
                __syncthreads(); // everyone has its fragments before the staging area is overwritten
            }
        }

        const char *bbase = reinterpret_cast<const char *>(p.B[shard]);
        auto issue_b = [&](int nt, int stage) {
#pragma unroll
            for (int i = 0; i < NLB; ++i) {
                const uint64_t sb = uniform64(bbase + (size_t)nt * (NT5 * 2) + (size_t)(32 * i) * (size_t)p.ldb * 2);
                dev::lds_dma16(voff_b, sb, lds0 + (uint32_t)stage * STB + (wave * 64u + (uint32_t)i * kThreads5) * 16u);
            }
        };
        issue_b(nt0, 0);
        int cs = 0;
        // rows m0 + wm0 .. + 63 of this wave all inside C: its stores are unconditional and their number is fixed
        const bool full = __builtin_amdgcn_readfirstlane((int)(m0 + wm0 + 64 <= M)) != 0;
        uint16_t *Cs = reinterpret_cast<uint16_t *>(p.C[shard]);

        for (int q = 0; q < run; ++q) {
            // my chunks of this unit's B tile have landed: everything but the previous unit's stores is complete
            if (q > 0 && full) __builtin_amdgcn_s_waitcnt(core3::waitcnt_vm(S));
            else __builtin_amdgcn_s_waitcnt(core3::waitcnt_vm(0));
            __syncthreads(); // everyone's have; everyone has finished reading the other stage
            if (q + 1 < run) issue_b(nt0 + q + 1, cs ^ 1);
            const char *Bs = smem + cs * STB;
            cs ^= 1;

            f32x16 acc[2][2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
            // the B fragments are requested LOOK k-steps before the products that use them are issued: under load the LDS
            // latency of the transpose reads is longer than the four products of one step (with one workgroup per CU,
            // K = 512, no other wave of the SIMD fills the gap: four steps ahead there, two otherwise)
            constexpr int LOOK = KT > 16 ? 4 : 2;
            bf16x8 bq[LOOK + 1][2];
#pragma unroll
            for (int a = 0; a < LOOK; ++a) {
                bq[a][0] = read_frag_b5(Bs, 0, a, lane);
                bq[a][1] = read_frag_b5(Bs, 32, a, lane);
            }
#pragma unroll
            for (int ks = 0; ks < KT; ++ks) {
                const bf16x8 b0 = bq[ks % (LOOK + 1)][0], b1 = bq[ks % (LOOK + 1)][1];
                if (ks + LOOK < KT) {
                    bq[(ks + LOOK) % (LOOK + 1)][0] = read_frag_b5(Bs, 0, ks + LOOK, lane);
                    bq[(ks + LOOK) % (LOOK + 1)][1] = read_frag_b5(Bs, 32, ks + LOOK, lane);
                }
                __builtin_amdgcn_sched_barrier(0); // (left alone, the scheduler starts the next step's products early and waits for these reads)
                // operands exchanged: the accumulators hold blocks of C^T (see the strip above)
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0, af[0][ks], acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1, af[0][ks], acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0, af[1][ks], acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1, af[1][ks], acc[1][1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }

            // ---- epilogue: 32 rows of the wave's 64 at a time through its strip, then out as 16-byte pieces of whole
            // 128-byte rows (8 lanes per row, 8 rows per store instruction)
            const int n0 = (nt0 + q) * NT5;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float v0 = acc[i][j][4 * g], v1 = acc[i][j][4 * g + 1], v2 = acc[i][j][4 * g + 2], v3 = acc[i][j][4 * g + 3];
                        v0 = fmaxf(v0, floor_v); v1 = fmaxf(v1, floor_v); v2 = fmaxf(v2, floor_v); v3 = fmaxf(v3, floor_v);
                        const core::u32x2 pk = {core::pack_bf16x2(v0, v1), core::pack_bf16x2(v2, v3)};
                        *reinterpret_cast<core::u32x2 *>(swr + (((4 * j + g) ^ sswz) << 4)) = pk;
                    }
                // wave-private data and LDS operations of a wave execute in order: only the compiler needs a fence
                __builtin_amdgcn_wave_barrier();
                u32x4 t[4]; // all four reads first: one LDS latency per block instead of four
#pragma unroll
                for (int v = 0; v < 4; ++v) t[v] = *reinterpret_cast<const u32x4 *>(srd[v & 1] + 8 * v * (NT5 * 2));
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row0 = m0 + wm0 + i * 32 + 8 * v; // wave-uniform: first of the 8 rows this instruction stores
                    const u32x4 o = v >= 2 ? u32x4{t[v][2], t[v][3], t[v][0], t[v][1]} : t[v];
                    char *dst = reinterpret_cast<char *>(Cs) + ((size_t)row0 * ldc + n0) * 2 + st_off;
                    if (full) dev::store16<NTS>(dst, o);
                    else if (row0 + (lane >> 3) < M) dev::store16<NTS>(dst, o);
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
        u += run;
    }
}

} // namespace core5
} // namespace tt
