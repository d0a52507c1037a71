// Third bf16 MFMA tile engine: a persistent, software-pipelined version of the direct-to-LDS engine (gemm_core2.h).
//
// One workgroup of eight waves stays on its CU and walks a list of 256 x 256 output tiles.  The K tiles (BK = 32 or 64
// deep) of ALL its output tiles form one stream of work items; operand tiles are fetched global -> LDS
// (global_load_lds_dwordx4) NS - 1 items ahead through a ring of NS LDS stages, so the first K tiles of the next output
// tile are already on their way while the current one is finished and written out.  Nothing waits for memory except
// the one s_waitcnt + barrier at the top of each item.
//
// Ring shape: two stages of 64 measured best on MI355X.  Thinner, deeper rings (BK = 32, four or five stages, up to two
// steps of lookahead) were slower on every workload: the skinny batch-256 products are not waiting for misses, they are
// bound by the global -> LDS path itself (each CU has to take in a tile of the shared small operand next to every tile
// of the streamed one; about 10 TB/s over the chip), and the compute-bound products lose more to the extra barriers
// than they gain in lookahead.
//
// LDS layouts and fragment reads follow gemm_core2.h (for BK = 32 a K-contiguous row is 64 bytes and the swizzle is
// chunk ^ ((row >> 2) & 3)).  Further differences:
//   - the loads are inline assembly with a scalar base and a 32-bit lane offset, computed once per output tile
//     (the builtin form makes the compiler put s_waitcnt vmcnt(0) in front of every fragment read);
//   - K must be a multiple of 64 (no tail handling in the K direction; the launcher falls back otherwise);
//   - results go through a small wave-private LDS area that lies outside the ring (bf16: 16 rows at a time, fp32
//     partial sums: 8), so the epilogue needs no workgroup barrier and never touches a stage that a prefetch may be
//     filling, and leave as 16-byte vectors of whole row segments; rows that cannot take 16-byte stores are stored
//     element by element straight from the accumulators.
#pragma once
#include <cstdint>
#include "tt_device.h"
#include "gemm_core.h"
#include "gemm_core2.h"

namespace tt {
namespace core3 {

using core::bf16x8;
using core::f32x16;
using core::u32x4;
using core2::s16x4;

constexpr int kThreads3 = 512;
constexpr int BM3 = 256, BN3 = 256;

template <int BK> constexpr int op_stage_bytes() { return 256 * BK * 2; }           // one operand, one stage
template <int BK> constexpr int loads_per_op() { return 256 * BK * 2 / 16 / kThreads3; } // 16-byte chunks per thread

constexpr int kEpiRows = 16, kEpiLd = 64 + 8;         // bf16 staging strip of one wave: 16 rows x 64 columns, padded
constexpr int kEpiBytes = 8 * kEpiRows * kEpiLd * 2;  // 18 KB for the eight waves
// fp32 staging strip of one wave: 8 rows x 64 columns, padded (fits in the bf16 strip's place)
constexpr int kEpiRowsF = 8, kEpiLdF = 64 + 4;
static_assert(kEpiRowsF * kEpiLdF * 4 <= kEpiRows * kEpiLd * 2, "the fp32 strip fits where the bf16 strip lies");

// Write-out of a wave's 128 x 64 fp32 accumulator tile (4 x 2 blocks of 32 x 32; a lane holds column lane % 32 and rows
// 8 g + 4 (lane / 32) + e % 4, g = e / 4, of each block) through a wave-private strip of kEpiRowsF x kEpiLdF floats: eight
// rows at a time are turned round in LDS and leave as 16-byte vectors, 16 lanes per 256-byte row segment, four rows per
// store instruction (stored straight from the accumulators a row segment takes 32 four-byte stores of a half wave: four
// times the store instructions, and measured 15-30 % slower on the products that write large fp32 partial sums).
// N must be a multiple of 4 and C 16-byte aligned.  (row0, col0): the wave tile's origin in C.
__device__ __forceinline__ void store_wave_tile_f32(f32x16 (&acc)[4][2], float *strip, float *C, int ldc, int row0, int col0, int M,
                                                    int N, bool relu, int lane)
{
    const int col_l = lane & 31, row_l = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int ee = 0; ee < 4; ++ee) {
                    float v = acc[i][j][4 * g + ee];
                    if (relu) v = fmaxf(v, 0.0f);
                    strip[(row_l + ee) * kEpiLdF + j * 32 + col_l] = v;
                }
            // wave-private data and LDS operations of a wave execute in order: only the compiler needs a fence
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                const int idx = lane + 64 * v, lrow = idx >> 4, vc = (idx & 15) * 4;
                const int row = row0 + i * 32 + 8 * g + lrow, col = col0 + vc;
                const core::f32x4 o = *reinterpret_cast<const core::f32x4 *>(strip + lrow * kEpiLdF + vc);
                if (row < M && col < N) // N is a multiple of 4 on this path: a vector is all in or all out
                    __builtin_nontemporal_store(o, reinterpret_cast<core::f32x4 *>(C + (size_t)row * ldc + col));
            }
            __builtin_amdgcn_wave_barrier();
        }
}

template <int BK, int NS, bool STAGED> constexpr size_t smem_bytes3()
{
    return (size_t)NS * 2 * op_stage_bytes<BK>() + (STAGED ? kEpiBytes : 0);
}

struct Params3 {
    const void *A[64];
    const void *B[64];
    void *C[64];
    int32_t M, N, K;
    int32_t lda, ldb, ldc;
    int32_t tiles_m, tiles_n;
    int32_t per_xcd;     // logical output tiles per XCD
    int32_t wg_per_xcd;  // resident workgroups per XCD (grid = 8 * wg_per_xcd)
    int32_t total;       // tiles_m * tiles_n * count * ksplit
    int32_t relu;
    int32_t ksplit, kchunk;
};

// position of one output tile
struct TilePos {
    int vshard, shard, m0, n0, kbeg, klen;
};

// j-th output tile of this workgroup; false when the list is exhausted
__device__ __forceinline__ bool tile_of(const Params3 &p, int j, TilePos *t)
{
    const int bid = blockIdx.x;
    const int li = bid / core::kXcds + j * p.wg_per_xcd;
    const int logical = (bid % core::kXcds) * p.per_xcd + li;
    if (li >= p.per_xcd || logical >= p.total) return false;
    const int tiles = p.tiles_m * p.tiles_n;
    t->vshard = logical / tiles;
    const int r = logical - t->vshard * tiles;
    int tm, tn;
    core::grouped_tile(r, p.tiles_m, p.tiles_n, &tm, &tn);
    t->m0 = tm * BM3;
    t->n0 = tn * BN3;
    t->shard = t->vshard / p.ksplit;
    t->kbeg = (t->vshard - t->shard * p.ksplit) * p.kchunk;
    t->klen = p.K - t->kbeg < p.kchunk ? p.K - t->kbeg : p.kchunk;
    return true;
}

// Stream of operand tiles of one operand over the whole work list of the workgroup.
//   KC = true : operand rows (m for A, n for B) have K contiguous (leading dimension ld = K extent of the matrix)
//   KC = false: K rows of the matrix are contiguous over the operand's rows (ld = row extent)
template <int BK, bool KC, bool IS_A> struct Feeder {
    static constexpr int NL = loads_per_op<BK>();
    uint32_t voff[NL];  // lane part of the address of this thread's chunks
    const char *base;   // wave-uniform part: start of the current K tile
    uint32_t kstep;     // bytes from one K tile to the next
    int kt, nk, j;      // K tile inside the output tile, their number, ordinal of the output tile
    bool live;

    __device__ __forceinline__ void bind(const Params3 &p, const TilePos &t)
    {
        const int tid = threadIdx.x;
        const void *mat = IS_A ? p.A[t.shard] : p.B[t.shard];
        const int ld = IS_A ? p.lda : p.ldb;
        const int rows = IS_A ? p.M : p.N;
        const int row0 = IS_A ? t.m0 : t.n0;
        if constexpr (KC) {
            // chunk c = tid + 512 i of the tile: row c / (BK/8), position c % (BK/8); the position holds k-chunk
            // position ^ swizzle(row) (see read_frag3)
            constexpr int CPR = BK / 8; // chunks per row
            base = reinterpret_cast<const char *>(mat) + (size_t)t.kbeg * 2;
            kstep = BK * 2;
            const int rl = tid / CPR; // row of chunk i = rl + (512 / CPR) i; the stride is a multiple of 16
            const int kc = (tid % CPR) ^ (CPR == 8 ? (rl >> 1) & 7 : (rl >> 2) & 3);
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                int r = row0 + rl + (kThreads3 / CPR) * i;
                r = r < rows ? r : rows - 1; // rows past the end only feed C rows that are never stored
                voff[i] = (uint32_t)r * (uint32_t)ld * 2u + (uint32_t)kc * 16u;
            }
        } else {
            // chunk c: k-row c / 32, position c % 32 holds row-chunk position ^ ((k & 3) << 1)
            base = reinterpret_cast<const char *>(mat) + (size_t)t.kbeg * (size_t)ld * 2;
            kstep = (uint32_t)BK * (uint32_t)ld * 2u;
            const int rc = (tid & 31) ^ (((tid >> 5) & 3) << 1);
            int r = row0 + rc * 8;
            r = r < rows ? r : rows - 8;
#pragma unroll
            for (int i = 0; i < NL; ++i)
                voff[i] = (uint32_t)((tid >> 5) + 16 * i) * (uint32_t)ld * 2u + (uint32_t)r * 2u;
        }
        kt = 0;
        nk = t.klen / BK;
    }

    __device__ __forceinline__ void start(const Params3 &p)
    {
        TilePos t;
        j = 0;
        live = tile_of(p, 0, &t);
        if (live) bind(p, t);
    }

    // Fetch chunk i (of NL) of the current K tile into the stage at LDS address lds (wave-uniform).
    __device__ __forceinline__ void issue_one(int i, uint32_t lds) const
    {
        const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        // the base is wave-uniform by construction; say so, or the "s" operand may be handed a vector register pair
        // (readfirstlane returns a signed int: go through uint32_t so the low half is not sign-extended)
        const uint64_t b64 = reinterpret_cast<uint64_t>(base);
        const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b64);
        const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b64 >> 32));
        const uint64_t sbase = ((uint64_t)b_hi << 32) | (uint64_t)b_lo;
        const uint32_t dst = lds + (wave * 64u + (uint32_t)i * kThreads3) * 16u;
        dev::lds_dma16(voff[i], sbase, dst);
    }

    // Move on to the next K tile.  Past the end of the list the last K tile stays current and is fetched again (into a
    // stage nobody reads), so every item issues the same number of loads and the wait count of the main loop stays
    // constant.
    __device__ __forceinline__ void advance(const Params3 &p)
    {
        if (!live) return;
        if (kt + 1 < nk) {
            ++kt;
            base += kstep;
            return;
        }
        TilePos t;
        if (tile_of(p, j + 1, &t)) {
            ++j;
            bind(p, t);
        } else {
            live = false; // keep pointing at the last K tile
        }
    }

    __device__ __forceinline__ void issue_and_advance(const Params3 &p, uint32_t lds)
    {
#pragma unroll
        for (int i = 0; i < NL; ++i) issue_one(i, lds);
        advance(p);
    }
};

constexpr int waitcnt_vm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// fragment (32 rows x 16 k) of an operand stage: rows rbase .. rbase+31 of the tile, k-step ks
template <int BK, bool KC> __device__ __forceinline__ bf16x8 read_frag3(const char *lds, int rbase, int ks, int lane)
{
    if constexpr (!KC || BK == 64) {
        return core2::read_frag<256, KC>(lds, rbase, ks, lane);
    } else {
        const int r = rbase + (lane & 31), q = ks * 2 + (lane >> 5);
        return *reinterpret_cast<const bf16x8 *>(lds + r * 64 + ((q ^ ((r >> 2) & 3)) << 4));
    }
}

template <int BK, int NS, bool A_KC, bool B_KC, bool OUT_BF16, bool STAGED, bool ILV>
__device__ __forceinline__ void run_tiles(const Params3 &p, char *smem)
{
    static_assert(NS >= 2 && (BK == 32 || BK == 64), "ring shape");
    constexpr int TM = 4, TN = 2, WN = 4; // 2 x 4 waves, 128 x 64 per wave
    constexpr int D = NS - 1;             // items of lookahead
    constexpr int OPB = op_stage_bytes<BK>(), STB = 2 * OPB;
    // loads that may still be in flight at the top of an item: those of the D - 1 items issued after it
    constexpr int W = (D - 1) * 2 * loads_per_op<BK>();
    static_assert(W <= 63, "vmcnt range");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave / WN) * (TM * 32), wn0 = (wave % WN) * (TN * 32);
    const uint32_t lds0 = dev::lds_addr(smem);

    Feeder<BK, A_KC, true> fa;
    Feeder<BK, B_KC, false> fb;
    fa.start(p);
    fb.start(p);
    TilePos cur;
    int jc = 0;
    if (!tile_of(p, 0, &cur)) return; // no work for this workgroup (uniform)

    int is = 0; // stage the next loads go to
#pragma unroll
    for (int s = 0; s < D; ++s) {
        fa.issue_and_advance(p, lds0 + (uint32_t)is * STB);
        fb.issue_and_advance(p, lds0 + (uint32_t)is * STB + OPB);
        is = is + 1 == NS ? 0 : is + 1;
    }

    int cs = 0; // stage of the item being multiplied
    const bool relu = p.relu != 0;
    const int M = p.M, N = p.N, ldc = p.ldc;
    for (;;) {
        f32x16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

        const int nk = cur.klen / BK;
        for (int kt = 0; kt < nk; ++kt) {
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(W)); // this wave's chunks of the item have landed
            __syncthreads();                           // everyone's have; everyone has finished reading the previous item
            const uint32_t lds_next = lds0 + (uint32_t)is * STB; // item kt + D goes into the stage of the previous item
            is = is + 1 == NS ? 0 : is + 1;
            const char *As = smem + cs * STB, *Bs = As + OPB;
            cs = cs + 1 == NS ? 0 : cs + 1;
            if constexpr (!ILV) {
                fa.issue_and_advance(p, lds_next);
                fb.issue_and_advance(p, lds_next + OPB);
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_iglp_opt(1);
            }
            static_assert(loads_per_op<BK>() == BK / 16, "one chunk of each operand per k-step");
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                if constexpr (ILV) {
                    // Fetch spread over the k-steps of the item: a wave that issues all its loads at once sits in the
                    // issue queue until the memory pipeline has taken them and only then starts to multiply.  Pays for
                    // short K loops (measured: K = 256); for long ones the compiler's own interleaving of fragment
                    // reads and MFMAs (iglp_opt), which the fences here switch off, is worth more.
                    fa.issue_one(ks, lds_next);
                    fb.issue_one(ks, lds_next + OPB);
                    __builtin_amdgcn_sched_barrier(0);
                }
                bf16x8 af[TM], bf[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) af[i] = read_frag3<BK, A_KC>(As, wm0 + i * 32, ks, lane);
#pragma unroll
                for (int j = 0; j < TN; ++j) bf[j] = read_frag3<BK, B_KC>(Bs, wn0 + j * 32, ks, lane);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
                if constexpr (ILV) __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (ILV) {
                fa.advance(p);
                fb.advance(p);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- epilogue.  A lane holds column (lane & 31) and rows 8*(e/4) + 4*(lane/32) + e%4 of each 32 x 32 block.
        // (Measured alternative, not kept: exchanging the MFMA operands gives every lane consecutive columns of one row,
        // so results could leave as 16-byte vectors without LDS; but each store instruction then touches 32 rows with
        // 32 bytes each, and those partial-line writes were slower than the staged row-contiguous ones below.)
        const int col_l = lane & 31, row_l = (lane >> 5) * 4;
        if constexpr (STAGED && !OUT_BF16) {
            float *strip = reinterpret_cast<float *>(smem + NS * STB) + wave * (kEpiRowsF * kEpiLdF);
            store_wave_tile_f32(acc, strip, reinterpret_cast<float *>(p.C[cur.vshard]), ldc, cur.m0 + wm0, cur.n0 + wn0, M, N, relu,
                                lane);
        } else if constexpr (!STAGED) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = cur.n0 + wn0 + j * 32 + col_l;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int row = cur.m0 + wm0 + i * 32 + 8 * (e >> 2) + row_l + (e & 3);
                        float v = acc[i][j][e];
                        if (relu) v = fmaxf(v, 0.0f);
                        if (row < M && col < N) {
                            if constexpr (OUT_BF16)
                                reinterpret_cast<uint16_t *>(p.C[cur.vshard])[(size_t)row * ldc + col] = (uint16_t)core::f32_to_bf16_bits(v);
                            else
                                __builtin_nontemporal_store(v, reinterpret_cast<float *>(p.C[cur.vshard]) + (size_t)row * ldc + col);
                        }
                    }
                }
        } else {
            uint16_t *strip = reinterpret_cast<uint16_t *>(smem + NS * STB) + wave * (kEpiRows * kEpiLd);
            uint16_t *Cs = reinterpret_cast<uint16_t *>(p.C[cur.vshard]);
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
                                uint16_t *d = strip + (8 * eg + row_l + ee) * kEpiLd + j * 32 + col_l;
                                d[0] = (uint16_t)(pk & 0xffffu);
                                d[kEpiLd] = (uint16_t)(pk >> 16);
                            }
                    // Wave-private data: LDS operations of one wave execute in order, so the reads below see the writes above and the
                    // next strip's writes cannot overtake them; no wait is needed, only a fence for the compiler's scheduler.
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int v = 0; v < 2; ++v) {
                        const int idx = lane + 64 * v, lrow = idx >> 3, vc = (idx & 7) * 8;
                        const int row = cur.m0 + wm0 + i * 32 + 16 * h + lrow, col = cur.n0 + wn0 + vc;
                        const u32x4 o = *reinterpret_cast<const u32x4 *>(strip + lrow * kEpiLd + vc);
                        if (row < M && col < N) // N is a multiple of 8 on this path: a vector is all in or all out
                            __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(Cs + (size_t)row * ldc + col));
                    }
                    __builtin_amdgcn_wave_barrier();
                }
        }

        ++jc;
        if (!tile_of(p, jc, &cur)) break;
    }
    // the re-fetches issued past the end of the list must have landed before the workgroup gives up its LDS
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
}

} // namespace core3
} // namespace tt
