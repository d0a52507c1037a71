// Convolution shard products as implicit GEMMs on the MFMA tile engine (gemm_core.h).
//
// Stride-1 cross-correlation with zero padding (the textbook definition; arXiv 1805.04170 Sec. 4.5 only says which
// dimensions of the 4-D tensors are cut).  Layouts: activations NHWC, filters [K][R][S][C]; per shard the channel
// counts are the shard's own (Cs input channels, Ks output channels), the batch is the shard's Ns images.
//
//   forward   Y[(n,p,q)][ko]   = sum_{(r,s,c)}  X[n, p+r-pad, q+s-pad, c] * W[ko][(r,s,c)]
//             GEMM M = Ns*P*Q, N = Ks, K = R*S*Cs;  A gathered (K contiguous along c), B dense rows of W
//   dgrad     dX[(n,h,w)][c]   = sum_{(r,s,ko)} dY[n, h+pad-r, w+pad-s, ko] * W[ko][r][s][c]
//             GEMM M = Ns*H*W, N = Cs, K = R*S*Ks;  A gathered from dY, B = filters read as [(r,s,ko)][c] (c contiguous)
//   wgrad     dW[ko][(r,s,c)]  = sum_{(n,p,q)}  dY[(n,p,q)][ko] * X[n, p+r-pad, q+s-pad, c]
//             GEMM M = Ks, N = R*S*Cs, K = Ns*P*Q;  A = dY transposed (dense), B gathered from X (c contiguous)
// No im2col buffer is ever materialised: the gather happens while operand tiles are staged into LDS.
#include <cstdint>
#include <cstdlib>
#include "tt_device.h"
#include "gemm_core.h"
#include "gemm_core2.h"
#include "tt_internal.h"
#include "launch_util.h"

namespace tt {
namespace {

using core::and_mask;
using core::kThreads;
using core::kXcds;
using core::u32x4;

struct ConvGeom {
    int32_t Ns, H, W, P, Q, R, S, pad;
    int32_t Cs, Ks; // channels per shard: input, output
};

struct ConvParams {
    const void *A[kMaxShards];
    const void *B[kMaxShards];
    void *C[kMaxShards];
    ConvGeom g;
    int32_t M, N, K, ldc;
    int32_t tiles_m, tiles_n, per_xcd, total, relu;
    // Fused shards (forward kernel only): members > 1 means one product covers `members` shards that share the left
    // operand; its N columns are those shards' column blocks side by side, member_cols (a multiple of 64) each, B is
    // their filter blocks lying one after the other in memory, and the result columns of member m of group g go to
    // C[g * members + m], a matrix of member_cols columns.
    int32_t members, member_cols;
};

__device__ __forceinline__ u32x4 load16(const char *base, int32_t elem_off)
{
    return *reinterpret_cast<const u32x4 *>(base + (ptrdiff_t)elem_off * 2);
}

// A operand of forward and dgrad: rows are output pixels (n, oy, ox), k = (tap, channel) with the channel contiguous.
// in_y = oy + off + sgn * r, in_x = ox + off + sgn * s   (forward: off = -pad, sgn = +1; dgrad: off = +pad, sgn = -1)
template <int SLOTS, bool ONE_TAP> struct GatherKC {
    static constexpr bool KC = true;
    static constexpr bool kFence = false;
    const char *base;
    int IH, IW, OH, OW, R, S, off, sgn, Ch; // Ch: channels per pixel of the source
    int rows, K;
    int32_t pix[SLOTS];   // element offset of source pixel (n, oy + off, ox + off), may be negative
    uint32_t taps[SLOTS]; // bit t set: tap t reads inside the image
    // per K tile, when a tile lies inside one tap (Ch a multiple of the tile depth): the tap and the offset of the
    // tile's first channel relative to pix[]
    int tile_k0, tile_tap;
    int32_t tile_delta;
    __device__ __forceinline__ void init(int slot, int row)
    {
        row = row < rows ? row : rows - 1;
        const int n = row / (OH * OW), rem = row - n * (OH * OW);
        const int oy = rem / OW, ox = rem - oy * OW;
        pix[slot] = ((n * IH + oy + off) * IW + ox + off) * Ch;
        uint32_t m = 0;
        for (int r = 0; r < R; ++r)
            for (int s = 0; s < S; ++s) {
                const int iy = oy + off + sgn * r, ix = ox + off + sgn * s;
                if (iy >= 0 && iy < IH && ix >= 0 && ix < IW) m |= 1u << (r * S + s);
            }
        taps[slot] = m;
    }
    __device__ __forceinline__ void begin_tile(int k0)
    {
        tile_k0 = k0;
        const int kk = k0 < K ? k0 : 0;
        tile_tap = kk / Ch;
        const int r = tile_tap / S, s = tile_tap - r * S;
        tile_delta = sgn * (r * IW + s) * Ch + (kk - tile_tap * Ch);
    }
    __device__ __forceinline__ u32x4 load_masked(int slot, int k) const
    {
        if constexpr (ONE_TAP) { // a K tile never straddles two taps (Ch is a multiple of the tile depth)
            const bool ok = k < K && ((taps[slot] >> tile_tap) & 1u);
            return and_mask(load16(base, ok ? pix[slot] + tile_delta + (k - tile_k0) : 0), ok);
        }
        const int tap = k / Ch, c = k - tap * Ch;
        const int r = tap / S, s = tap - r * S;
        const bool ok = k < K && ((taps[slot] >> tap) & 1u);
        const int32_t o = pix[slot] + sgn * (r * IW + s) * Ch + c;
        return and_mask(load16(base, ok ? o : 0), ok);
    }
    __device__ __forceinline__ u32x4 load(int slot, int k) const { return load_masked(slot, k); }
};

// B operand of dgrad: filters [Ks][R][S][Cs] read as rows c (contiguous), k = (tap, ko)
template <int SLOTS> struct FilterRC {
    static constexpr bool KC = false;
    static constexpr bool kFence = false;
    const char *base;
    int RS, Cs, Ks, rows, K;
    int32_t c0[SLOTS];
    __device__ __forceinline__ void init(int slot, int row) { c0[slot] = row < rows ? row : rows - 8; }
    __device__ __forceinline__ void begin_tile(int) {}
    template <bool KMASK> __device__ __forceinline__ void load4(int slot, int k, u32x4 *out) const
    {
        // four consecutive k: one division, then step (ko wraps into the next tap)
        const int kf = k < K ? k : K - 1;
        int tap = kf / Ks, ko = kf - tap * Ks;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool ok = k + q < K;
            out[q] = and_mask(load16(base, (ko * RS + tap) * Cs + c0[slot]), ok);
            if (k + q + 1 < K) { ++ko; if (ko == Ks) { ko = 0; ++tap; } }
        }
    }
};

// B operand of wgrad: rows are (tap, c) with c contiguous, k = (n, p, q) walks the output pixels
template <int SLOTS> struct GatherRC {
    static constexpr bool KC = false;
    static constexpr bool kFence = false;
    const char *base;
    int H, W, P, Q, S, pad, Cs, rows, K;
    int32_t dy[SLOTS], dx[SLOTS], c0[SLOTS];
    __device__ __forceinline__ void init(int slot, int row)
    {
        row = row < rows ? row : rows - 8;
        const int tap = row / Cs;
        c0[slot] = row - tap * Cs;
        const int r = tap / S;
        dy[slot] = r - pad;
        dx[slot] = tap - r * S - pad;
    }
    __device__ __forceinline__ void begin_tile(int) {}
    template <bool KMASK> __device__ __forceinline__ void load4(int slot, int k, u32x4 *out) const
    {
        const int kf = k < K ? k : K - 1;
        int n = kf / (P * Q);
        const int rem = kf - n * (P * Q);
        int p = rem / Q, q = rem - p * Q;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int iy = p + dy[slot], ix = q + dx[slot];
            const bool ok = k + j < K && iy >= 0 && iy < H && ix >= 0 && ix < W;
            const int32_t o = ((n * H + iy) * W + ix) * Cs + c0[slot];
            out[j] = and_mask(load16(base, ok ? o : 0), ok);
            if (++q == Q) { q = 0; if (++p == P) { p = 0; ++n; } }
        }
    }
};

struct TileId { int shard, m0, n0; };
template <int BM, int BN> __device__ __forceinline__ bool tile_of(const ConvParams &p, TileId *t)
{
    const int logical = core::logical_block(p.per_xcd, p.total);
    if (logical < 0) return false;
    const int tiles = p.tiles_m * p.tiles_n;
    t->shard = logical / tiles;
    const int r = logical - t->shard * tiles;
    // consecutive workgroups walk the N tiles of one M tile: they share the gathered A rows in L2
    t->n0 = (r % p.tiles_n) * BN;
    t->m0 = (r / p.tiles_n) * BM;
    return true;
}

// OP 0: forward, 1: dgrad
template <int BM, int BN, int WN, int DEPTH, bool KMASK, int OP, bool OUT_BF16, bool ONE_TAP, int WM = 2>
__global__ __launch_bounds__(WM * WN * 64, WM * WN / 4) void conv_gather_a_kernel(const ConvParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    TileId t;
    if (!tile_of<BM, BN>(p, &t)) return;
    const ConvGeom &g = p.g;
    constexpr int NT = WM * WN * 64;
    GatherKC<core::Slots<BM, true, NT>::value, ONE_TAP> la;
    la.base = reinterpret_cast<const char *>(p.A[t.shard]);
    la.R = g.R; la.S = g.S;
    la.rows = p.M; la.K = p.K;
    if (OP == 0) { la.IH = g.H; la.IW = g.W; la.OH = g.P; la.OW = g.Q; la.off = -g.pad; la.sgn = 1; la.Ch = g.Cs; }
    else         { la.IH = g.P; la.IW = g.Q; la.OH = g.H; la.OW = g.W; la.off = g.pad;  la.sgn = -1; la.Ch = g.Ks; }
    if constexpr (OP == 0) {
        core::DenseKC<core::Slots<BN, true, NT>::value> lb;
        lb.base = reinterpret_cast<const char *>(p.B[t.shard * p.members]);
        lb.ld = p.K; lb.rows = p.N; lb.K = p.K;
        // every wave owns 64 columns of the tile, which lie in one member's block: the wave writes through that member's
        // pointer, moved back by the block's first column so that the tile's own column numbers address it
        static_assert(BN / WN == 64, "a wave's columns lie in one member block");
        void *Cw = p.C[t.shard];
        int ldc = p.ldc;
        if (p.members > 1) {
            const int col0 = t.n0 + ((threadIdx.x >> 6) % WN) * 64;
            int m = col0 / p.member_cols;
            m = m < p.members ? m : p.members - 1; // columns past N are never stored
            Cw = reinterpret_cast<char *>(p.C[t.shard * p.members + m]) - (ptrdiff_t)m * p.member_cols * (OUT_BF16 ? 2 : 4);
            ldc = p.member_cols;
        }
        core::tile_product<BM, BN, WM, WN, DEPTH, KMASK, OUT_BF16, true>(la, lb, Cw, ldc, p.M, p.N, p.K, t.m0, t.n0, p.relu != 0, smem);
    } else {
        FilterRC<core::Slots<BN, false, NT>::value> lb;
        lb.base = reinterpret_cast<const char *>(p.B[t.shard]);
        lb.RS = g.R * g.S; lb.Cs = g.Cs; lb.Ks = g.Ks; lb.rows = p.N; lb.K = p.K;
        core::tile_product<BM, BN, WM, WN, DEPTH, KMASK, OUT_BF16, true>(la, lb, p.C[t.shard], p.ldc, p.M, p.N, p.K, t.m0, t.n0, p.relu != 0, smem);
    }
}

template <int BM, int BN, int WN, int DEPTH, bool KMASK, bool OUT_BF16>
__global__ __launch_bounds__(WN * 128, WN / 2) void conv_wgrad_kernel(const ConvParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    TileId t;
    if (!tile_of<BM, BN>(p, &t)) return;
    const ConvGeom &g = p.g;
    constexpr int NT = WN * 128;
    core::DenseRC<core::Slots<BM, false, NT>::value> la; // dY shard [(n,p,q)][ko]: rows ko contiguous
    la.base = reinterpret_cast<const char *>(p.A[t.shard]);
    la.ld = g.Ks; la.rows = p.M; la.K = p.K;
    GatherRC<core::Slots<BN, false, NT>::value> lb;
    lb.base = reinterpret_cast<const char *>(p.B[t.shard]);
    lb.H = g.H; lb.W = g.W; lb.P = g.P; lb.Q = g.Q; lb.S = g.S; lb.pad = g.pad; lb.Cs = g.Cs; lb.rows = p.N; lb.K = p.K;
    core::tile_product<BM, BN, 2, WN, DEPTH, KMASK, OUT_BF16, true>(la, lb, p.C[t.shard], p.ldc, p.M, p.N, p.K, t.m0, t.n0, false, smem);
}

// ---- weight gradient with the reduction over pixels re-cut evenly --------------------------------------------------
// The shards that an F3 cut makes add up into the same filter block (Sec. 4.2.1, third aligned form), so the pixels of
// all of them form ONE reduction range per output block, and how that range is cut into partial sums is free: the
// reduction kernel adds whatever partial sums it is given.  Cutting it into `parts` equal runs of 64-pixel K tiles
// (a run may start in one shard and end in the next) makes the number of equal work items a free choice, so a launch
// can fill the chip in whole rounds where the 2^k3 natural partial sums would leave it a ragged last round.
struct SplitGeom {
    int32_t parts;  // partial sums per output block
    int32_t nred;   // shards per output block (2^k3)
    int32_t ktps;   // K tiles (64 pixels) per shard
    uint8_t red_ids[kMaxShards]; // id bits (at the F3 cuts) of the q-th shard of a block
    uint8_t blk_ids[kMaxShards]; // id bits (at the F1 / F2 cuts) of block b
};
struct WgradSplitParams {
    ConvParams c; // A, B: by shard id; C: partial sum number blk * parts + part
    SplitGeom sp;
};

// where K tile g of a block's reduction range lies: its shard's buffer and the pixel it starts at inside that shard.
// A work item touches at most kSegs consecutive shards (the launcher sees to that); their base addresses are read from
// the kernel arguments once, so that no table lookup sits between the K tiles' loads.
constexpr int kSegs = 4;
struct Segment {
    const char *b[kSegs];
    int q0, ktps, g0;
    __device__ __forceinline__ void bind(const void *const *tab, const uint8_t *red_ids, int blk_bits, int nred, int ktps_, int g0_)
    {
        ktps = ktps_;
        g0 = g0_;
        q0 = g0 / ktps;
#pragma unroll
        for (int j = 0; j < kSegs; ++j) {
            const int q = q0 + j < nred ? q0 + j : nred - 1;
            b[j] = reinterpret_cast<const char *>(tab[blk_bits | red_ids[q]]);
        }
    }
    __device__ __forceinline__ const char *locate(int k0, int *kshift) const
    {
        const int g = g0 + k0 / core::BK, q = g / ktps;
        *kshift = (g - q * ktps) * core::BK - k0;
        const int j = q - q0;
        return j == 0 ? b[0] : (j == 1 ? b[1] : (j == 2 ? b[2] : b[3]));
    }
};

// dY rows (output channels contiguous) over the segmented pixel range; k counts from the start of the work item
template <int SLOTS> struct SegDenseRC {
    static constexpr bool KC = false;
    static constexpr bool kFence = false;
    Segment seg;
    const char *base;
    int kshift;
    int ld, rows, K;
    uint32_t off[SLOTS];
    __device__ __forceinline__ void init(int slot, int row) { off[slot] = (uint32_t)(row < rows ? row : rows - 8) * 2u; }
    __device__ __forceinline__ void begin_tile(int k0) { base = seg.locate(k0, &kshift); }
    template <bool KMASK> __device__ __forceinline__ void load4(int slot, int k, u32x4 *out) const
    {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            out[q] = *reinterpret_cast<const u32x4 *>(base + (size_t)(off[slot] + (uint32_t)(k + kshift + q) * (uint32_t)ld * 2u));
    }
};

// the gathered X rows of GatherRC over the segmented pixel range
template <int SLOTS> struct SegGatherRC {
    static constexpr bool KC = false;
    static constexpr bool kFence = false;
    Segment seg;
    const char *base;
    int kshift;
    int H, W, P, Q, S, pad, Cs, rows, K;
    int32_t dy[SLOTS], dx[SLOTS], c0[SLOTS];
    __device__ __forceinline__ void init(int slot, int row)
    {
        row = row < rows ? row : rows - 8;
        const int tap = row / Cs;
        c0[slot] = row - tap * Cs;
        const int r = tap / S;
        dy[slot] = r - pad;
        dx[slot] = tap - r * S - pad;
    }
    __device__ __forceinline__ void begin_tile(int k0) { base = seg.locate(k0, &kshift); }
    template <bool KMASK> __device__ __forceinline__ void load4(int slot, int k, u32x4 *out) const
    {
        const int kl = k + kshift; // pixel inside the shard; the four pixels lie in one K tile, so in one shard
        int n = kl / (P * Q);
        const int rem = kl - n * (P * Q);
        int p = rem / Q, q = rem - p * Q;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int iy = p + dy[slot], ix = q + dx[slot];
            const bool ok = iy >= 0 && iy < H && ix >= 0 && ix < W;
            const int32_t o = ((n * H + iy) * W + ix) * Cs + c0[slot];
            out[j] = and_mask(load16(base, ok ? o : 0), ok);
            if (++q == Q) { q = 0; if (++p == P) { p = 0; ++n; } }
        }
    }
};

template <int BM, int BN, int WN, int DEPTH>
__global__ __launch_bounds__(WN * 128, WN / 2) void conv_wgrad_split_kernel(const WgradSplitParams w)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    const ConvParams &p = w.c;
    const int logical = core::logical_block(p.per_xcd, p.total);
    if (logical < 0) return;
    // items that share a pixel run are neighbours: they read the same dY and X rows through one L2
    const int tiles = p.tiles_m * p.tiles_n;
    const int bp = logical / tiles, r = logical - bp * tiles;
    const int blk = bp / w.sp.parts, part = bp - blk * w.sp.parts;
    const int n0 = (r % p.tiles_n) * BN, m0 = (r / p.tiles_n) * BM;
    const int G = w.sp.nred * w.sp.ktps;
    const int g0 = (int)((int64_t)part * G / w.sp.parts), g1 = (int)((int64_t)(part + 1) * G / w.sp.parts);
    const int K = (g1 - g0) * core::BK; // at least one K tile: the launcher keeps parts <= G
    const ConvGeom &g = p.g;
    constexpr int NT = WN * 128;
    SegDenseRC<core::Slots<BM, false, NT>::value> la;
    la.seg.bind(w.c.A, w.sp.red_ids, w.sp.blk_ids[blk], w.sp.nred, w.sp.ktps, g0);
    la.ld = g.Ks; la.rows = p.M; la.K = K;
    SegGatherRC<core::Slots<BN, false, NT>::value> lb;
    lb.seg.bind(w.c.B, w.sp.red_ids, w.sp.blk_ids[blk], w.sp.nred, w.sp.ktps, g0);
    lb.H = g.H; lb.W = g.W; lb.P = g.P; lb.Q = g.Q; lb.S = g.S; lb.pad = g.pad; lb.Cs = g.Cs; lb.rows = p.N; lb.K = K;
    core::tile_product<BM, BN, 2, WN, DEPTH, false, false, true>(la, lb, p.C[bp], p.ldc, p.M, p.N, K, m0, n0, false, smem);
}

// The same product on the engine that loads tiles straight into LDS (gemm_core2.h): both operands are stored with the
// pixels as the slow dimension, so their tiles go into LDS as they lie in memory and the fragments come out through LDS
// transpose reads; no register transposes and no LDS store instructions.  256 x 256 tiles, eight waves, one workgroup per CU.
struct SegDenseRC2 {
    static constexpr bool KC = false;
    Segment seg;
    int ld, rows;
    template <int ROWS> __device__ __forceinline__ void issue(int row0, int k0, char *lds) const
    {
        static_assert(ROWS == 256, "tile side");
        int kshift;
        const char *base = seg.locate(k0, &kshift);
        const int tid = threadIdx.x, wave = tid >> 6;
        const int kr = tid >> 5, pc = tid & 31; // chunk tid + 512 i: k-row kr + 16 i, position pc (see core2::issue_tile)
        int r0 = row0 + ((pc ^ ((kr & 3) << 1)) << 3);
        r0 = r0 < rows ? r0 : rows - 8; // rows past the end only feed C rows that are never stored
        const char *a = base + ((size_t)(k0 + kshift + kr) * (size_t)ld + (size_t)r0) * 2;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            core2::load_chunk_to_lds(a + (size_t)i * 16 * (size_t)ld * 2, lds + (size_t)(wave * 64 + i * core2::kThreads2) * 16);
    }
};

struct PixelStep { int dn, dp, dq; }; // a run of pixels as whole images, whole rows and columns

struct SegGatherRC2 {
    static constexpr bool KC = false;
    Segment seg;
    int H, W, P, Q, S, pad, Cs, rows, Ns;
    PixelStep s16, s64;
    // position (image, row, column) of this thread's first pixel of the K tile it last issued; the tiles of a work item
    // are issued in order, each 64 pixels after the one before
    mutable int n_, p_, q_;
    __device__ __forceinline__ static void step(const PixelStep &d, int P, int Q, int &n, int &p, int &q)
    {
        q += d.dq;
        const int cq = q >= Q;
        q -= cq ? Q : 0;
        p += d.dp + cq;
        const int cp = p >= P;
        p -= cp ? P : 0;
        n += d.dn + cp;
    }
    template <int ROWS> __device__ __forceinline__ void issue(int row0, int k0, char *lds) const
    {
        static_assert(ROWS == 256, "tile side");
        int kshift;
        const char *base = seg.locate(k0, &kshift);
        const int tid = threadIdx.x, wave = tid >> 6;
        const int kr = tid >> 5, pc = tid & 31;
        int r0 = row0 + ((pc ^ ((kr & 3) << 1)) << 3);
        r0 = r0 < rows ? r0 : rows - 8;
        const int tap = r0 / Cs, c0 = r0 - tap * Cs;
        const int fr = tap / S, dy = fr - pad, dx = tap - fr * S - pad;
        if (k0 == 0) {
            const int kl = kshift + kr; // pixel inside the shard
            n_ = kl / (P * Q);
            const int rem = kl - n_ * (P * Q);
            p_ = rem / Q;
            q_ = rem - p_ * Q;
        } else {
            step(s64, P, Q, n_, p_, q_);
            n_ -= n_ >= Ns ? Ns : 0; // the run went on into the next shard
        }
        int n = n_, p = p_, q = q_;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int iy = p + dy, ix = q + dx;
            const bool ok = iy >= 0 && iy < H && ix >= 0 && ix < W;
            const char *a = base + ((size_t)((n * H + iy) * W + ix) * (size_t)Cs + (size_t)c0) * 2;
            core2::load_chunk_to_lds(ok ? (const void *)a : (const void *)core2::g_zero_chunk,
                                     lds + (size_t)(wave * 64 + i * core2::kThreads2) * 16);
            step(s16, P, Q, n, p, q);
        }
    }
};

__device__ __forceinline__ PixelStep pixel_step(int d, int P, int Q)
{
    PixelStep s;
    s.dn = d / (P * Q);
    const int rem = d - s.dn * (P * Q);
    s.dp = rem / Q;
    s.dq = rem - s.dp * Q;
    return s;
}

__global__ __launch_bounds__(core2::kThreads2, 2) void conv_wgrad_split2_kernel(const WgradSplitParams w)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    const ConvParams &p = w.c;
    const int logical = core::logical_block(p.per_xcd, p.total);
    if (logical < 0) return;
    const int tiles = p.tiles_m * p.tiles_n;
    const int bp = logical / tiles, r = logical - bp * tiles;
    const int blk = bp / w.sp.parts, part = bp - blk * w.sp.parts;
    const int n0 = (r % p.tiles_n) * 256, m0 = (r / p.tiles_n) * 256;
    const int G = w.sp.nred * w.sp.ktps;
    const int g0 = (int)((int64_t)part * G / w.sp.parts), g1 = (int)((int64_t)(part + 1) * G / w.sp.parts);
    const int K = (g1 - g0) * core::BK;
    const ConvGeom &g = p.g;
    SegDenseRC2 la;
    la.seg.bind(w.c.A, w.sp.red_ids, w.sp.blk_ids[blk], w.sp.nred, w.sp.ktps, g0);
    la.ld = g.Ks; la.rows = p.M;
    SegGatherRC2 lb;
    lb.seg.bind(w.c.B, w.sp.red_ids, w.sp.blk_ids[blk], w.sp.nred, w.sp.ktps, g0);
    lb.H = g.H; lb.W = g.W; lb.P = g.P; lb.Q = g.Q; lb.S = g.S; lb.pad = g.pad; lb.Cs = g.Cs; lb.rows = p.N; lb.Ns = g.Ns;
    lb.s16 = pixel_step(16, g.P, g.Q);
    lb.s64 = pixel_step(64, g.P, g.Q);
    lb.n_ = lb.p_ = lb.q_ = 0;
    core2::tile_product2<false, true>(la, lb, p.C[bp], p.ldc, p.M, p.N, K, m0, n0, false, reinterpret_cast<char *>(smem));
}

// Filters [Ks][R][S][Cs] -> [Cs][R][S][Ks] with the taps reversed: with these the gradient w.r.t. the input IS a forward
// convolution of dY (padding R - 1 - pad), so it runs on the forward kernel, whose two operands are both K-contiguous
// (the dedicated kernel has to transpose the filters in registers on their way to LDS and measured 25 % slower).
struct FlipParams {
    const void *src[kMaxShards];
    void *dst[kMaxShards];
    int32_t Ks, RS, Cs;
};
__global__ __launch_bounds__(256) void filter_flip_kernel(const FlipParams p)
{
    const int shard = blockIdx.y;
    const int idx = blockIdx.x * 256 + threadIdx.x; // (ko block of 8, tap, c), c fastest: the 2-byte reads coalesce over c
    const int total = p.Cs * p.RS * (p.Ks / 8);
    if (idx >= total) return;
    const int c = idx % p.Cs, rest = idx / p.Cs;
    const int t = rest % p.RS, kb = rest / p.RS;
    const uint16_t *src = reinterpret_cast<const uint16_t *>(p.src[shard]);
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t lo = src[((size_t)(kb * 8 + 2 * j) * p.RS + (p.RS - 1 - t)) * p.Cs + c];
        const uint32_t hi = src[((size_t)(kb * 8 + 2 * j + 1) * p.RS + (p.RS - 1 - t)) * p.Cs + c];
        w[j] = lo | (hi << 16);
    }
    const u32x4 o = {w[0], w[1], w[2], w[3]};
    *reinterpret_cast<u32x4 *>(reinterpret_cast<uint16_t *>(p.dst[shard]) + ((size_t)c * p.RS + t) * p.Ks + kb * 8) = o;
}

// the same for channel counts that are multiples of 64: a workgroup turns one 64 (ko) x 64 (c) block of one tap around in
// LDS, so both the reads (128 contiguous bytes of c) and the writes (128 contiguous bytes of ko) coalesce
__global__ __launch_bounds__(256) void filter_flip_tiled_kernel(const FlipParams p)
{
    __shared__ uint16_t tile[64][64 + 8];
    const int shard = blockIdx.y;
    const int cb_n = p.Cs / 64, kb_n = p.Ks / 64;
    int b = blockIdx.x;
    const int cb = b % cb_n; b /= cb_n;
    const int kb = b % kb_n;
    const int t = b / kb_n;
    const uint16_t *src = reinterpret_cast<const uint16_t *>(p.src[shard]);
    uint16_t *dst = reinterpret_cast<uint16_t *>(p.dst[shard]);
    const int tid = threadIdx.x, row = tid >> 3, cv = (tid & 7) * 8; // 32 rows x 8 vectors per pass
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int ko = kb * 64 + row + 32 * h;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(src + ((size_t)ko * p.RS + (p.RS - 1 - t)) * p.Cs + cb * 64 + cv);
        *reinterpret_cast<u32x4 *>(&tile[row + 32 * h][cv]) = v;
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int c = row + 32 * h; // output row: channel c of the block, 8 consecutive ko per lane
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = (uint32_t)tile[cv + 2 * j][c] | ((uint32_t)tile[cv + 2 * j + 1][c] << 16);
        const u32x4 o = {w[0], w[1], w[2], w[3]};
        *reinterpret_cast<u32x4 *>(dst + ((size_t)(cb * 64 + c) * p.RS + t) * p.Ks + kb * 64 + cv) = o;
    }
}

// ---- fp32 convolutions: the definition, one output element per thread, fp32 fused multiply-adds in a fixed order
// (taps outermost, channels or pixels innermost).  No tensor-core path exists for fp32 operands here; these kernels are
// bound by plain arithmetic and serve small layers (the fp32 workload of the benchmark is a fully-connected stack).
struct ConvF32Params {
    const float *A[kMaxShards];
    const float *B[kMaxShards];
    void *C[kMaxShards];
    ConvGeom g;
    int32_t relu, out_bf16;
    uint32_t per_shard; // output elements per shard
};

__device__ __forceinline__ void store_out(void *C, size_t i, float v, bool relu, bool out_bf16)
{
    if (relu) v = fmaxf(v, 0.0f);
    if (out_bf16) reinterpret_cast<uint16_t *>(C)[i] = (uint16_t)core::f32_to_bf16_bits(v);
    else reinterpret_cast<float *>(C)[i] = v;
}

// OP 0: Y[(n,p,q)][ko] from X and W;  1: dX[(n,h,w)][c] from dY and W;  2: dW[ko][(r,s,c)] from dY and X
template <int OP> __global__ __launch_bounds__(256) void conv_f32_kernel(const ConvF32Params p)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= p.per_shard) return;
    const int shard = blockIdx.y;
    const ConvGeom &g = p.g;
    const float *A = p.A[shard], *B = p.B[shard];
    float acc = 0.0f;
    if (OP == 0) {
        const int ko = i % g.Ks, pix = i / g.Ks;
        const int n = pix / (g.P * g.Q), rem = pix - n * (g.P * g.Q), oy = rem / g.Q, ox = rem - oy * g.Q;
        for (int r = 0; r < g.R; ++r)
            for (int s = 0; s < g.S; ++s) {
                const int iy = oy + r - g.pad, ix = ox + s - g.pad;
                if (iy < 0 || iy >= g.H || ix < 0 || ix >= g.W) continue;
                const float *x = A + ((size_t)(n * g.H + iy) * g.W + ix) * g.Cs;
                const float *w = B + ((size_t)(ko * g.R + r) * g.S + s) * g.Cs;
                for (int c = 0; c < g.Cs; ++c) acc = fmaf(x[c], w[c], acc);
            }
    } else if (OP == 1) {
        const int c = i % g.Cs, pix = i / g.Cs;
        const int n = pix / (g.H * g.W), rem = pix - n * (g.H * g.W), h = rem / g.W, w_ = rem - h * g.W;
        for (int r = 0; r < g.R; ++r)
            for (int s = 0; s < g.S; ++s) {
                const int oy = h + g.pad - r, ox = w_ + g.pad - s;
                if (oy < 0 || oy >= g.P || ox < 0 || ox >= g.Q) continue;
                const float *dy = A + ((size_t)(n * g.P + oy) * g.Q + ox) * g.Ks;
                for (int ko = 0; ko < g.Ks; ++ko) acc = fmaf(dy[ko], B[((size_t)(ko * g.R + r) * g.S + s) * g.Cs + c], acc);
            }
    } else {
        const int c = i % g.Cs, rest = i / g.Cs;
        const int s = rest % g.S, rest2 = rest / g.S, r = rest2 % g.R, ko = rest2 / g.R;
        for (int n = 0; n < g.Ns; ++n)
            for (int oy = 0; oy < g.P; ++oy) {
                const int iy = oy + r - g.pad;
                if (iy < 0 || iy >= g.H) continue;
                for (int ox = 0; ox < g.Q; ++ox) {
                    const int ix = ox + s - g.pad;
                    if (ix < 0 || ix >= g.W) continue;
                    acc = fmaf(A[((size_t)(n * g.P + oy) * g.Q + ox) * g.Ks + ko], B[((size_t)(n * g.H + iy) * g.W + ix) * g.Cs + c], acc);
                }
            }
    }
    store_out(p.C[shard], i, acc, p.relu != 0, p.out_bf16 != 0);
}

template <typename Kern> tt_status launch(Kern kern, size_t smem, ConvParams &p, int BM, int BN, int threads, int count, hipStream_t s)
{
    if (ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem) != TT_OK) return TT_EDEVICE;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    const int64_t total = (int64_t)p.tiles_m * p.tiles_n * count;
    if (total >= (int64_t(1) << 30)) return TT_EUNSUPPORTED;
    p.total = (int32_t)total;
    p.per_xcd = (int32_t)((total + kXcds - 1) / kXcds);
    hipLaunchKernelGGL(kern, dim3((uint32_t)p.per_xcd * kXcds), dim3(threads), smem, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

// Tile choice as for the dense products: 256 x 256 with eight waves when the launch has enough tiles, else 256 x 128
// or 128 x 128 with four waves.  TT_CONV_TILE=0|1|2 overrides (tuning aid).
int conv_tile(int64_t M, int64_t N, int count)
{
    const int forced = tuning_int("TT_CONV_TILE", -1);
    if (forced >= 0 && forced <= 2) return forced;
    const int64_t big = ((M + 255) / 256) * ((N + 255) / 256) * count;
    if (M > 128 && N > 128 && big >= 128) return 2;
    return M > 128 ? 0 : 1;
}

template <int OP, bool OUT_BF16, bool ONE_TAP> tt_status launch_gather_a_t(ConvParams &p, int count, hipStream_t s)
{
    const bool kmask = p.K % core::BK != 0;
    const int tile = conv_tile(p.M, p.N, count);
    // at most 64 output columns per shard (channels cut eight ways): 256 x 64 tiles, four waves of 64 x 64, so that no
    // wave multiplies columns that do not exist
    if constexpr (OP == 0) // (the filter loader of the direct data-gradient path needs 128 columns for its 256 threads)
    if (p.N <= 64 && p.M > 128 && tuning_int("TT_CONV_TILE", -1) < 0) {
        constexpr size_t sm = core::smem_bytes<256, 64, 2>();
        return kmask ? launch(conv_gather_a_kernel<256, 64, 1, 2, true, OP, OUT_BF16, ONE_TAP, 4>, sm, p, 256, 64, 256, count, s)
                     : launch(conv_gather_a_kernel<256, 64, 1, 2, false, OP, OUT_BF16, ONE_TAP, 4>, sm, p, 256, 64, 256, count, s);
    }
    if (tile == 2) {
        constexpr size_t sm = core::smem_bytes<256, 256>();
        return kmask ? launch(conv_gather_a_kernel<256, 256, 4, 1, true, OP, OUT_BF16, ONE_TAP>, sm, p, 256, 256, 512, count, s)
                     : launch(conv_gather_a_kernel<256, 256, 4, 1, false, OP, OUT_BF16, ONE_TAP>, sm, p, 256, 256, 512, count, s);
    }
    if (tile == 0) {
        constexpr size_t sm = core::smem_bytes<256, 128>();
        return kmask ? launch(conv_gather_a_kernel<256, 128, 2, 2, true, OP, OUT_BF16, ONE_TAP>, sm, p, 256, 128, 256, count, s)
                     : launch(conv_gather_a_kernel<256, 128, 2, 2, false, OP, OUT_BF16, ONE_TAP>, sm, p, 256, 128, 256, count, s);
    }
    constexpr size_t sm = core::smem_bytes<128, 128>();
    return kmask ? launch(conv_gather_a_kernel<128, 128, 2, 1, true, OP, OUT_BF16, ONE_TAP>, sm, p, 128, 128, 256, count, s)
                 : launch(conv_gather_a_kernel<128, 128, 2, 1, false, OP, OUT_BF16, ONE_TAP>, sm, p, 128, 128, 256, count, s);
}

template <int OP, bool OUT_BF16> tt_status launch_gather_a(ConvParams &p, int count, hipStream_t s)
{
    const int ch = OP == 0 ? p.g.Cs : p.g.Ks; // channels per pixel of the gathered tensor
    return ch % core::BK == 0 ? launch_gather_a_t<OP, OUT_BF16, true>(p, count, s)
                              : launch_gather_a_t<OP, OUT_BF16, false>(p, count, s);
}

template <bool OUT_BF16> tt_status launch_wgrad(ConvParams &p, int count, hipStream_t s)
{
    const bool kmask = p.K % core::BK != 0;
    // the pixel-walking gather of the weight gradient measured slower with the eight-wave tile: keep four waves
    int tile = conv_tile(p.M, p.N, count);
    if (tile == 2 && tuning_int("TT_CONV_TILE", -1) < 0) tile = 0;
    if (tile == 2) {
        constexpr size_t sm = core::smem_bytes<256, 256>();
        return kmask ? launch(conv_wgrad_kernel<256, 256, 4, 1, true, OUT_BF16>, sm, p, 256, 256, 512, count, s)
                     : launch(conv_wgrad_kernel<256, 256, 4, 1, false, OUT_BF16>, sm, p, 256, 256, 512, count, s);
    }
    if (tile == 0) {
        constexpr size_t sm = core::smem_bytes<256, 128>();
        return kmask ? launch(conv_wgrad_kernel<256, 128, 2, 2, true, OUT_BF16>, sm, p, 256, 128, 256, count, s)
                     : launch(conv_wgrad_kernel<256, 128, 2, 2, false, OUT_BF16>, sm, p, 256, 128, 256, count, s);
    }
    constexpr size_t sm = core::smem_bytes<128, 128>();
    return kmask ? launch(conv_wgrad_kernel<128, 128, 2, 1, true, OUT_BF16>, sm, p, 128, 128, 256, count, s)
                 : launch(conv_wgrad_kernel<128, 128, 2, 1, false, OUT_BF16>, sm, p, 128, 128, 256, count, s);
}

bool aligned16(const void *const *ptrs, int n)
{
    for (int i = 0; i < n; ++i)
        if (!ptrs[i] || (reinterpret_cast<uintptr_t>(ptrs[i]) & 15)) return false;
    return true;
}

} // namespace

// op: TT_OP_FWD  A = X shards,  B = filter shards, C = Y shards  (Ns*P*Q x Ks)
//     TT_OP_DGRAD A = dY shards, B = filter shards, C = dX shards (Ns*H*W x Cs)
//     TT_OP_WGRAD A = dY shards, B = X shards,      C = dW shards (Ks x R*S*Cs)
// Shard geometry: Ns images, Cs input channels, Ks output channels per shard.
tt_status launch_conv(int op, int count, const void *const *A, const void *const *B, void *const *C, int64_t Ns,
                      int64_t Cs, int64_t Ks, int64_t H, int64_t W, int64_t R, int64_t S, int64_t pad, int out_dtype,
                      int act, void *stream, void *const *flip_ws, int in_dtype)
{
    if (!A || !B || !C || count < 1 || count > kMaxShards) return TT_EINVAL;
    if (Ns <= 0 || Cs <= 0 || Ks <= 0 || H <= 0 || W <= 0 || R <= 0 || S <= 0 || pad < 0) return TT_EINVAL;
    const int64_t P = H + 2 * pad - R + 1, Q = W + 2 * pad - S + 1;
    if (P <= 0 || Q <= 0) return TT_EINVAL;
    if (out_dtype != TT_BF16 && out_dtype != TT_F32) return TT_EINVAL;
    if (in_dtype != TT_BF16 && in_dtype != TT_F32) return TT_EINVAL;
    if (in_dtype == TT_F32) {
        if (op != TT_OP_FWD && op != TT_OP_DGRAD && op != TT_OP_WGRAD) return TT_EINVAL;
        const int64_t lim32 = int64_t(1) << 31;
        if (Ns * H * W * Cs >= lim32 || Ns * P * Q * Ks >= lim32 || Ks * R * S * Cs >= lim32) return TT_EUNSUPPORTED;
        ConvF32Params f;
        for (int i = 0; i < kMaxShards; ++i) {
            if (i < count && (!A[i] || !B[i] || !C[i])) return TT_EINVAL;
            f.A[i] = i < count ? static_cast<const float *>(A[i]) : nullptr;
            f.B[i] = i < count ? static_cast<const float *>(B[i]) : nullptr;
            f.C[i] = i < count ? C[i] : nullptr;
        }
        f.g = ConvGeom{(int32_t)Ns, (int32_t)H, (int32_t)W, (int32_t)P, (int32_t)Q, (int32_t)R, (int32_t)S, (int32_t)pad,
                       (int32_t)Cs, (int32_t)Ks};
        f.relu = act == TT_ACT_RELU;
        f.out_bf16 = out_dtype == TT_BF16;
        const int64_t outs = op == TT_OP_FWD ? Ns * P * Q * Ks : (op == TT_OP_DGRAD ? Ns * H * W * Cs : Ks * R * S * Cs);
        f.per_shard = (uint32_t)outs;
        const int64_t Mg = op == TT_OP_FWD ? Ns * P * Q : (op == TT_OP_DGRAD ? Ns * H * W : Ks);
        const int64_t Ng = op == TT_OP_FWD ? Ks : (op == TT_OP_DGRAD ? Cs : R * S * Cs);
        const int64_t Kg = op == TT_OP_FWD ? R * S * Cs : (op == TT_OP_DGRAD ? R * S * Ks : Ns * P * Q);
        const uint64_t ob32 = out_dtype == TT_BF16 ? 2 : 4;
        const uint64_t xb = (uint64_t)(Ns * H * W * Cs), yb = (uint64_t)(Ns * P * Q * Ks), wb = (uint64_t)(Ks * R * S * Cs);
        const uint64_t bytes32 = op == TT_OP_FWD ? 4 * (xb + wb) + ob32 * yb : (op == TT_OP_DGRAD ? 4 * (yb + wb) + ob32 * xb : 4 * (yb + xb) + ob32 * wb);
        ProfileScope scope(stream, op == TT_OP_FWD ? TT_K_CONV_FWD : (op == TT_OP_DGRAD ? TT_K_CONV_DGRAD : TT_K_CONV_WGRAD), count, Mg,
                           Ng, Kg, bytes32 * (uint64_t)count, 2ull * (uint64_t)Mg * (uint64_t)Ng * (uint64_t)Kg * (uint64_t)count);
        const dim3 grid((uint32_t)((outs + 255) / 256), (uint32_t)count);
        hipStream_t s32 = reinterpret_cast<hipStream_t>(stream);
        if (op == TT_OP_FWD) hipLaunchKernelGGL(conv_f32_kernel<0>, grid, dim3(256), 0, s32, f);
        else if (op == TT_OP_DGRAD) hipLaunchKernelGGL(conv_f32_kernel<1>, grid, dim3(256), 0, s32, f);
        else hipLaunchKernelGGL(conv_f32_kernel<2>, grid, dim3(256), 0, s32, f);
        return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
    }
    // the MFMA engine moves 16-byte vectors along channels and keeps offsets in 32 bits
    if (Cs % 8 || Ks % 8 || R * S > 32) return TT_EUNSUPPORTED;
    const int64_t lim = int64_t(1) << 30;
    if (Ns * H * W * Cs >= lim || Ns * P * Q * Ks >= lim || Ks * R * S * Cs >= lim) return TT_EUNSUPPORTED;
    if (!aligned16(A, count) || !aligned16(B, count) || !aligned16(const_cast<const void *const *>(C), count)) return TT_EUNSUPPORTED;

    ConvParams p;
    for (int i = 0; i < kMaxShards; ++i) {
        p.A[i] = i < count ? A[i] : nullptr;
        p.B[i] = i < count ? B[i] : nullptr;
        p.C[i] = i < count ? C[i] : nullptr;
    }
    p.g = ConvGeom{(int32_t)Ns, (int32_t)H, (int32_t)W, (int32_t)P, (int32_t)Q, (int32_t)R, (int32_t)S, (int32_t)pad,
                   (int32_t)Cs, (int32_t)Ks};
    p.relu = act == TT_ACT_RELU;
    p.members = 1;
    p.member_cols = 0;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const bool obf = out_dtype == TT_BF16;
    const uint64_t ob = obf ? 2 : 4;
    int64_t M, N, K;
    int kclass;
    if (op == TT_OP_FWD) { M = Ns * P * Q; N = Ks; K = R * S * Cs; kclass = TT_K_CONV_FWD; }
    else if (op == TT_OP_DGRAD) { M = Ns * H * W; N = Cs; K = R * S * Ks; kclass = TT_K_CONV_DGRAD; }
    else if (op == TT_OP_WGRAD) { M = Ks; N = R * S * Cs; K = Ns * P * Q; kclass = TT_K_CONV_WGRAD; }
    else return TT_EINVAL;
    if (K < 8) return TT_EUNSUPPORTED;
    p.M = (int32_t)M; p.N = (int32_t)N; p.K = (int32_t)K; p.ldc = (int32_t)N;
    // algorithmic bytes: each tensor of the shard touched once
    const uint64_t x_b = (uint64_t)(Ns * H * W * Cs) * 2, y_b = (uint64_t)(Ns * P * Q * Ks), w_b = (uint64_t)(Ks * R * S * Cs);
    const uint64_t bytes = op == TT_OP_FWD ? x_b + w_b * 2 + y_b * ob
                         : op == TT_OP_DGRAD ? y_b * 2 + w_b * 2 + (uint64_t)(Ns * H * W * Cs) * ob
                                             : y_b * 2 + x_b + w_b * ob;
    ProfileScope scope(stream, kclass, count, M, N, K, bytes * (uint64_t)count,
                       2ull * (uint64_t)M * (uint64_t)N * (uint64_t)K * (uint64_t)count);
    if (op == TT_OP_FWD) return obf ? launch_gather_a<0, true>(p, count, s) : launch_gather_a<0, false>(p, count, s);
    if (op == TT_OP_DGRAD && flip_ws && R == S && pad <= R - 1 && !tuning_int("TT_CONV_DGRAD_DIRECT", 0)) {
        // as a forward convolution of dY (P x Q images, Ks channels) with the flipped filters, padding R - 1 - pad;
        // M, N, K of the implicit GEMM are the same
        FlipParams f;
        for (int i = 0; i < kMaxShards; ++i) {
            if (i < count && (!flip_ws[i] || (reinterpret_cast<uintptr_t>(flip_ws[i]) & 15))) return TT_EINVAL;
            f.src[i] = i < count ? B[i] : nullptr;
            f.dst[i] = i < count ? flip_ws[i] : nullptr;
            p.B[i] = i < count ? flip_ws[i] : nullptr;
        }
        f.Ks = (int32_t)Ks; f.RS = (int32_t)(R * S); f.Cs = (int32_t)Cs;
        if (Cs % 64 == 0 && Ks % 64 == 0) {
            hipLaunchKernelGGL(filter_flip_tiled_kernel, dim3((uint32_t)((Cs / 64) * (Ks / 64) * R * S), (uint32_t)count), dim3(256), 0, s, f);
        } else {
            const int64_t threads = Cs * R * S * (Ks / 8);
            hipLaunchKernelGGL(filter_flip_kernel, dim3((uint32_t)((threads + 255) / 256), (uint32_t)count), dim3(256), 0, s, f);
        }
        if (hipGetLastError() != hipSuccess) return TT_EDEVICE;
        p.g = ConvGeom{(int32_t)Ns, (int32_t)P, (int32_t)Q, (int32_t)H, (int32_t)W, (int32_t)R, (int32_t)S,
                       (int32_t)(R - 1 - pad), (int32_t)Ks, (int32_t)Cs};
        return obf ? launch_gather_a<0, true>(p, count, s) : launch_gather_a<0, false>(p, count, s);
    }
    if (op == TT_OP_DGRAD) return obf ? launch_gather_a<1, true>(p, count, s) : launch_gather_a<1, false>(p, count, s);
    return obf ? launch_wgrad<true>(p, count, s) : launch_wgrad<false>(p, count, s);
}


// Weight-gradient products of all output blocks with each block's pixel range cut into `parts` partial sums (see
// SplitGeom).  A, B: dY and X shards by shard id (2^k entries); C: nblk * parts fp32 buffers of Ks x (R*S*Cs), buffer
// blk * parts + part.  blk_ids / red_ids: id bits of block b / of a block's q-th shard.  Ns images per shard; the pixels
// of a shard must be a multiple of 64 (TT_EUNSUPPORTED otherwise: the caller takes the per-shard path).
tt_status launch_conv_wgrad_split(int k, int nblk, int nred, const uint8_t *blk_ids, const uint8_t *red_ids, int parts,
                                  const void *const *A, const void *const *B, void *const *C, int64_t Ns, int64_t Cs,
                                  int64_t Ks, int64_t H, int64_t W, int64_t R, int64_t S, int64_t pad, int engine,
                                  void *stream)
{
    if (engine != 1 && engine != 2) return TT_EINVAL;
    if (!A || !B || !C || !blk_ids || !red_ids || !valid_k(k) || nblk < 1 || nred < 1 || nblk * nred != (1 << k)) return TT_EINVAL;
    if (parts < 1 || nblk * parts > kMaxShards) return TT_EINVAL;
    if (Ns <= 0 || Cs <= 0 || Ks <= 0 || H <= 0 || W <= 0 || R <= 0 || S <= 0 || pad < 0) return TT_EINVAL;
    const int64_t P = H + 2 * pad - R + 1, Q = W + 2 * pad - S + 1;
    if (P <= 0 || Q <= 0) return TT_EINVAL;
    if (Cs % 8 || Ks % 8 || R * S > 32 || Ks <= 128) return TT_EUNSUPPORTED;
    const int64_t lim = int64_t(1) << 30, pixels = Ns * P * Q;
    if (Ns * H * W * Cs >= lim || pixels * Ks >= lim || Ks * R * S * Cs >= lim) return TT_EUNSUPPORTED;
    if (pixels % core::BK || (int64_t)nred * (pixels / core::BK) < parts) return TT_EUNSUPPORTED;
    {
        // shards one work item can touch: its K tiles, rounded up to whole shards, plus one for a start inside a shard
        const int64_t ktps = pixels / core::BK, len = (nred * ktps + parts - 1) / parts;
        if ((len + ktps - 1) / ktps + 1 > kSegs && nred > kSegs) return TT_EUNSUPPORTED;
    }
    const int n = 1 << k;
    if (!aligned16(A, n) || !aligned16(B, n) || !aligned16(const_cast<const void *const *>(C), nblk * parts)) return TT_EUNSUPPORTED;

    WgradSplitParams w;
    ConvParams &p = w.c;
    for (int i = 0; i < kMaxShards; ++i) {
        p.A[i] = i < n ? A[i] : nullptr;
        p.B[i] = i < n ? B[i] : nullptr;
        p.C[i] = i < nblk * parts ? C[i] : nullptr;
        w.sp.red_ids[i] = i < nred ? red_ids[i] : 0;
        w.sp.blk_ids[i] = i < nblk ? blk_ids[i] : 0;
        if ((i < nred && red_ids[i] >= n) || (i < nblk && blk_ids[i] >= n)) return TT_EINVAL;
    }
    p.g = ConvGeom{(int32_t)Ns, (int32_t)H, (int32_t)W, (int32_t)P, (int32_t)Q, (int32_t)R, (int32_t)S, (int32_t)pad,
                   (int32_t)Cs, (int32_t)Ks};
    p.relu = 0;
    p.members = 1;
    p.member_cols = 0;
    p.M = (int32_t)Ks; p.N = (int32_t)(R * S * Cs); p.K = (int32_t)pixels; p.ldc = p.N;
    w.sp.parts = parts; w.sp.nred = nred; w.sp.ktps = (int32_t)(pixels / core::BK);
    const uint64_t x_b = (uint64_t)(Ns * H * W * Cs) * 2, y_b = (uint64_t)(pixels * Ks) * 2, w_b = (uint64_t)(Ks * R * S * Cs) * 4;
    ProfileScope scope(stream, TT_K_CONV_WGRAD, n, p.M, p.N, p.K, (x_b + y_b) * (uint64_t)n + w_b * (uint64_t)(nblk * parts),
                       2ull * (uint64_t)p.M * (uint64_t)p.N * (uint64_t)p.K * (uint64_t)n);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    // engine 1: register-staged, 256 x 128 tiles, four waves, two workgroups per CU (the tile the per-shard weight
    // gradient uses); engine 2: straight into LDS, 256 x 256 tiles, eight waves, one workgroup per CU
    p.tiles_m = (p.M + 255) / 256;
    p.tiles_n = (p.N + (engine == 2 ? 255 : 127)) / (engine == 2 ? 256 : 128);
    const int64_t total = (int64_t)p.tiles_m * p.tiles_n * nblk * parts;
    if (total >= (int64_t(1) << 30)) return TT_EUNSUPPORTED;
    p.total = (int32_t)total;
    p.per_xcd = (int32_t)((total + kXcds - 1) / kXcds);
    if (engine == 2) {
        auto kern = conv_wgrad_split2_kernel;
        if (ensure_dynamic_lds(reinterpret_cast<const void *>(kern), core2::kSmemBytes) != TT_OK) return TT_EDEVICE;
        hipLaunchKernelGGL(kern, dim3((uint32_t)p.per_xcd * kXcds), dim3(core2::kThreads2), core2::kSmemBytes, s, w);
    } else {
        auto kern = conv_wgrad_split_kernel<256, 128, 2, 2>;
        constexpr size_t sm = core::smem_bytes<256, 128>();
        if (ensure_dynamic_lds(reinterpret_cast<const void *>(kern), sm) != TT_OK) return TT_EDEVICE;
        hipLaunchKernelGGL(kern, dim3((uint32_t)p.per_xcd * kXcds), dim3(256), sm, s, w);
    }
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}


// Forward products (op TT_OP_FWD), or data gradients run as forward products of dY with flipped filters (op TT_OP_DGRAD),
// of `groups` groups of `members` shards each that share their left operand (X resp. dY replicated over the cuts that split
// the output channels resp. the input channels): one product per group with all members' columns side by side, so that a
// group reads its left operand once instead of once per member (with 64 columns per shard the per-shard products take in
// four times the bytes per flop of a 256-wide tile).
//   A[g]: the group's left operand (Ns images);  B[g * members + m]: member m's filter block;  C[g * members + m]: its result
//   cols: columns per member (output channels for FWD, input channels for DGRAD), a multiple of 64;  red: channels of the
//   contraction per pixel (input channels for FWD, output channels for DGRAD).
//   flip_ws (DGRAD): per member a scratch buffer of its filter block's size.
// The members' filter blocks (FWD) resp. scratch buffers (DGRAD) must lie one after the other in memory; if they do not,
// or a shape does not fit, TT_EUNSUPPORTED: the caller runs the members one by one.
tt_status launch_conv_fused(int op, int groups, int members, const void *const *A, const void *const *B, void *const *C,
                            int64_t Ns, int64_t cols, int64_t red, int64_t H, int64_t W, int64_t R, int64_t S, int64_t pad,
                            int out_dtype, int act, void *stream, void *const *flip_ws)
{
    if (!A || !B || !C || groups < 1 || members < 2 || groups * members > kMaxShards) return TT_EINVAL;
    if (op != TT_OP_FWD && op != TT_OP_DGRAD) return TT_EINVAL;
    if (Ns <= 0 || cols <= 0 || red <= 0 || H <= 0 || W <= 0 || R <= 0 || S <= 0 || pad < 0) return TT_EINVAL;
    const int64_t P = H + 2 * pad - R + 1, Q = W + 2 * pad - S + 1;
    if (P <= 0 || Q <= 0) return TT_EINVAL;
    if (out_dtype != TT_BF16 && out_dtype != TT_F32) return TT_EINVAL;
    if (op == TT_OP_DGRAD && (!flip_ws || R != S || pad > R - 1)) return TT_EUNSUPPORTED;
    if (cols % 64 || red % 8 || R * S > 32) return TT_EUNSUPPORTED;
    const int n = groups * members;
    const int64_t N = cols * members, K = R * S * red, lim = int64_t(1) << 30;
    const int64_t in_px = op == TT_OP_FWD ? H * W : P * Q, out_px = op == TT_OP_FWD ? P * Q : H * W; // per image
    if (Ns * in_px * red >= lim || Ns * out_px * N >= lim || N * K >= lim) return TT_EUNSUPPORTED;
    if (!aligned16(A, groups) || !aligned16(B, n) || !aligned16(const_cast<const void *const *>(C), n)) return TT_EUNSUPPORTED;
    const void *const *blocks = op == TT_OP_FWD ? B : const_cast<const void *const *>(flip_ws);
    const size_t block_bytes = (size_t)cols * (size_t)K * 2;
    for (int g = 0; g < groups; ++g)
        for (int m = 0; m < members; ++m) {
            const void *b = blocks[g * members + m];
            if (!b || (reinterpret_cast<uintptr_t>(b) & 15)) return op == TT_OP_FWD ? TT_EUNSUPPORTED : TT_EINVAL;
            if (m > 0 && static_cast<const char *>(b) != static_cast<const char *>(blocks[g * members]) + (size_t)m * block_bytes)
                return TT_EUNSUPPORTED;
        }
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const bool obf = out_dtype == TT_BF16;
    const int64_t M = Ns * out_px;
    const uint64_t ob = obf ? 2 : 4;
    // algorithmic bytes as the per-shard launches count them: each shard's tensors touched once
    const uint64_t bytes = ((uint64_t)(Ns * in_px * red) * 2 + (uint64_t)(cols * K) * 2 + (uint64_t)(M * cols) * ob) * (uint64_t)n;
    ProfileScope scope(stream, op == TT_OP_FWD ? TT_K_CONV_FWD : TT_K_CONV_DGRAD, n, M, cols, K, bytes,
                       2ull * (uint64_t)M * (uint64_t)cols * (uint64_t)K * (uint64_t)n);
    ConvParams p;
    for (int i = 0; i < kMaxShards; ++i) {
        p.A[i] = i < groups ? A[i] : nullptr;
        p.B[i] = i < n ? blocks[i] : nullptr;
        p.C[i] = i < n ? C[i] : nullptr;
    }
    if (op == TT_OP_DGRAD) {
        // member m's filters [red][R][S][cols] -> [cols][R][S][red] with the taps reversed, into its scratch buffer
        FlipParams f;
        for (int i = 0; i < kMaxShards; ++i) {
            f.src[i] = i < n ? B[i] : nullptr;
            f.dst[i] = i < n ? flip_ws[i] : nullptr;
        }
        f.Ks = (int32_t)red; f.RS = (int32_t)(R * S); f.Cs = (int32_t)cols;
        if (red % 64 == 0) {
            hipLaunchKernelGGL(filter_flip_tiled_kernel, dim3((uint32_t)((cols / 64) * (red / 64) * R * S), (uint32_t)n), dim3(256), 0, s, f);
        } else {
            const int64_t threads = cols * R * S * (red / 8);
            hipLaunchKernelGGL(filter_flip_kernel, dim3((uint32_t)((threads + 255) / 256), (uint32_t)n), dim3(256), 0, s, f);
        }
        if (hipGetLastError() != hipSuccess) return TT_EDEVICE;
        p.g = ConvGeom{(int32_t)Ns, (int32_t)P, (int32_t)Q, (int32_t)H, (int32_t)W, (int32_t)R, (int32_t)S,
                       (int32_t)(R - 1 - pad), (int32_t)red, (int32_t)N};
    } else {
        p.g = ConvGeom{(int32_t)Ns, (int32_t)H, (int32_t)W, (int32_t)P, (int32_t)Q, (int32_t)R, (int32_t)S, (int32_t)pad,
                       (int32_t)red, (int32_t)N};
    }
    p.relu = act == TT_ACT_RELU;
    p.members = members;
    p.member_cols = (int32_t)cols;
    p.M = (int32_t)M; p.N = (int32_t)N; p.K = (int32_t)K; p.ldc = (int32_t)N;
    return obf ? launch_gather_a<0, true>(p, groups, s) : launch_gather_a<0, false>(p, groups, s);
}

} // namespace tt
