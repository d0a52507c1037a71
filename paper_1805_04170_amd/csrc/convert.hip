// Tiling conversion ("retile"), gated conversion and partial-sum reduction kernels.
//
// Sec. 5.2 of arXiv 1805.04170 converts between tilings in three steps (sender slices, receiver fetches,
// receiver concatenates).  With all shards in one HBM the three steps collapse into one gather-copy: by the
// flattening theorem (Sec. 4.4) source and destination tilings are regular grids, so every destination block is a
// grid of equally sized "pieces", each lying inside exactly one source shard.  One launch covers all shards; a
// workgroup's piece coordinates are wave-uniform (scalar) and each lane only moves 16-byte vectors.
//
// These kernels are HBM-bound: coalesced 128-bit accesses, several loads in flight per lane, no LDS.
#include <cstdint>
#include <cstdlib>
#include "tt_device.h"
#include "tt_bf16.h"
#include "launch_util.h"
#include "tt_internal.h"

namespace tt {
namespace {

constexpr int kThreads = 256;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct GridDev {
    uint32_t maskR, maskC, maskX;
    uint32_t kC;      // number of C cuts (to split a block number into row / column block)
    uint32_t srows;   // shard rows
    uint32_t scols_v; // shard columns in vectors (= leading dimension in vectors)
};

struct ConvertParams {
    const void *src[kMaxShards];
    const void *msk[kMaxShards];
    void *dst[kMaxShards];
    uint8_t rep_ids[kMaxShards]; // id bits of the r-th destination replica
    GridDev A, Am, B;
    uint32_t k;
    uint32_t nrep;                 // replicas of every destination block
    uint32_t piece_rows, piece_cv; // piece extent: rows, vectors per row
    uint32_t pieces_c, pieces;     // pieces per destination block: along columns, total
    uint32_t tiles_per_piece;
    uint32_t piece_vecs;           // piece_rows * piece_cv
    uint32_t step_rows, step_cv;   // kThreads vectors expressed as (rows, vectors) of a piece
    uint32_t unroll;
};

__device__ __forceinline__ uint32_t deposit_bits(uint32_t v, uint32_t mask, uint32_t k)
{
    uint32_t out = 0;
    int n = __popc(mask);
    for (int b = (int)k - 1; b >= 0; --b)
        if (mask & (1u << b)) { --n; if ((v >> n) & 1u) out |= 1u << b; }
    return out;
}

struct PieceLoc { uint32_t shard; uint64_t base_v; }; // shard id and vector offset of the piece's first element

__device__ __forceinline__ PieceLoc locate(const GridDev &g, uint32_t k, uint32_t row0, uint32_t col0_v, uint32_t pref)
{
    uint32_t rb = row0 / g.srows, ro = row0 - rb * g.srows;
    uint32_t cb = col0_v / g.scols_v, co = col0_v - cb * g.scols_v;
    PieceLoc p;
    p.shard = deposit_bits(rb, g.maskR, k) | deposit_bits(cb, g.maskC, k) | (pref & g.maskX);
    p.base_v = (uint64_t)ro * g.scols_v + co;
    return p;
}

template <typename V> struct Lanes;
template <> struct Lanes<u32x4> { static constexpr int bytes = 16; };
template <> struct Lanes<u32x2> { static constexpr int bytes = 8; };
template <> struct Lanes<uint32_t> { static constexpr int bytes = 4; };
template <> struct Lanes<uint16_t> { static constexpr int bytes = 2; };
template <> struct Lanes<uint8_t> { static constexpr int bytes = 1; };

__device__ __forceinline__ uint32_t gate_bf16_pair(uint32_t v, uint32_t m)
{
    // keep each 16-bit half of v where the matching bf16 of m is > 0 (positive, non-zero, not NaN)
    uint32_t lo = m & 0xffffu, hi = m >> 16;
    bool klo = lo != 0 && lo <= 0x7f80u;
    bool khi = hi != 0 && hi <= 0x7f80u;
    return (klo ? (v & 0xffffu) : 0u) | (khi ? (v & 0xffff0000u) : 0u);
}
__device__ __forceinline__ uint32_t gate_f32(uint32_t v, uint32_t m) { return __uint_as_float(m) > 0.0f ? v : 0u; }

// GATE: 0 = plain copy, 1 = bf16 gate, 2 = f32 gate
template <int GATE> __device__ __forceinline__ uint32_t gate_word(uint32_t v, uint32_t m)
{
    if (GATE == 1) return gate_bf16_pair(v, m);
    if (GATE == 2) return gate_f32(v, m);
    return v;
}
template <int GATE> __device__ __forceinline__ u32x4 gate(u32x4 v, u32x4 m)
{
    u32x4 o = {gate_word<GATE>(v.x, m.x), gate_word<GATE>(v.y, m.y), gate_word<GATE>(v.z, m.z), gate_word<GATE>(v.w, m.w)};
    return o;
}
template <int GATE> __device__ __forceinline__ u32x2 gate(u32x2 v, u32x2 m)
{
    u32x2 o = {gate_word<GATE>(v.x, m.x), gate_word<GATE>(v.y, m.y)};
    return o;
}
template <int GATE> __device__ __forceinline__ uint32_t gate(uint32_t v, uint32_t m) { return gate_word<GATE>(v, m); }
template <int GATE> __device__ __forceinline__ uint16_t gate(uint16_t v, uint16_t m)
{
    // only reachable for bf16 (a 2-byte vector cannot hold an f32)
    return (m != 0 && m <= 0x7f80u) ? v : (uint16_t)0;
}
template <int GATE> __device__ __forceinline__ uint8_t gate(uint8_t v, uint8_t) { return v; }

template <typename V, int GATE, int U>
__global__ __launch_bounds__(kThreads) void convert_kernel(const ConvertParams p)
{
    // wave-uniform decomposition of the workgroup number
    uint32_t bid = blockIdx.x;
    uint32_t tile = bid % p.tiles_per_piece;
    uint32_t rest = bid / p.tiles_per_piece;
    uint32_t piece = rest % p.pieces;
    uint32_t blk = rest / p.pieces;
    uint32_t pr = piece / p.pieces_c, pc = piece - pr * p.pieces_c;
    uint32_t rbB = blk >> p.B.kC, cbB = blk & ((1u << p.B.kC) - 1u);
    uint32_t row0 = rbB * p.B.srows + pr * p.piece_rows;       // global row of the piece
    uint32_t col0 = cbB * p.B.scols_v + pc * p.piece_cv;       // global column (vectors) of the piece
    uint32_t dst0 = deposit_bits(rbB, p.B.maskR, p.k) | deposit_bits(cbB, p.B.maskC, p.k);

    PieceLoc sa = locate(p.A, p.k, row0, col0, dst0);
    const V *src = reinterpret_cast<const V *>(p.src[sa.shard]) + sa.base_v;
    const V *msk = nullptr;
    uint32_t m_ld = 0;
    if (GATE != 0) {
        PieceLoc sm = locate(p.Am, p.k, row0, col0, dst0);
        msk = reinterpret_cast<const V *>(p.msk[sm.shard]) + sm.base_v;
        m_ld = p.Am.scols_v;
    }
    uint64_t dbase = (uint64_t)(pr * p.piece_rows) * p.B.scols_v + pc * p.piece_cv;

    uint32_t idx = tile * (kThreads * U) + threadIdx.x;
    uint32_t row = idx / p.piece_cv, cv = idx - row * p.piece_cv;

    V val[U];
    uint64_t doff[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        ok[u] = idx < p.piece_vecs;
        doff[u] = dbase + (uint64_t)row * p.B.scols_v + cv;
        // unconditional loads (lanes past the end re-read the piece's first vector and store nothing): loads under a
        // branch would be waited for one by one
        {
            V v = __builtin_nontemporal_load(src + (ok[u] ? (uint64_t)row * p.A.scols_v + cv : 0));
            if (GATE != 0) v = gate<GATE>(v, __builtin_nontemporal_load(msk + (ok[u] ? (uint64_t)row * m_ld + cv : 0)));
            val[u] = v;
        }
        idx += kThreads;
        row += p.step_rows;
        cv += p.step_cv;
        if (cv >= p.piece_cv) { cv -= p.piece_cv; ++row; }
    }
    for (uint32_t r = 0; r < p.nrep; ++r) {
        V *dst = reinterpret_cast<V *>(p.dst[dst0 | p.rep_ids[r]]);
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ok[u]) __builtin_nontemporal_store(val[u], dst + doff[u]);
    }
}

// ------------------------------------------------------------------ reduce

struct ReduceParams {
    const float *part[kMaxShards];
    void *dst[kMaxShards];
    uint8_t rep_ids[kMaxShards]; // destination replica id bits
    uint8_t red_ids[kMaxShards]; // id bits of partial number p
    GridDev Z, B;                // scols_v in units of EV elements
    uint32_t k, nrep, nred;
    uint32_t ksplit; // partial buffers per shard (extra split of the reduction dimension inside a shard)
    uint32_t relu;
    uint32_t piece_rows, piece_cv, pieces_c, pieces, tiles_per_piece, piece_vecs, step_rows, step_cv;
};

template <int EV> struct FVec;
template <> struct FVec<4> { using type = f32x4; };
template <> struct FVec<1> { using type = float; };

// CHUNK partial buffers are read per round with all loads in flight together (a last round may be shorter: the count
// need not be a multiple of CHUNK); lanes past the end of a piece read a clamped in-range address and store nothing.
template <int EV, bool OUT_BF16, int U, int CHUNK>
__global__ __launch_bounds__(kThreads) void reduce_kernel(const ReduceParams p)
{
    using FV = typename FVec<EV>::type;
    uint32_t bid = blockIdx.x;
    uint32_t tile = bid % p.tiles_per_piece;
    uint32_t rest = bid / p.tiles_per_piece;
    uint32_t piece = rest % p.pieces;
    uint32_t blk = rest / p.pieces;
    uint32_t pr = piece / p.pieces_c, pc = piece - pr * p.pieces_c;
    uint32_t rbB = blk >> p.B.kC, cbB = blk & ((1u << p.B.kC) - 1u);
    uint32_t row0 = rbB * p.B.srows + pr * p.piece_rows;
    uint32_t col0 = cbB * p.B.scols_v + pc * p.piece_cv;
    uint32_t dst0 = deposit_bits(rbB, p.B.maskR, p.k) | deposit_bits(cbB, p.B.maskC, p.k);
    PieceLoc sz = locate(p.Z, p.k, row0, col0, 0u);
    uint64_t dbase = (uint64_t)(pr * p.piece_rows) * p.B.scols_v + pc * p.piece_cv;

    uint32_t idx = tile * (kThreads * U) + threadIdx.x;
    uint32_t row = idx / p.piece_cv, cv = idx - row * p.piece_cv;

    float acc[U][EV];
    uint64_t soff[U], doff[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        ok[u] = idx < p.piece_vecs;
        soff[u] = ok[u] ? sz.base_v + (uint64_t)row * p.Z.scols_v + cv : sz.base_v;
        doff[u] = dbase + (uint64_t)row * p.B.scols_v + cv;
#pragma unroll
        for (int e = 0; e < EV; ++e) acc[u][e] = 0.0f;
        idx += kThreads;
        row += p.step_rows;
        cv += p.step_cv;
        if (cv >= p.piece_cv) { cv -= p.piece_cv; ++row; }
    }
    // partial sums are added in increasing partial number: a fixed order, independent of the launch shape
    const uint32_t total = p.nred * p.ksplit;
    for (uint32_t q0 = 0; q0 < total; q0 += CHUNK) {
        FV v[CHUNK][U];
#pragma unroll
        for (int j = 0; j < CHUNK; ++j) {
            const uint32_t qq = q0 + j < total ? q0 + j : total - 1, q = qq / p.ksplit, c = qq - q * p.ksplit;
            const FV *src = reinterpret_cast<const FV *>(p.part[(sz.shard | p.red_ids[q]) * p.ksplit + c]);
#pragma unroll
            for (int u = 0; u < U; ++u) v[j][u] = __builtin_nontemporal_load(src + soff[u]);
        }
#pragma unroll
        for (int j = 0; j < CHUNK; ++j)
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (q0 + j >= total) continue; // short last round (wave-uniform): the re-read buffer is not added again
                if constexpr (EV == 4) {
                    acc[u][0] += v[j][u].x; acc[u][1] += v[j][u].y; acc[u][2] += v[j][u].z; acc[u][3] += v[j][u].w;
                } else {
                    acc[u][0] += v[j][u];
                }
            }
    }
    if (p.relu) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int e = 0; e < EV; ++e) acc[u][e] = fmaxf(acc[u][e], 0.0f);
    }
    for (uint32_t r = 0; r < p.nrep; ++r) {
        void *d = p.dst[dst0 | p.rep_ids[r]];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!ok[u]) continue;
            if constexpr (OUT_BF16) {
                if constexpr (EV == 4) {
                    u32x2 o;
                    o.x = pack_bf16x2(acc[u][0], acc[u][1]);
                    o.y = pack_bf16x2(acc[u][2], acc[u][3]);
                    __builtin_nontemporal_store(o, reinterpret_cast<u32x2 *>(d) + doff[u]);
                } else {
                    reinterpret_cast<uint16_t *>(d)[doff[u]] = (uint16_t)f32_to_bf16_bits(acc[u][0]);
                }
            } else {
                if constexpr (EV == 4) {
                    f32x4 o = {acc[u][0], acc[u][1], acc[u][2], acc[u][3]};
                    __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(d) + doff[u]);
                } else {
                    reinterpret_cast<float *>(d)[doff[u]] = acc[u][0];
                }
            }
        }
    }
}

GridDev to_dev(const Grid &g, int64_t vec_elems)
{
    GridDev d;
    d.maskR = g.maskR; d.maskC = g.maskC; d.maskX = g.maskX;
    d.kC = (uint32_t)g.kC;
    d.srows = (uint32_t)g.srows;
    d.scols_v = (uint32_t)(g.scols / vec_elems);
    return d;
}

bool aligned_all(const void *const *ptrs, int n, size_t a)
{
    for (int i = 0; i < n; ++i)
        if (reinterpret_cast<uintptr_t>(ptrs[i]) % a) return false;
    return true;
}

template <typename V, int GATE> tt_status launch_convert_v(const ConvertParams &p, uint32_t blocks, hipStream_t s)
{
    if (p.unroll == 16) hipLaunchKernelGGL((convert_kernel<V, GATE, 16>), dim3(blocks), dim3(kThreads), 0, s, p);
    else if (p.unroll == 8) hipLaunchKernelGGL((convert_kernel<V, GATE, 8>), dim3(blocks), dim3(kThreads), 0, s, p);
    else if (p.unroll == 4) hipLaunchKernelGGL((convert_kernel<V, GATE, 4>), dim3(blocks), dim3(kThreads), 0, s, p);
    else if (p.unroll == 2) hipLaunchKernelGGL((convert_kernel<V, GATE, 2>), dim3(blocks), dim3(kThreads), 0, s, p);
    else if (p.unroll == 1) hipLaunchKernelGGL((convert_kernel<V, GATE, 1>), dim3(blocks), dim3(kThreads), 0, s, p);
    else return TT_EINVAL; // the grid was sized for p.unroll vectors per lane: no other kernel may run on it
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

template <int GATE> tt_status launch_convert_g(int vbytes, const ConvertParams &p, uint32_t blocks, hipStream_t s)
{
    switch (vbytes) {
    case 16: return launch_convert_v<u32x4, GATE>(p, blocks, s);
    case 8: return launch_convert_v<u32x2, GATE>(p, blocks, s);
    case 4: return launch_convert_v<uint32_t, GATE>(p, blocks, s);
    case 2: return launch_convert_v<uint16_t, GATE>(p, blocks, s);
    default: return launch_convert_v<uint8_t, GATE>(p, blocks, s);
    }
}

} // namespace

// Work per lane: enough vectors in flight to cover HBM latency, but keep >= ~4 workgroups per CU when the tensor
// is small.
static int pick_unroll(uint64_t total_vecs)
{
    // measured on the 205 MB weight: 4 vectors per lane 5.78 TB/s, 8: 5.68, 16: 5.33; on 8 MB activations (512 K
    // vectors) 4 per lane is 30 % faster than 1, on 2 MB ones (128 K vectors) 2 per lane equal to 1 and 4 slower
    if (total_vecs >= (uint64_t)1 << 19) return 4;
    if (total_vecs >= (uint64_t)1 << 17) return 2;
    return 1;
}

tt_status launch_convert(void *const *dst, const uint8_t *Bl, const void *const *src, const uint8_t *Al,
                         const void *const *mask, const uint8_t *Aml, int k, int64_t rows, int64_t cols,
                         int elem_bytes, int gate_dtype, bool dst_unique, void *stream)
{
    if (!dst || !src || !valid_k(k) || rows < 0 || cols < 0) return TT_EINVAL;
    if (rows == 0 || cols == 0) return TT_OK;
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8) return TT_EINVAL;
    if (rows >= (int64_t(1) << 31) || cols * elem_bytes >= (int64_t(1) << 31)) return TT_EUNSUPPORTED;
    Grid A, Am, B;
    if (!make_grid(Al, k, rows, cols, &A) || !make_grid(Bl, k, rows, cols, &B)) return TT_EINFEASIBLE;
    const bool gated = mask != nullptr;
    if (gated && !make_grid(Aml, k, rows, cols, &Am)) return TT_EINFEASIBLE;
    const int n = 1 << k;
    for (int s = 0; s < n; ++s)
        if (!dst[s] || !src[s] || (gated && !mask[s])) return TT_EINVAL;

    int64_t piece_rows = A.srows < B.srows ? A.srows : B.srows;
    int64_t piece_cols = A.scols < B.scols ? A.scols : B.scols;
    if (gated) {
        if (Am.srows < piece_rows) piece_rows = Am.srows;
        if (Am.scols < piece_cols) piece_cols = Am.scols;
    }
    // widest vector that divides every row pitch and keeps every pointer aligned
    int vbytes = 16;
    while (vbytes > elem_bytes &&
           ((piece_cols * elem_bytes) % vbytes || !aligned_all(src, n, vbytes) ||
            !aligned_all(const_cast<const void *const *>(dst), n, vbytes) || (gated && !aligned_all(mask, n, vbytes))))
        vbytes >>= 1;
    const int64_t vec_elems = vbytes / elem_bytes;

    ConvertParams p;
    for (int s = 0; s < kMaxShards; ++s) {
        p.src[s] = s < n ? src[s] : nullptr;
        p.dst[s] = s < n ? dst[s] : nullptr;
        p.msk[s] = (gated && s < n) ? mask[s] : nullptr;
        p.rep_ids[s] = 0;
    }
    p.A = to_dev(A, vec_elems);
    p.B = to_dev(B, vec_elems);
    p.Am = gated ? to_dev(Am, vec_elems) : p.A;
    p.k = (uint32_t)k;
    p.nrep = dst_unique ? 1u : 1u << B.kX; // dst_unique: replicas alias one buffer, write it once
    for (uint32_t r = 0; r < p.nrep; ++r) p.rep_ids[r] = (uint8_t)deposit(r, B.maskX, k);
    const int64_t piece_cv = piece_cols / vec_elems;
    const uint64_t unique_vecs = (uint64_t)rows * (uint64_t)(cols / vec_elems);
    p.unroll = (uint32_t)pick_unroll(unique_vecs);
    if (const int u = tuning_int("TT_CVT_U", 0); u == 1 || u == 2 || u == 4 || u == 8 || u == 16) p.unroll = (uint32_t)u;
    p.piece_rows = (uint32_t)piece_rows;
    p.piece_cv = (uint32_t)piece_cv;
    p.pieces_c = (uint32_t)(B.scols / piece_cols);
    p.pieces = (uint32_t)((B.srows / piece_rows) * (B.scols / piece_cols));
    uint64_t piece_vecs = (uint64_t)piece_rows * (uint64_t)piece_cv;
    if (piece_vecs >= (uint64_t(1) << 31)) return TT_EUNSUPPORTED;
    p.piece_vecs = (uint32_t)piece_vecs;
    const uint32_t per_tile = (uint32_t)kThreads * p.unroll;
    p.tiles_per_piece = (uint32_t)((piece_vecs + per_tile - 1) / per_tile);
    p.step_rows = (uint32_t)(kThreads / piece_cv);
    p.step_cv = (uint32_t)(kThreads % piece_cv);
    uint64_t blocks = (uint64_t)p.tiles_per_piece * p.pieces * (uint64_t(1) << (B.kR + B.kC));
    if (blocks >= (uint64_t(1) << 31)) return TT_EUNSUPPORTED;

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    // algorithmic traffic: every unique block read once (plus the gate source), every destination copy written once
    const uint64_t tensor_bytes = (uint64_t)rows * (uint64_t)cols * (uint64_t)elem_bytes;
    ProfileScope scope(stream, gated ? TT_K_GATE : TT_K_CONVERT, n, rows, cols, elem_bytes,
                       tensor_bytes * ((gated ? 2u : 1u) + p.nrep), 0);
    if (!gated) return launch_convert_g<0>(vbytes, p, (uint32_t)blocks, s);
    if (gate_dtype == TT_BF16) return launch_convert_g<1>(vbytes, p, (uint32_t)blocks, s);
    if (gate_dtype == TT_F32) return launch_convert_g<2>(vbytes, p, (uint32_t)blocks, s);
    return TT_EINVAL;
}

template <int EV, bool OUT_BF16, int U> static tt_status launch_reduce_u(const ReduceParams &p, uint32_t blocks, hipStream_t s)
{
    const uint32_t total = p.nred * p.ksplit;
    if (total >= 8) hipLaunchKernelGGL((reduce_kernel<EV, OUT_BF16, U, 8>), dim3(blocks), dim3(kThreads), 0, s, p);
    else if (total >= 4) hipLaunchKernelGGL((reduce_kernel<EV, OUT_BF16, U, 4>), dim3(blocks), dim3(kThreads), 0, s, p);
    else if (total >= 2) hipLaunchKernelGGL((reduce_kernel<EV, OUT_BF16, U, 2>), dim3(blocks), dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((reduce_kernel<EV, OUT_BF16, U, 1>), dim3(blocks), dim3(kThreads), 0, s, p);
    return hipGetLastError() == hipSuccess ? TT_OK : TT_EDEVICE;
}

template <int EV, bool OUT_BF16> static tt_status launch_reduce_e(const ReduceParams &p, uint32_t blocks, int unroll, hipStream_t s)
{
    // with 8 partials per round in flight one vector per lane already keeps the memory system busy
    if (unroll == 4) return launch_reduce_u<EV, OUT_BF16, 4>(p, blocks, s);
    if (unroll == 2) return launch_reduce_u<EV, OUT_BF16, 2>(p, blocks, s);
    return launch_reduce_u<EV, OUT_BF16, 1>(p, blocks, s);
}

tt_status launch_reduce(void *const *dst, const uint8_t *Bl, int out_dtype, const float *const *partials,
                        const uint8_t *zl, int k, int64_t rows, int64_t cols, int act, int ksplit, void *stream, bool per_block)
{
    // in-shard splits come in powers of two (the launch code that cuts K makes no others); per-block partial sums in any number
    if (ksplit < 1 || (!per_block && (ksplit & (ksplit - 1)) != 0) || (ksplit << k) > kMaxShards) return TT_EINVAL;
    if (!dst || !partials || !valid_k(k) || rows < 0 || cols < 0) return TT_EINVAL;
    if (rows == 0 || cols == 0) return TT_OK;
    if (out_dtype != TT_F32 && out_dtype != TT_BF16) return TT_EINVAL;
    if (act != TT_ACT_NONE && act != TT_ACT_RELU) return TT_EINVAL;
    if (rows >= (int64_t(1) << 31) || cols >= (int64_t(1) << 31)) return TT_EUNSUPPORTED;
    Grid Z, B;
    if (!make_grid(zl, k, rows, cols, &Z) || !make_grid(Bl, k, rows, cols, &B)) return TT_EINFEASIBLE;
    const int n = 1 << k;
    for (int s = 0; s < n; ++s)
        if (!dst[s]) return TT_EINVAL;
    // per_block: only the table entries of shard ids with zero bits at the kRed cuts are used
    for (int s = 0; s < n; ++s)
        for (int c = 0; c < ksplit; ++c)
            if (!(per_block && ((uint32_t)s & Z.maskX)) && !partials[s * ksplit + c]) return TT_EINVAL;
    int64_t piece_rows = Z.srows < B.srows ? Z.srows : B.srows;
    int64_t piece_cols = Z.scols < B.scols ? Z.scols : B.scols;
    const size_t out_b = out_dtype == TT_BF16 ? 2 : 4;
    int ev = 4;
    bool parts_aligned = true;
    for (int s = 0; s < n * ksplit; ++s)
        if (!(per_block && ((uint32_t)(s / ksplit) & Z.maskX)) && reinterpret_cast<uintptr_t>(partials[s]) % 16) parts_aligned = false;
    if (piece_cols % 4 || !parts_aligned ||
        !aligned_all(const_cast<const void *const *>(dst), n, 4 * out_b))
        ev = 1;

    ReduceParams p;
    for (int s = 0; s < kMaxShards; ++s) {
        p.part[s] = (s < n * ksplit && !(per_block && ((uint32_t)(s / ksplit) & Z.maskX))) ? partials[s] : nullptr;
        p.dst[s] = s < n ? dst[s] : nullptr;
        p.rep_ids[s] = 0;
        p.red_ids[s] = 0;
    }
    p.Z = to_dev(Z, ev);
    p.B = to_dev(B, ev);
    p.k = (uint32_t)k;
    p.nrep = 1u << B.kX;
    p.nred = per_block ? 1u : 1u << Z.kX;
    p.ksplit = (uint32_t)ksplit;
    p.relu = act == TT_ACT_RELU;
    for (uint32_t r = 0; r < p.nrep; ++r) p.rep_ids[r] = (uint8_t)deposit(r, B.maskX, k);
    for (uint32_t q = 0; q < p.nred; ++q) p.red_ids[q] = per_block ? 0 : (uint8_t)deposit(q, Z.maskX, k);
    const int64_t piece_cv = piece_cols / ev;
    uint64_t piece_vecs = (uint64_t)piece_rows * (uint64_t)piece_cv;
    if (piece_vecs >= (uint64_t(1) << 31)) return TT_EUNSUPPORTED;
    const uint64_t unique_vecs = (uint64_t)rows * (uint64_t)(cols / ev);
    // Vectors per lane, measured on MI355X (256 x 1000 .. 512 x 8192 outputs, 2 .. 16 partial sums): one below 128 K
    // vectors (more workgroups matter more than loads in flight), two up to a million; above that two for one or two
    // partial sums, four for four (16 loads in flight per lane), one for eight or more (already eight in flight).
    const uint32_t n_part = p.nred * (uint32_t)ksplit;
    int unroll = 1;
    if (unique_vecs >= (uint64_t)1 << 20) unroll = n_part >= 8 ? 1 : (n_part == 4 ? 4 : 2);
    else if (unique_vecs >= (uint64_t)1 << 17) unroll = 2;
    if (const int u = tuning_int("TT_RED_U", 0); u == 1 || u == 2 || u == 4) unroll = u;
    p.piece_rows = (uint32_t)piece_rows;
    p.piece_cv = (uint32_t)piece_cv;
    p.pieces_c = (uint32_t)(B.scols / piece_cols);
    p.pieces = (uint32_t)((B.srows / piece_rows) * (B.scols / piece_cols));
    p.piece_vecs = (uint32_t)piece_vecs;
    const uint32_t per_tile = (uint32_t)(kThreads * unroll);
    p.tiles_per_piece = (uint32_t)((piece_vecs + per_tile - 1) / per_tile);
    p.step_rows = (uint32_t)(kThreads / piece_cv);
    p.step_cv = (uint32_t)(kThreads % piece_cv);
    uint64_t blocks = (uint64_t)p.tiles_per_piece * p.pieces * (uint64_t(1) << (B.kR + B.kC));
    if (blocks >= (uint64_t(1) << 31)) return TT_EUNSUPPORTED;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const uint64_t elems = (uint64_t)rows * (uint64_t)cols;
    ProfileScope scope(stream, TT_K_REDUCE, n, rows, cols, (int64_t)out_b, elems * 4u * p.nred * p.ksplit + elems * out_b * p.nrep, 0);
    if (ev == 4) return out_dtype == TT_BF16 ? launch_reduce_e<4, true>(p, (uint32_t)blocks, unroll, s)
                                              : launch_reduce_e<4, false>(p, (uint32_t)blocks, unroll, s);
    return out_dtype == TT_BF16 ? launch_reduce_e<1, true>(p, (uint32_t)blocks, unroll, s)
                                : launch_reduce_e<1, false>(p, (uint32_t)blocks, unroll, s);
}

} // namespace tt

// ------------------------------------------------------------------- C ABI

extern "C" tt_status tt_retile(void *const *dst, tt_tiling B, const void *const *src, tt_tiling A, int k, int64_t rows,
                               int64_t cols, int elem_bytes, void *stream)
{
    if (!tt::valid_k(k) || !tt::valid_tiling(A, k) || !tt::valid_tiling(B, k)) return TT_EINVAL;
    return tt::launch_convert(dst, B.cut, src, A.cut, nullptr, nullptr, k, rows, cols, elem_bytes, 0, false, stream);
}

extern "C" tt_status tt_retile_gate(void *const *dst, tt_tiling B, const void *const *src, tt_tiling A,
                                    const void *const *mask, tt_tiling Am, int k, int64_t rows, int64_t cols, int dtype,
                                    void *stream)
{
    if (!tt::valid_k(k) || !tt::valid_tiling(A, k) || !tt::valid_tiling(B, k)) return TT_EINVAL;
    if (dtype != TT_F32 && dtype != TT_BF16) return TT_EINVAL;
    if (mask && !tt::valid_tiling(Am, k)) return TT_EINVAL;
    return tt::launch_convert(dst, B.cut, src, A.cut, mask, Am.cut, k, rows, cols, dtype == TT_BF16 ? 2 : 4, dtype, false, stream);
}

extern "C" tt_status tt_reduce(void *const *dst, tt_tiling B, int out_dtype, const float *const *partials,
                               const uint8_t *forms, int k, int64_t rows, int64_t cols, int act, void *stream)
{
    if (!tt::valid_k(k) || !tt::valid_tiling(B, k) || (k > 0 && !forms)) return TT_EINVAL;
    uint8_t zl[TT_MAX_K];
    for (int j = 0; j < k; ++j) {
        if (forms[j] > TT_F3) return TT_EINVAL;
        zl[j] = forms[j] == TT_F1 ? TT_R : (forms[j] == TT_F2 ? TT_C : tt::kRed);
    }
    return tt::launch_reduce(dst, B.cut, out_dtype, partials, zl, k, rows, cols, act, 1, stream);
}
