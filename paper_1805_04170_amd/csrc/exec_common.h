// Host-side machinery shared by the layer execute calls: the three phases of Sec. 4.2.1 / Sec. 5.2 of
// arXiv 1805.04170 (input conversion, shard products, output conversion / reduction) expressed as pointer tables
// over shard buffers plus launches of the conversion, reduction and product kernels.
//
// On one GPU a conversion between two tilings whose blocks have the same shape moves nothing: the aligned operand
// is a re-numbering of the stored shards, so the pointer table is permuted instead of copying (inputs are only
// read).  Likewise replicas of an aligned temporary share one buffer.  Real copies happen only when block shapes
// differ, or when the gradient gate has to be applied.
#pragma once
#include <cstdlib>
#include <cstring>
#include "tt_internal.h"

namespace tt {

// bump allocator over the caller's workspace; in dry mode it only measures
struct Workspace {
    char *base = nullptr;
    size_t cap = 0, used = 0;
    bool dry = false, overflow = false;
    void *take(size_t bytes)
    {
        size_t off = align_up(used, 256);
        used = off + bytes;
        if (dry) return reinterpret_cast<void *>(uintptr_t(0x100000) + off); // never dereferenced
        if (used > cap) { overflow = true; return nullptr; }
        return base + off;
    }
};

// a tensor as 2^k shard pointers under a tiling (entries may alias each other)
struct Sharded {
    const void *ptr[kMaxShards];
    tt_tiling t;
    int64_t rows = 0, cols = 0;
};

inline void set_sharded(Sharded *s, const void *const *ptrs, tt_tiling t, int k, int64_t rows, int64_t cols)
{
    for (int i = 0; i < (1 << k); ++i) s->ptr[i] = ptrs ? ptrs[i] : nullptr; // NULL only in workspace queries
    s->t = t;
    s->rows = rows;
    s->cols = cols;
}

// src (stored) -> aligned tiling a.  mask: optional gate source (same shape); dtype only matters when gating.
inline tt_status prepare_operand(const Sharded &src, const tt_tiling &a, int k, int elem_bytes, const Sharded *mask,
                                 int dtype, Workspace &ws, void *stream, Sharded *out)
{
    Grid gs, ga;
    if (!make_grid(src.t.cut, k, src.rows, src.cols, &gs) || !make_grid(a.cut, k, src.rows, src.cols, &ga)) return TT_EINFEASIBLE;
    const int n = 1 << k;
    out->t = a;
    out->rows = src.rows;
    out->cols = src.cols;
    if (!mask && gs.kR == ga.kR && gs.kC == ga.kC) {
        for (int s = 0; s < n; ++s) {
            uint32_t rb = extract((uint32_t)s, ga.maskR, k), cb = extract((uint32_t)s, ga.maskC, k);
            uint32_t sid = deposit(rb, gs.maskR, k) | deposit(cb, gs.maskC, k) | ((uint32_t)s & gs.maskX);
            out->ptr[s] = src.ptr[sid];
        }
        return TT_OK;
    }
    const int nblk = 1 << (ga.kR + ga.kC);
    const size_t blk_bytes = (size_t)ga.srows * (size_t)ga.scols * (size_t)elem_bytes;
    void *blk[kMaxShards];
    for (int b = 0; b < nblk; ++b) blk[b] = ws.take(blk_bytes);
    if (ws.overflow) return TT_EWORKSPACE;
    void *dst[kMaxShards];
    for (int s = 0; s < n; ++s) {
        uint32_t rb = extract((uint32_t)s, ga.maskR, k), cb = extract((uint32_t)s, ga.maskC, k);
        dst[s] = blk[(rb << ga.kC) | cb];
        out->ptr[s] = dst[s];
    }
    if (ws.dry) return TT_OK;
    return launch_convert(dst, a.cut, src.ptr, src.t.cut, mask ? mask->ptr : nullptr, mask ? mask->t.cut : nullptr, k,
                          src.rows, src.cols, elem_bytes, dtype, /*dst_unique=*/true, stream);
}

// Where the shard products write, and what has to follow.
struct OutputPlan {
    void *gemm_out[kMaxShards];
    int gemm_dtype = TT_F32;
    int gemm_act = TT_ACT_NONE;
    int mode = 0; // 0: products write the stored shards; 1: conversion afterwards; 2: reduction afterwards
    int ksplit = 1; // > 1: each shard product is cut further along K into ksplit partial sums (mode 2)
    uint8_t zl[TT_MAX_K];
};

// zl: the temporary outputs' grid letters per cut (TT_R, TT_C or kRed) in the coordinates of the rows x cols matrix
// ksplit: extra K split inside every shard (see pick_ksplit); forces the reduction path
inline tt_status plan_output_letters(const uint8_t *zl, const tt_tiling &tZ, void *const *Z, int64_t rows, int64_t cols,
                                     int k, int dtype, int act, Workspace &ws, OutputPlan *op, int ksplit = 1)
{
    Grid gz, gt;
    for (int j = 0; j < k; ++j) op->zl[j] = zl[j];
    if (!make_grid(op->zl, k, rows, cols, &gz) || !make_grid(tZ.cut, k, rows, cols, &gt)) return TT_EINFEASIBLE;
    const int n = 1 << k;
    const size_t esz = dtype == TT_BF16 ? 2 : 4;
    op->ksplit = ksplit;
    if (ksplit == 1 && gz.kX == 0 && gt.kX == 0 && gz.kR == gt.kR && gz.kC == gt.kC) {
        op->mode = 0;
        op->gemm_dtype = dtype;
        op->gemm_act = act;
        for (int s = 0; s < n; ++s) {
            uint32_t rb = extract((uint32_t)s, gz.maskR, k), cb = extract((uint32_t)s, gz.maskC, k);
            op->gemm_out[s] = Z ? Z[deposit(rb, gt.maskR, k) | deposit(cb, gt.maskC, k)] : nullptr;
        }
        return TT_OK;
    }
    const bool red = gz.kX > 0 || ksplit > 1;
    if (n * ksplit > kMaxShards) return TT_EINVAL;
    op->mode = red ? 2 : 1;
    op->gemm_dtype = red ? TT_F32 : dtype;
    op->gemm_act = red ? TT_ACT_NONE : act; // the element-wise function comes after the sum
    const size_t bytes = (size_t)gz.srows * (size_t)gz.scols * (red ? 4 : esz);
    for (int s = 0; s < n * ksplit; ++s) op->gemm_out[s] = ws.take(bytes);
    return ws.overflow ? TT_EWORKSPACE : TT_OK;
}

inline tt_status plan_output(const uint8_t *forms, const tt_tiling &tZ, void *const *Z, int64_t rows, int64_t cols, int k,
                             int dtype, int act, Workspace &ws, OutputPlan *op, int ksplit = 1)
{
    uint8_t zl[TT_MAX_K];
    aligned_tilings(forms, k, nullptr, nullptr, zl);
    return plan_output_letters(zl, tZ, Z, rows, cols, k, dtype, act, ws, op, ksplit);
}

// Extra split of the reduction dimension inside every shard product.  Skinny products (few output tiles, long K: the
// batch-256 layers) leave most CUs idle and too few bytes in flight to stream the weights; cutting K puts more
// workgroups on the machine at the price of fp32 partial sums that the reduction kernel adds up.
// The launch cuts K into chunks of ceil(K / s) rounded up to the tile depth of 64; a split is usable only if that
// leaves the last chunk non-empty (K = 1664 cut eight ways would give chunks of 256, of which six and a half exist).
inline bool ksplit_fits(int64_t K, int s)
{
    const int64_t chunk = ((K + s - 1) / s + 63) / 64 * 64;
    return s == 1 || chunk * (s - 1) < K;
}

inline int pick_ksplit(int64_t M, int64_t N, int64_t K, int count, int dtype, bool a_contig8, bool b_contig8)
{
    if (dtype != TT_BF16 || !a_contig8 || !b_contig8) return 1;
#ifdef TT_TUNING
    if (const char *e = std::getenv("TT_KSPLIT")) { // development builds only; powers of two, as the reduction assumes
        const int f = std::atoi(e);
        if (f >= 1 && (f & (f - 1)) == 0 && K / f >= 256 && count * f <= kMaxShards && ksplit_fits(K, f)) return f;
    }
#endif
    const int64_t blocks = ((M + 255) / 256) * ((N + 255) / 256) * count; // 256 x 256 tiles, one per CU
    // chunks stay at least 512 deep, except where the launch would otherwise occupy under a quarter of the CUs (the
    // 1000-wide last layer): there chunks down to 192 still pay for the extra partial sums
    // enough 256 x 128 tiles for the engine that runs two workgroups per CU: no split, so no partial sums to write and add
    // (the first-layer data gradient of the VGG-16 classifier: 74 us and no reduction instead of 64 us + 17 us)
    static const int min_half = tuning_int("TT_KSPLIT_HALF", 192);
    if (min_half > 0 && ((M + 255) / 256) * ((N + 127) / 128) * count >= min_half) return 1;
    int s = 1;
    // splitting stops once every second CU has a 256 x 256 tile's worth of work (at 200 the first AlexNet forward product,
    // 8 x 256 x 1024 x 4608, was cut eight ways: twice the partial sums of four ways for no faster a product, 4 % of its step)
    static const int min_blocks = tuning_int("TT_KSPLIT_BLOCKS", 128);
    while (blocks * s < min_blocks && s < 8 && K / (2 * s) >= (blocks * s < 64 ? 192 : 512) && count * 2 * s <= kMaxShards &&
           ksplit_fits(K, 2 * s))
        s *= 2;
    return s;
}

inline tt_status finish_output(const OutputPlan &op, const tt_tiling &tZ, void *const *Z, int64_t rows, int64_t cols, int k,
                               int dtype, int act, void *stream)
{
    if (op.mode == 0) return TT_OK;
    if (op.mode == 1) {
        tt_tiling az;
        for (int j = 0; j < k; ++j) az.cut[j] = op.zl[j];
        return launch_convert(Z, tZ.cut, const_cast<const void *const *>(op.gemm_out), az.cut, nullptr, nullptr, k, rows,
                              cols, dtype == TT_BF16 ? 2 : 4, 0, false, stream);
    }
    return launch_reduce(Z, tZ.cut, dtype, reinterpret_cast<const float *const *>(op.gemm_out), op.zl, k, rows, cols, act,
                         op.ksplit, stream);
}

inline bool forms_feasible(const uint8_t *forms, int k, int64_t M, int64_t N, int64_t K)
{
    int c[3] = {0, 0, 0};
    for (int j = 0; j < k; ++j) {
        if (forms[j] > TT_F3) return false;
        c[forms[j]]++;
    }
    return M % (int64_t(1) << c[0]) == 0 && N % (int64_t(1) << c[1]) == 0 && K % (int64_t(1) << c[2]) == 0;
}

inline void form_counts(const uint8_t *forms, int k, int *k1, int *k2, int *k3)
{
    *k1 = *k2 = *k3 = 0;
    for (int j = 0; j < k; ++j) { *k1 += forms[j] == TT_F1; *k2 += forms[j] == TT_F2; *k3 += forms[j] == TT_F3; }
}

} // namespace tt
