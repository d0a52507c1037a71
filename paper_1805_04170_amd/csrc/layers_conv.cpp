// Convolution layer under a k-cut tiling (Sec. 4.5 of arXiv 1805.04170: only the batch and channel dimensions of the
// 4-D tensors are cut), run in the three phases of Sec. 4.2.1 / Sec. 5.2 like the fully-connected layer.
//
// 2-D views used for conversions and reductions (storage is NHWC / [K][R][S][C]):
//   activations  (N*H*W) x C   : tiling letters as given (R = batch rows, C = channel columns)
//   filters      (K*R*S) x C   : the filter tiling's R (input channels) cuts the columns, its C (output channels) cuts
//                                the rows, i.e. the letters are swapped on the storage matrix.
#include "exec_common.h"

namespace tt {
namespace {

struct ConvArgs {
    const tt_layer *layer;
    int64_t batch;
    int k, dtype;
    tt_tiling tX, tW, tY, tdY, tdX;
    const uint8_t *forms_a, *forms_b;
    const void *const *X, *const *W, *const *Y, *const *dY;
    void *const *Yout, *const *dX, *const *dW;
    bool with_dx;
    void *stream;
};

struct Dims { int64_t N, C, K, H, W, R, S, pad, P, Q; };

tt_status check(const ConvArgs &a, Dims *d)
{
    if (!a.layer || a.layer->kind != TT_CONV2D || a.batch <= 0) return TT_EINVAL;
    if (!valid_k(a.k)) return TT_EINVAL;
    if (a.dtype != TT_BF16 && a.dtype != TT_F32) return TT_EINVAL;
    if (a.layer->act != TT_ACT_NONE && a.layer->act != TT_ACT_RELU) return TT_EINVAL;
    const tt_layer &l = *a.layer;
    if (l.n_in <= 0 || l.n_out <= 0 || l.H <= 0 || l.W <= 0 || l.R <= 0 || l.S <= 0 || l.pad < 0) return TT_EINVAL;
    *d = Dims{a.batch, l.n_in, l.n_out, l.H, l.W, l.R, l.S, l.pad, l.H + 2 * l.pad - l.R + 1, l.W + 2 * l.pad - l.S + 1};
    if (d->P <= 0 || d->Q <= 0) return TT_EINVAL;
    return TT_OK;
}

tt_status pick_forms(const uint8_t *given, uint8_t *out, int k, const CostTensor &X, const CostTensor &Y,
                     const CostTensor &Z, int64_t M, int64_t K, int64_t N, const tt_tiling &tx, const tt_tiling &ty,
                     const tt_tiling &tz)
{
    if (given) {
        std::memcpy(out, given, (size_t)k);
        return forms_feasible(out, k, M, N, K) ? TT_OK : TT_EINFEASIBLE;
    }
    return matmul_cost(X, Y, Z, M, K, N, tx.cut, ty.cut, tz.cut, k, out, nullptr) == ~uint64_t(0) ? TT_EINFEASIBLE : TT_OK;
}

// an activation tensor as a sharded (N*HW) x channels matrix; the batch must split evenly
tt_status act_view(Sharded *s, const void *const *ptrs, const tt_tiling &t, int k, int64_t N, int64_t hw, int64_t ch)
{
    int kR = 0;
    for (int j = 0; j < k; ++j) kR += t.cut[j] == TT_R;
    if (N % (int64_t(1) << kR)) return TT_EINFEASIBLE;
    set_sharded(s, ptrs, t, k, N * hw, ch);
    return TT_OK;
}

// the filter tensor as a sharded (K*R*S) x C matrix with swapped letters
tt_status filter_view(Sharded *s, const void *const *ptrs, const tt_tiling &t, int k, const Dims &d)
{
    int kC = 0;
    for (int j = 0; j < k; ++j) kC += t.cut[j] == TT_C;
    if (d.K % (int64_t(1) << kC)) return TT_EINFEASIBLE;
    set_sharded(s, ptrs, transpose_tiling(t, k), k, d.K * d.R * d.S, d.C);
    return TT_OK;
}

// Number of partial sums per filter block, and the tile engine, for the weight gradient with an evenly cut reduction
// range; parts = 0 when that path does not apply.  The work items (output tiles times partial sums) run in rounds of as
// many as the chip holds; a round takes as long as one item's K tiles; every partial sum is written and read once more by
// the reduction.  Times in microseconds from measured rates on MI355X with the chip full: engine 1 (256 x 128 tiles, 512
// resident) 3.9 us per K tile, engine 2 (256 x 256 tiles, 256 resident) 2.6 us; partial sums at 4 TB/s.
struct WgradChoice { int parts, engine; };
WgradChoice pick_wgrad_parts(int k, int nblk, int nred, int64_t ktps, int64_t Ks, int64_t ncols, size_t blk_bytes)
{
    const int64_t total_kt = (int64_t)nred * ktps;
    const int max_parts = kMaxShards >> k;
    WgradChoice best{0, 1};
    double best_us = 0.0;
    const int forced = tuning_int("TT_WGRAD_PARTS", 0), forced_engine = tuning_int("TT_WGRAD_ENGINE", 0); // development builds only
    for (int engine = 1; engine <= 2; ++engine) {
        if (forced_engine && engine != forced_engine) continue;
        const int64_t tile_n = engine == 2 ? 256 : 128, resident = engine == 2 ? 256 : 512;
        const double kt_us = engine == 2 ? 2.6 : 3.9;
        const int64_t tiles = ((Ks + 255) / 256) * ((ncols + tile_n - 1) / tile_n);
        for (int parts = 1; parts <= max_parts && parts <= total_kt; ++parts) {
            const int64_t len = (total_kt + parts - 1) / parts;
            if (nred > 4 && (len + ktps - 1) / ktps + 1 > 4) continue; // an item may touch at most four shards
            if (parts == forced) return WgradChoice{parts, engine};
            const int64_t rounds = (nblk * tiles * parts + resident - 1) / resident;
            const double us = (double)rounds * (double)len * kt_us + (double)nblk * parts * (double)blk_bytes * 2.0 / 4.0e6;
            if (best.parts == 0 || us < best_us) { best = WgradChoice{parts, engine}; best_us = us; }
        }
    }
    return best;
}

// Shards that differ only in their side at the F2 cuts read the same left operand (its aligned tiling replicates it
// there).  Where each of them has few columns (at most 128: narrow tiles take in the left operand once per 64 or 128
// columns), they are run as one product per group, `members` column blocks side by side.
struct F2Group {
    int members = 1, groups = 0; // members == 1: run the shards one by one
    uint32_t mask2 = 0, mask_g = 0;
    uint32_t shard(int g, int m, int k) const { return deposit((uint32_t)g, mask_g, k) | deposit((uint32_t)m, mask2, k); }
};
F2Group f2_group(const uint8_t *forms, int k, int64_t cols_per_shard, int dtype)
{
    F2Group r;
    for (int j = 0; j < k; ++j)
        if (forms[j] == TT_F2) r.mask2 |= 1u << (k - 1 - j);
    r.mask_g = ((1u << k) - 1u) & ~r.mask2;
    const int k2 = __builtin_popcount(r.mask2);
    r.groups = (1 << k) >> k2;
    if (k2 > 0 && dtype == TT_BF16 && cols_per_shard <= 128 && cols_per_shard % 64 == 0 && tuning_int("TT_CONV_FUSE", 1) != 0)
        r.members = 1 << k2;
    else
        r.groups = 1 << k;
    return r;
}

tt_status forward(const ConvArgs &a, const Dims &d, Workspace &ws)
{
    const int k = a.k, n = 1 << k;
    if (!valid_tiling(a.tX, k) || !valid_tiling(a.tW, k) || !valid_tiling(a.tY, k)) return TT_EINVAL;
    const int64_t hw = d.H * d.W, pq = d.P * d.Q, rs = d.R * d.S;
    uint8_t f[TT_MAX_K];
    // product in the paper's terms: X (batch x C) times W (C x K) -> Y (batch x K); areas carry H*W, R*S, P*Q
    tt_status st = pick_forms(a.forms_a, f, k, {d.N, d.C, hw}, {d.C, d.K, rs}, {d.N, d.K, pq}, d.N, d.C, d.K, a.tX, a.tW, a.tY);
    if (st != TT_OK) return st;
    tt_tiling aX, aW;
    aligned_tilings(f, k, &aX, &aW, nullptr);
    int k1, k2, k3;
    form_counts(f, k, &k1, &k2, &k3);
    Sharded X, W, Xa, Wa;
    if ((st = act_view(&X, a.X, a.tX, k, d.N, hw, d.C)) != TT_OK) return st;
    if ((st = filter_view(&W, a.W, a.tW, k, d)) != TT_OK) return st;
    const int esz = a.dtype == TT_BF16 ? 2 : 4;
    // With fused shards the filters are converted to the aligned tiling with the F2 cuts replicated instead: every group
    // then holds ONE matrix of all its members' filter rows, member blocks one after the other.
    const F2Group fg = f2_group(f, k, d.K >> k2, a.dtype);
    tt_tiling aWs = transpose_tiling(aW, k);
    if (fg.members > 1)
        for (int j = 0; j < k; ++j)
            if (f[j] == TT_F2) aWs.cut[j] = TT_REP;
    if ((st = prepare_operand(X, aX, k, esz, nullptr, a.dtype, ws, a.stream, &Xa)) != TT_OK) return st;
    if ((st = prepare_operand(W, aWs, k, esz, nullptr, a.dtype, ws, a.stream, &Wa)) != TT_OK) return st;
    OutputPlan op;
    if ((st = plan_output(f, a.tY, a.Yout, d.N * pq, d.K, k, a.dtype, a.layer->act, ws, &op)) != TT_OK) return st;
    if (ws.dry) return TT_OK;
    if (fg.members > 1) {
        const void *fa[kMaxShards], *fb[kMaxShards];
        void *fc[kMaxShards];
        const size_t block_bytes = (size_t)(d.K >> k2) * (size_t)rs * (size_t)(d.C >> k3) * 2;
        for (int g = 0; g < fg.groups; ++g) {
            fa[g] = Xa.ptr[fg.shard(g, 0, k)];
            for (int m = 0; m < fg.members; ++m) {
                fb[g * fg.members + m] = static_cast<const char *>(Wa.ptr[fg.shard(g, 0, k)]) + (size_t)m * block_bytes;
                fc[g * fg.members + m] = op.gemm_out[fg.shard(g, m, k)];
            }
        }
        st = launch_conv_fused(TT_OP_FWD, fg.groups, fg.members, fa, fb, fc, d.N >> k1, d.K >> k2, d.C >> k3, d.H, d.W, d.R, d.S,
                               d.pad, op.gemm_dtype, op.gemm_act, a.stream, nullptr);
        if (st == TT_EUNSUPPORTED) { // shard by shard on the same buffers: member m's filters are block m of its group's matrix
            const void *xs[kMaxShards], *wsh[kMaxShards];
            for (int g = 0; g < fg.groups; ++g)
                for (int m = 0; m < fg.members; ++m) {
                    xs[fg.shard(g, m, k)] = fa[g];
                    wsh[fg.shard(g, m, k)] = fb[g * fg.members + m];
                }
            st = launch_conv(TT_OP_FWD, n, xs, wsh, op.gemm_out, d.N >> k1, d.C >> k3, d.K >> k2, d.H, d.W, d.R, d.S, d.pad,
                             op.gemm_dtype, op.gemm_act, a.stream, nullptr, a.dtype);
        }
    } else {
        st = launch_conv(TT_OP_FWD, n, Xa.ptr, Wa.ptr, op.gemm_out, d.N >> k1, d.C >> k3, d.K >> k2, d.H, d.W, d.R, d.S, d.pad,
                         op.gemm_dtype, op.gemm_act, a.stream, nullptr, a.dtype);
    }
    if (st != TT_OK) return st;
    return finish_output(op, a.tY, a.Yout, d.N * pq, d.K, k, a.dtype, a.layer->act, a.stream);
}

tt_status backward(const ConvArgs &a, const Dims &d, Workspace &ws)
{
    const int k = a.k, n = 1 << k;
    const bool relu = a.layer->act == TT_ACT_RELU;
    if (!valid_tiling(a.tX, k) || !valid_tiling(a.tW, k) || !valid_tiling(a.tdY, k)) return TT_EINVAL;
    if (relu && !valid_tiling(a.tY, k)) return TT_EINVAL;
    if (a.with_dx && !valid_tiling(a.tdX, k)) return TT_EINVAL;
    const int64_t hw = d.H * d.W, pq = d.P * d.Q, rs = d.R * d.S;
    const int esz = a.dtype == TT_BF16 ? 2 : 4;
    const bool bf16 = a.dtype == TT_BF16;
    tt_status st;
    Sharded dY, Y, X, W;
    if ((st = act_view(&dY, a.dY, a.tdY, k, d.N, pq, d.K)) != TT_OK) return st;
    if (relu && (st = act_view(&Y, a.Y, a.tY, k, d.N, pq, d.K)) != TT_OK) return st;
    if ((st = act_view(&X, a.X, a.tX, k, d.N, hw, d.C)) != TT_OK) return st;
    if ((st = filter_view(&W, a.W, a.tW, k, d)) != TT_OK) return st;
    Sharded G = dY; // gated once, on the way to the first aligned tiling that needs it
    bool gated = !relu;

    if (a.with_dx) {
        // dX (batch x C) = G (batch x K) times W^T (K x C): F1 batch, F2 input channels, F3 output channels
        uint8_t f[TT_MAX_K];
        const tt_tiling tWt = transpose_tiling(a.tW, k);
        st = pick_forms(a.forms_a, f, k, {d.N, d.K, pq}, {d.K, d.C, rs}, {d.N, d.C, hw}, d.N, d.K, d.C, a.tdY, tWt, a.tdX);
        if (st != TT_OK) return st;
        tt_tiling aG, aWt;
        aligned_tilings(f, k, &aG, &aWt, nullptr);
        int k1, k2, k3;
        form_counts(f, k, &k1, &k2, &k3);
        Sharded Ga, Wa;
        // Output channels cut (F3) so far that a shard keeps at most 128 of them: every shard's product then has a short
        // reduction (nine K tiles at 64 channels and 3 x 3 taps) and writes a whole fp32 partial sum of dX, which the
        // reduction kernel reads again.  On one GPU nothing forces that: the shards of a group (equal at every other cut)
        // read disjoint channel blocks of dY and of the filters, so with both brought to the aligned tiling with the F3
        // cuts replicated instead of split (one more copy of dY, which the weight gradient below then uses as it is; the
        // filters are small) the group is ONE product over all output channels that writes dX once, in its final type;
        // what is left of the output conversion is the copy into the stored tiling (its replicas, if it has any).
        const F2Group fg0 = f2_group(f, k, d.C >> k2, a.dtype);
        if (bf16 && k3 > 0 && (d.K >> k3) <= 128 && d.K > 128 && fg0.members == 1 && tuning_int("TT_DGRAD_MERGE", 1) != 0) {
            uint32_t mask_m = 0;
            uint8_t zl[TT_MAX_K];
            tt_tiling aGm = aG, aWm = aWt;
            for (int j = 0; j < k; ++j) {
                if (f[j] == TT_F3) {
                    mask_m |= 1u << (k - 1 - j);
                    aGm.cut[j] = aWm.cut[j] = TT_REP;
                }
                zl[j] = f[j] == TT_F1 ? TT_R : (f[j] == TT_F2 ? TT_C : TT_REP);
            }
            const uint32_t mask_keep = ((1u << k) - 1u) & ~mask_m;
            const int kp = k - k3, np = 1 << kp;
            if ((st = prepare_operand(G, aGm, k, esz, gated ? nullptr : &Y, a.dtype, ws, a.stream, &Ga)) != TT_OK) return st;
            G = Ga; // gated (if it had to be) and whole in its channels: the weight gradient starts from this copy
            gated = true;
            if ((st = prepare_operand(W, aWm, k, esz, nullptr, a.dtype, ws, a.stream, &Wa)) != TT_OK) return st;
            Grid gz;
            if (!make_grid(zl, k, d.N * hw, d.C, &gz)) return TT_EINFEASIBLE;
            const size_t out_bytes = (size_t)gz.srows * (size_t)gz.scols * 2;
            const size_t fbytes = (size_t)d.K * (size_t)rs * (size_t)(d.C >> k2) * 2;
            const void *Gp[kMaxShards], *Wp[kMaxShards], *src[kMaxShards];
            void *outp[kMaxShards], *flipp[kMaxShards];
            for (int sp = 0; sp < np; ++sp) {
                const uint32_t sid = deposit((uint32_t)sp, mask_keep, k);
                Gp[sp] = Ga.ptr[sid];
                Wp[sp] = Wa.ptr[sid];
                outp[sp] = ws.take(out_bytes);
                flipp[sp] = ws.take(fbytes);
            }
            for (int sh = 0; sh < n; ++sh) src[sh] = outp[extract((uint32_t)sh, mask_keep, k)]; // the group's result, whichever member is asked
            if (ws.overflow) return TT_EWORKSPACE;
            if (!ws.dry) {
                st = launch_conv(TT_OP_DGRAD, np, Gp, Wp, outp, d.N >> k1, d.C >> k2, d.K, d.H, d.W, d.R, d.S, d.pad, a.dtype,
                                 TT_ACT_NONE, a.stream, flipp, a.dtype);
                if (st != TT_OK) return st;
                st = launch_convert(a.dX, a.tdX.cut, src, zl, nullptr, nullptr, k, d.N * hw, d.C, esz, 0, false, a.stream);
                if (st != TT_OK) return st;
            }
        } else {
        if ((st = prepare_operand(G, aG, k, esz, gated ? nullptr : &Y, a.dtype, ws, a.stream, &Ga)) != TT_OK) return st;
        if (!gated) { G = Ga; gated = true; }
        // aligned tiling of W^T, expressed on W, then on the filter storage matrix: two swaps cancel
        if ((st = prepare_operand(W, aWt, k, esz, nullptr, a.dtype, ws, a.stream, &Wa)) != TT_OK) return st;
        OutputPlan op;
        if ((st = plan_output(f, a.tdX, a.dX, d.N * hw, d.C, k, a.dtype, TT_ACT_NONE, ws, &op)) != TT_OK) return st;
        // scratch for the flipped filters of every shard (the dX product then runs as a forward convolution of dY;
        // bf16 only: the fp32 kernels read the filters as they are)
        void *flip[kMaxShards];
        const size_t fbytes = (size_t)(d.K >> k3) * (size_t)rs * (size_t)(d.C >> k2) * 2;
        if (bf16) {
            // handed out group by group (shards that differ only at the F2 cuts, in the order of their column blocks), so
            // that a group's buffers lie one after the other: the fused product reads them as one filter matrix
            uint32_t mask2 = 0;
            for (int j = 0; j < k; ++j)
                if (f[j] == TT_F2) mask2 |= 1u << (k - 1 - j);
            const uint32_t mask_g = ((1u << k) - 1u) & ~mask2;
            const int members = 1 << __builtin_popcount(mask2);
            for (int g = 0; g < n / members; ++g)
                for (int m = 0; m < members; ++m)
                    flip[deposit((uint32_t)g, mask_g, k) | deposit((uint32_t)m, mask2, k)] = ws.take(fbytes);
        }
        if (ws.overflow) return TT_EWORKSPACE;
        if (!ws.dry) {
            const F2Group fg = f2_group(f, k, d.C >> k2, a.dtype);
            st = TT_EUNSUPPORTED;
            if (fg.members > 1) {
                const void *fa[kMaxShards], *fb[kMaxShards];
                void *fc[kMaxShards], *ff[kMaxShards];
                for (int g = 0; g < fg.groups; ++g) {
                    fa[g] = Ga.ptr[fg.shard(g, 0, k)];
                    for (int m = 0; m < fg.members; ++m) {
                        const uint32_t sid = fg.shard(g, m, k);
                        fb[g * fg.members + m] = Wa.ptr[sid];
                        fc[g * fg.members + m] = op.gemm_out[sid];
                        ff[g * fg.members + m] = flip[sid];
                    }
                }
                st = launch_conv_fused(TT_OP_DGRAD, fg.groups, fg.members, fa, fb, fc, d.N >> k1, d.C >> k2, d.K >> k3, d.H, d.W, d.R,
                                       d.S, d.pad, op.gemm_dtype, TT_ACT_NONE, a.stream, ff);
            }
            if (st == TT_EUNSUPPORTED) // filters that the flipped-filter path does not take: shard by shard
                st = launch_conv(TT_OP_DGRAD, n, Ga.ptr, Wa.ptr, op.gemm_out, d.N >> k1, d.C >> k2, d.K >> k3, d.H, d.W, d.R, d.S,
                                 d.pad, op.gemm_dtype, TT_ACT_NONE, a.stream, bf16 ? flip : nullptr, a.dtype);
            if (st != TT_OK) return st;
            if ((st = finish_output(op, a.tdX, a.dX, d.N * hw, d.C, k, a.dtype, TT_ACT_NONE, a.stream)) != TT_OK) return st;
        }
        } // (the per-shard / fused path)
    }
    {
        // dW (C x K) = X^T (C x batch) times G (batch x K): F1 input channels, F2 output channels, F3 batch
        uint8_t f[TT_MAX_K];
        const tt_tiling tXt = transpose_tiling(a.tX, k);
        st = pick_forms(a.forms_b, f, k, {d.C, d.N, hw}, {d.N, d.K, pq}, {d.C, d.K, rs}, d.C, d.N, d.K, tXt, a.tdY, a.tW);
        if (st != TT_OK) return st;
        tt_tiling aXt, aG;
        aligned_tilings(f, k, &aXt, &aG, nullptr);
        int k1, k2, k3;
        form_counts(f, k, &k1, &k2, &k3);
        Sharded Xa, Ga;
        const int64_t rows_w = d.K * rs; // the filter storage matrix is (K*R*S) x C
        // Channels cut so far that a shard keeps at most 128 of them leave every shard a sliver of the product: 64 rows of
        // dY^T against the whole gathered X where the output channels are cut (F2), or the whole dY^T against 64 gathered
        // channels per tap where the input channels are cut (F1: 576 columns make two and a quarter 256-wide tiles), and
        // the other operand, which the aligned tiling replicates at those cuts, is read again by every shard of the group.
        // Such shards run as ONE product over all their channels: the operand that was cut is brought to the aligned
        // tiling with those cuts replicated instead of split (dY: one more copy, made by the conversion that gates it
        // anyway; X stored replicated: nothing moves), the product is the evenly cut one below with those cuts taken out
        // of the shard numbering, and the reduction kernel, which scatters whole blocks into the stored tiling, sees those
        // cuts like cuts whose partial sums are already added up.
        if (bf16 && tuning_int("TT_WGRAD_MERGE", 1) != 0) {
            const bool m1 = k1 > 0 && (d.C >> k1) <= 128 && d.C > 128, m2 = k2 > 0 && (d.K >> k2) <= 128 && d.K > 128;
            const int64_t Cm = m1 ? d.C : d.C >> k1, Km = m2 ? d.K : d.K >> k2, Ns = d.N >> k3; // per product
            const int64_t lim = int64_t(1) << 30; // the evenly cut product's own limits (32-bit offsets, 16-byte chunks, tap masks)
            const bool fits = Cm % 8 == 0 && Km % 8 == 0 && Km > 128 && rs <= 32 && Ns * hw * Cm < lim && Ns * pq * Km < lim &&
                              Km * rs * Cm < lim && (Ns * pq) % 64 == 0;
            uint32_t mask_m = 0;
            uint8_t zr[TT_MAX_K], zp[TT_MAX_K]; // letters for the reduction (k cuts) and for the product (the cuts kept)
            tt_tiling aGm = aG, aXm = transpose_tiling(aXt, k);
            int kp = 0;
            for (int j = 0; j < k; ++j) {
                if ((f[j] == TT_F2 && m2) || (f[j] == TT_F1 && m1)) {
                    mask_m |= 1u << (k - 1 - j);
                    (f[j] == TT_F2 ? aGm : aXm).cut[j] = TT_REP;
                    zr[j] = kRed;
                } else {
                    zr[j] = zp[kp++] = f[j] == TT_F1 ? TT_C : (f[j] == TT_F2 ? TT_R : kRed);
                }
            }
            const uint32_t mask_keep = ((1u << k) - 1u) & ~mask_m;
            Grid gp, gr;
            if ((m1 || m2) && fits && make_grid(zp, kp, rows_w, d.C, &gp) && make_grid(zr, k, rows_w, d.C, &gr)) {
                const int nred = 1 << gp.kX, nblk = (1 << kp) >> gp.kX;
                const size_t blk_bytes = (size_t)gp.srows * (size_t)gp.scols * 4;
                const WgradChoice choice = pick_wgrad_parts(k, nblk, nred, Ns * pq / 64, Km, rs * Cm, blk_bytes);
                if (choice.parts > 0) {
                    if ((st = prepare_operand(X, aXm, k, esz, nullptr, a.dtype, ws, a.stream, &Xa)) != TT_OK) return st;
                    if ((st = prepare_operand(G, aGm, k, esz, gated ? nullptr : &Y, a.dtype, ws, a.stream, &Ga)) != TT_OK) return st;
                    const int parts = choice.parts;
                    uint8_t blk_ids[kMaxShards], red_ids[kMaxShards];
                    const uint32_t mask_blk = ((1u << kp) - 1u) & ~gp.maskX;
                    for (int b = 0; b < nblk; ++b) blk_ids[b] = (uint8_t)deposit((uint32_t)b, mask_blk, kp);
                    for (int q = 0; q < nred; ++q) red_ids[q] = (uint8_t)deposit((uint32_t)q, gp.maskX, kp);
                    void *sums[kMaxShards];
                    const float *table[kMaxShards];
                    for (int i = 0; i < kMaxShards; ++i) table[i] = nullptr;
                    for (int b = 0; b < nblk; ++b)
                        for (int c = 0; c < parts; ++c) {
                            sums[b * parts + c] = ws.take(blk_bytes);
                            // block b among the k cuts: its id in the product's numbering, spread over the cuts that were kept
                            table[deposit((uint32_t)blk_ids[b], mask_keep, k) * parts + c] = static_cast<const float *>(sums[b * parts + c]);
                        }
                    if (ws.overflow) return TT_EWORKSPACE;
                    if (ws.dry) return TT_OK;
                    const void *Gp[kMaxShards], *Xp[kMaxShards];
                    for (int s = 0; s < (1 << kp); ++s) {
                        const uint32_t sid = deposit((uint32_t)s, mask_keep, k);
                        Gp[s] = Ga.ptr[sid];
                        Xp[s] = Xa.ptr[sid];
                    }
                    st = launch_conv_wgrad_split(kp, nblk, nred, blk_ids, red_ids, parts, Gp, Xp, sums, Ns, Cm, Km, d.H, d.W, d.R, d.S,
                                                 d.pad, choice.engine, a.stream);
                    if (st != TT_OK) return st;
                    return launch_reduce(a.dW, transpose_tiling(a.tW, k).cut, a.dtype, table, zr, k, rows_w, d.C, TT_ACT_NONE, parts,
                                         a.stream, true);
                }
            }
        }
        if ((st = prepare_operand(X, transpose_tiling(aXt, k), k, esz, nullptr, a.dtype, ws, a.stream, &Xa)) != TT_OK) return st;
        if ((st = prepare_operand(G, aG, k, esz, gated ? nullptr : &Y, a.dtype, ws, a.stream, &Ga)) != TT_OK) return st;
        // the output grid on the filter storage matrix (K*R*S) x C: F1 cuts its columns, F2 its rows
        uint8_t zl[TT_MAX_K];
        for (int j = 0; j < k; ++j) zl[j] = f[j] == TT_F1 ? TT_C : (f[j] == TT_F2 ? TT_R : kRed);
        const tt_tiling tWs = transpose_tiling(a.tW, k);
        // The reduction of this product runs over every pixel of every image of the shard.
        const int64_t Ns = d.N >> k3, Cs = d.C >> k1, Ks = d.K >> k2;
        // First choice: the pixels of all shards that add up into one filter block form one reduction range, cut into
        // `parts` equal runs (pick_wgrad_parts; conv.hip says why that is free).  The partial sums then belong to a block,
        // not to a shard: buffer c of block b sits at table entry (b's shard id with zero F3 bits) * parts + c, which is
        // where the reduction kernel looks for it.
        Grid gz;
        if (!make_grid(zl, k, d.K * rs, d.C, &gz)) return TT_EINFEASIBLE;
        const int nred = 1 << gz.kX, nblk = n >> gz.kX;
        const size_t blk_bytes = (size_t)gz.srows * (size_t)gz.scols * 4;
        const WgradChoice choice = bf16 && (Ns * pq) % 64 == 0 && Ks > 128 ? pick_wgrad_parts(k, nblk, nred, Ns * pq / 64, Ks, rs * Cs, blk_bytes)
                                                                     : WgradChoice{0, 1};
        const int parts = choice.parts;
        if (parts > 0 && !(parts == 1 && nred == 1)) {
            uint8_t blk_ids[kMaxShards], red_ids[kMaxShards];
            const uint32_t mask_blk = ((1u << k) - 1u) & ~gz.maskX;
            for (int b = 0; b < nblk; ++b) blk_ids[b] = (uint8_t)deposit((uint32_t)b, mask_blk, k);
            for (int q = 0; q < nred; ++q) red_ids[q] = (uint8_t)deposit((uint32_t)q, gz.maskX, k);
            void *sums[kMaxShards];        // as the product numbers them: blk * parts + part
            const float *table[kMaxShards]; // as the reduction looks them up
            for (int i = 0; i < kMaxShards; ++i) table[i] = nullptr;
            for (int b = 0; b < nblk; ++b)
                for (int c = 0; c < parts; ++c) {
                    sums[b * parts + c] = ws.take(blk_bytes);
                    table[blk_ids[b] * parts + c] = static_cast<const float *>(sums[b * parts + c]);
                }
            if (ws.overflow) return TT_EWORKSPACE;
            if (ws.dry) return TT_OK;
            st = launch_conv_wgrad_split(k, nblk, nred, blk_ids, red_ids, parts, Ga.ptr, Xa.ptr, sums, Ns, Cs, Ks, d.H, d.W, d.R,
                                         d.S, d.pad, choice.engine, a.stream);
            if (st != TT_OK) return st; // (the shapes were checked above with the launcher's own conditions)
            return launch_reduce(a.dW, tWs.cut, a.dtype, table, zl, k, d.K * rs, d.C, TT_ACT_NONE, parts, a.stream, true);
        }
        // Otherwise: where the filter block of a shard gives too few output tiles to occupy the chip (input or output
        // channels cut, the batch not), the images of a shard are dealt to `split` sub-products, each writing its own fp32
        // partial sum, which the reduction kernel adds up together with the partial sums of the F3 cuts.  A sub-product is
        // the same product on a slice of the two operands: both are image-major, so the slice is an offset into the shard.
        int split = 1;
        {
            const int64_t tiles = ((Ks + 255) / 256) * ((rs * Cs + 127) / 128) * n; // 256 x 128 tiles of the filter gradient
            while (tiles * split < 256 && split < 8 && Ns % (2 * split) == 0 && n * 2 * split <= kMaxShards &&
                   (Ns / (2 * split)) * pq >= 2048)
                split *= 2;
        }
        OutputPlan op;
        if ((st = plan_output_letters(zl, tWs, a.dW, d.K * rs, d.C, k, a.dtype, TT_ACT_NONE, ws, &op, split)) != TT_OK) return st;
        if (!ws.dry) {
            const void *Gs[kMaxShards], *Xs[kMaxShards];
            const int64_t Nsub = Ns / split;
            for (int s = 0; s < n; ++s)
                for (int c = 0; c < split; ++c) {
                    Gs[s * split + c] = static_cast<const char *>(Ga.ptr[s]) + (size_t)c * Nsub * pq * Ks * esz;
                    Xs[s * split + c] = static_cast<const char *>(Xa.ptr[s]) + (size_t)c * Nsub * hw * Cs * esz;
                }
            st = launch_conv(TT_OP_WGRAD, n * split, Gs, Xs, op.gemm_out, Nsub, Cs, Ks, d.H, d.W, d.R, d.S, d.pad, op.gemm_dtype,
                             TT_ACT_NONE, a.stream, nullptr, a.dtype);
            if (st != TT_OK) return st;
            if ((st = finish_output(op, tWs, a.dW, d.K * rs, d.C, k, a.dtype, TT_ACT_NONE, a.stream)) != TT_OK) return st;
        }
    }
    return TT_OK;
}

bool null_in(const void *const *p, int n)
{
    if (!p) return true;
    for (int i = 0; i < n; ++i) if (!p[i]) return true;
    return false;
}

tt_status bind_workspace(Workspace &ws, void *workspace, size_t ws_bytes)
{
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255)) return TT_EWORKSPACE;
    ws.base = static_cast<char *>(workspace);
    ws.cap = workspace ? ws_bytes : 0;
    return TT_OK;
}

} // namespace
} // namespace tt

extern "C" tt_status tt_conv_workspace_bytes(const tt_layer *layer, int64_t batch, int k, int dtype, int op, tt_tiling tX,
                                             tt_tiling tW, tt_tiling tY, tt_tiling tdY, tt_tiling tdX,
                                             const uint8_t *forms_a, const uint8_t *forms_b, int with_dx, size_t *bytes)
{
    if (!bytes) return TT_EINVAL;
    tt::ConvArgs a{layer, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_a, forms_b, nullptr, nullptr, nullptr, nullptr,
                   nullptr, nullptr, nullptr, with_dx != 0, nullptr};
    tt::Dims d;
    tt_status st = tt::check(a, &d);
    if (st != TT_OK) return st;
    tt::Workspace ws;
    ws.dry = true;
    if (op == TT_OP_FWD) st = tt::forward(a, d, ws);
    else if (op == TT_OP_DGRAD) st = tt::backward(a, d, ws);
    else return TT_EINVAL;
    if (st != TT_OK) return st;
    *bytes = tt::align_up(ws.used, 256);
    return TT_OK;
}

extern "C" tt_status tt_conv_forward(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                                     tt_tiling tY, const uint8_t *forms, const void *const *X, const void *const *W,
                                     void *const *Y, void *workspace, size_t ws_bytes, void *stream)
{
    tt::ConvArgs a{layer, batch, k, dtype, tX, tW, tY, tY, tX, forms, nullptr, X, W, nullptr, nullptr, Y, nullptr, nullptr,
                   false, stream};
    tt::Dims d;
    tt_status st = tt::check(a, &d);
    if (st != TT_OK) return st;
    const int n = 1 << k;
    if (tt::null_in(X, n) || tt::null_in(W, n) || tt::null_in(const_cast<const void *const *>(Y), n)) return TT_EINVAL;
    tt::Workspace ws;
    if ((st = tt::bind_workspace(ws, workspace, ws_bytes)) != TT_OK) return st;
    return tt::forward(a, d, ws);
}

extern "C" tt_status tt_conv_backward(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                                      tt_tiling tY, tt_tiling tdY, tt_tiling tdX, const uint8_t *forms_dgrad,
                                      const uint8_t *forms_wgrad, const void *const *X, const void *const *W,
                                      const void *const *Y, const void *const *dY, void *const *dX, void *const *dW,
                                      void *workspace, size_t ws_bytes, void *stream)
{
    tt::ConvArgs a{layer, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_dgrad, forms_wgrad, X, W, Y, dY, nullptr, dX, dW,
                   dX != nullptr, stream};
    tt::Dims d;
    tt_status st = tt::check(a, &d);
    if (st != TT_OK) return st;
    const int n = 1 << k;
    if (tt::null_in(X, n) || tt::null_in(W, n) || tt::null_in(dY, n) || tt::null_in(const_cast<const void *const *>(dW), n)) return TT_EINVAL;
    if (layer->act == TT_ACT_RELU && tt::null_in(Y, n)) return TT_EINVAL;
    if (dX && tt::null_in(const_cast<const void *const *>(dX), n)) return TT_EINVAL;
    tt::Workspace ws;
    if ((st = tt::bind_workspace(ws, workspace, ws_bytes)) != TT_OK) return st;
    return tt::backward(a, d, ws);
}
