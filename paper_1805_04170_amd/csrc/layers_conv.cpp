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
    if (a.dtype != TT_BF16) return TT_EUNSUPPORTED; // the implicit-GEMM kernels are bf16 / fp32-accumulate only
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
    if ((st = prepare_operand(X, aX, k, 2, nullptr, a.dtype, ws, a.stream, &Xa)) != TT_OK) return st;
    if ((st = prepare_operand(W, transpose_tiling(aW, k), k, 2, nullptr, a.dtype, ws, a.stream, &Wa)) != TT_OK) return st;
    OutputPlan op;
    if ((st = plan_output(f, a.tY, a.Yout, d.N * pq, d.K, k, a.dtype, a.layer->act, ws, &op)) != TT_OK) return st;
    if (ws.dry) return TT_OK;
    st = launch_conv(TT_OP_FWD, n, Xa.ptr, Wa.ptr, op.gemm_out, d.N >> k1, d.C >> k3, d.K >> k2, d.H, d.W, d.R, d.S, d.pad,
                     op.gemm_dtype, op.gemm_act, a.stream);
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
        if ((st = prepare_operand(G, aG, k, 2, gated ? nullptr : &Y, a.dtype, ws, a.stream, &Ga)) != TT_OK) return st;
        if (!gated) { G = Ga; gated = true; }
        // aligned tiling of W^T, expressed on W, then on the filter storage matrix: two swaps cancel
        if ((st = prepare_operand(W, aWt, k, 2, nullptr, a.dtype, ws, a.stream, &Wa)) != TT_OK) return st;
        OutputPlan op;
        if ((st = plan_output(f, a.tdX, a.dX, d.N * hw, d.C, k, a.dtype, TT_ACT_NONE, ws, &op)) != TT_OK) return st;
        // scratch for the flipped filters of every shard (the dX product then runs as a forward convolution of dY)
        void *flip[kMaxShards];
        const size_t fbytes = (size_t)(d.K >> k3) * (size_t)rs * (size_t)(d.C >> k2) * 2;
        for (int s = 0; s < n; ++s) flip[s] = ws.take(fbytes);
        if (ws.overflow) return TT_EWORKSPACE;
        if (!ws.dry) {
            st = launch_conv(TT_OP_DGRAD, n, Ga.ptr, Wa.ptr, op.gemm_out, d.N >> k1, d.C >> k2, d.K >> k3, d.H, d.W, d.R, d.S,
                             d.pad, op.gemm_dtype, TT_ACT_NONE, a.stream, flip);
            if (st != TT_OK) return st;
            if ((st = finish_output(op, a.tdX, a.dX, d.N * hw, d.C, k, a.dtype, TT_ACT_NONE, a.stream)) != TT_OK) return st;
        }
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
        if ((st = prepare_operand(X, transpose_tiling(aXt, k), k, 2, nullptr, a.dtype, ws, a.stream, &Xa)) != TT_OK) return st;
        if ((st = prepare_operand(G, aG, k, 2, gated ? nullptr : &Y, a.dtype, ws, a.stream, &Ga)) != TT_OK) return st;
        // the output grid on the filter storage matrix (K*R*S) x C: F1 cuts its columns, F2 its rows
        uint8_t zl[TT_MAX_K];
        for (int j = 0; j < k; ++j) zl[j] = f[j] == TT_F1 ? TT_C : (f[j] == TT_F2 ? TT_R : kRed);
        const tt_tiling tWs = transpose_tiling(a.tW, k);
        // The reduction of this product runs over every pixel of every image of the shard.  Where the filter block of a
        // shard gives too few output tiles to occupy the chip (input or output channels cut, the batch not), the images of
        // a shard are dealt to `split` sub-products, each writing its own fp32 partial sum, which the reduction kernel adds
        // up together with the partial sums of the F3 cuts.  A sub-product is the same product on a slice of the two
        // operands: both are image-major, so the slice is an offset into the shard.
        const int64_t Ns = d.N >> k3, Cs = d.C >> k1, Ks = d.K >> k2;
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
                    Gs[s * split + c] = static_cast<const char *>(Ga.ptr[s]) + (size_t)c * Nsub * pq * Ks * 2;
                    Xs[s * split + c] = static_cast<const char *>(Xa.ptr[s]) + (size_t)c * Nsub * hw * Cs * 2;
                }
            st = launch_conv(TT_OP_WGRAD, n * split, Gs, Xs, op.gemm_out, Nsub, Cs, Ks, d.H, d.W, d.R, d.S, d.pad, op.gemm_dtype,
                             TT_ACT_NONE, a.stream);
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
