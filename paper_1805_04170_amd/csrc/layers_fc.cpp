// Fully-connected layer under a k-cut tiling: forward x_l = f(x_{l-1} W_l) and backward
// dC/dx_{l-1} = df(dC/dx_l) W_l^T, dC/dW_l = x_{l-1}^T df(dC/dx_l) (Sec. 2.1 of arXiv 1805.04170), each product run
// in the three phases of Sec. 4.2.1 / Sec. 5.2.
#include <hip/hip_runtime.h>
#include "exec_common.h"

namespace tt {
namespace {

struct FcArgs {
    const tt_layer *layer;
    int64_t batch;
    int k, dtype;
    tt_tiling tX, tW, tY, tdY, tdX;
    const uint8_t *forms_a, *forms_b;
    const void *const *X, *const *W, *const *Y, *const *dY;
    void *const *Yout, *const *dX, *const *dW;
    bool with_dx;
    void *stream;
    void *aux = nullptr; // optional second stream: the weight-gradient product runs there, beside the dX product
};

// Fork / join between the caller's two streams.  The events live per host thread and are made once; recording one
// again replaces its earlier use, which is what each call wants.
struct StreamFork {
    hipStream_t main = nullptr, side = nullptr;
    bool forked = false;
    static bool events(hipEvent_t *fork_ev, hipEvent_t *join_ev)
    {
        static thread_local hipEvent_t ev[2] = {nullptr, nullptr};
        for (int i = 0; i < 2; ++i)
            if (!ev[i] && hipEventCreateWithFlags(&ev[i], hipEventDisableTiming) != hipSuccess) return false;
        *fork_ev = ev[0];
        *join_ev = ev[1];
        return true;
    }
    // work enqueued on side after this call starts after everything enqueued on main so far
    tt_status fork(void *main_stream, void *side_stream)
    {
        main = reinterpret_cast<hipStream_t>(main_stream);
        side = reinterpret_cast<hipStream_t>(side_stream);
        hipEvent_t f, j;
        if (!events(&f, &j)) return TT_EDEVICE;
        if (hipEventRecord(f, main) != hipSuccess || hipStreamWaitEvent(side, f, 0) != hipSuccess) return TT_EDEVICE;
        forked = true;
        return TT_OK;
    }
    // work enqueued on main after this call starts after everything enqueued on side so far
    tt_status join()
    {
        if (!forked) return TT_OK;
        forked = false;
        hipEvent_t f, j;
        if (!events(&f, &j)) return TT_EDEVICE;
        if (hipEventRecord(j, side) != hipSuccess || hipStreamWaitEvent(main, j, 0) != hipSuccess) return TT_EDEVICE;
        return TT_OK;
    }
    ~StreamFork() { (void)join(); } // error paths: never leave the side stream dangling (it may be under capture)
};

tt_status check_common(const FcArgs &a)
{
    if (!a.layer || a.layer->kind != TT_FC || a.batch <= 0 || a.layer->n_in <= 0 || a.layer->n_out <= 0) return TT_EINVAL;
    if (!valid_k(a.k) || (a.dtype != TT_BF16 && a.dtype != TT_F32)) return TT_EINVAL;
    if (a.layer->act != TT_ACT_NONE && a.layer->act != TT_ACT_RELU) return TT_EINVAL;
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
    uint64_t c = matmul_cost(X, Y, Z, M, K, N, tx.cut, ty.cut, tz.cut, k, out, nullptr);
    return c == ~uint64_t(0) ? TT_EINFEASIBLE : TT_OK;
}

tt_status forward(const FcArgs &a, Workspace &ws)
{
    const int k = a.k, n = 1 << k;
    const int64_t M = a.batch, K = a.layer->n_in, N = a.layer->n_out;
    const int esz = a.dtype == TT_BF16 ? 2 : 4;
    if (!valid_tiling(a.tX, k) || !valid_tiling(a.tW, k) || !valid_tiling(a.tY, k)) return TT_EINVAL;
    uint8_t forms[TT_MAX_K];
    tt_status st = pick_forms(a.forms_a, forms, k, {M, K, 1}, {K, N, 1}, {M, N, 1}, M, K, N, a.tX, a.tW, a.tY);
    if (st != TT_OK) return st;
    tt_tiling aX, aW;
    aligned_tilings(forms, k, &aX, &aW, nullptr);
    int k1, k2, k3;
    form_counts(forms, k, &k1, &k2, &k3);

    Sharded X, W, Xa, Wa;
    set_sharded(&X, a.X, a.tX, k, M, K);
    set_sharded(&W, a.W, a.tW, k, K, N);
    if ((st = prepare_operand(X, aX, k, esz, nullptr, a.dtype, ws, a.stream, &Xa)) != TT_OK) return st;
    if ((st = prepare_operand(W, aW, k, esz, nullptr, a.dtype, ws, a.stream, &Wa)) != TT_OK) return st;
    OutputPlan op;
    const int64_t Ms = M >> k1, Ns = N >> k2, Ks = K >> k3;
    const int ksplit = pick_ksplit(Ms, Ns, Ks, n, a.dtype, Ks % 8 == 0, Ns % 8 == 0);
    if ((st = plan_output(forms, a.tY, a.Yout, M, N, k, a.dtype, a.layer->act, ws, &op, ksplit)) != TT_OK) return st;
    if (ws.dry) return TT_OK;
    st = launch_gemm(n, Xa.ptr, Wa.ptr, op.gemm_out, Ms, Ns, Ks, 0, 0, a.dtype, op.gemm_dtype, op.gemm_act, ksplit,
                     a.stream);
    if (st != TT_OK) return st;
    return finish_output(op, a.tY, a.Yout, M, N, k, a.dtype, a.layer->act, a.stream);
}

tt_status backward(const FcArgs &a, Workspace &ws)
{
    const int k = a.k, n = 1 << k;
    const int64_t b = a.batch, ni = a.layer->n_in, no = a.layer->n_out;
    const int esz = a.dtype == TT_BF16 ? 2 : 4;
    const bool relu = a.layer->act == TT_ACT_RELU;
    if (!valid_tiling(a.tX, k) || !valid_tiling(a.tW, k) || !valid_tiling(a.tdY, k)) return TT_EINVAL;
    if (relu && !valid_tiling(a.tY, k)) return TT_EINVAL;
    if (a.with_dx && !valid_tiling(a.tdX, k)) return TT_EINVAL;
    tt_status st;

    Sharded dY, Y, X, W;
    set_sharded(&dY, a.dY, a.tdY, k, b, no);
    set_sharded(&Y, a.Y, a.tY, k, b, no);
    set_sharded(&X, a.X, a.tX, k, b, ni);
    set_sharded(&W, a.W, a.tW, k, ni, no);

    // G = df(dY): the gate is applied once, while converting dY to the first aligned tiling that needs it;
    // afterwards that aligned copy stands in for the stored gradient.
    Sharded G = dY;
    bool gated = !relu;

    // dX = G W^T : M = b, K = n_out, N = n_in; second operand is W transposed
    uint8_t fd[TT_MAX_K];
    Sharded Ga_d;
    tt_tiling aW_d;
    int d1 = 0, d2 = 0, d3 = 0;
    if (a.with_dx) {
        const tt_tiling tWt = transpose_tiling(a.tW, k);
        st = pick_forms(a.forms_a, fd, k, {b, no, 1}, {no, ni, 1}, {b, ni, 1}, b, no, ni, a.tdY, tWt, a.tdX);
        if (st != TT_OK) return st;
        tt_tiling aG, aWt;
        aligned_tilings(fd, k, &aG, &aWt, nullptr);
        aW_d = transpose_tiling(aWt, k); // expressed on W as stored (n_in x n_out)
        form_counts(fd, k, &d1, &d2, &d3);
        if ((st = prepare_operand(G, aG, k, esz, gated ? nullptr : &Y, a.dtype, ws, a.stream, &Ga_d)) != TT_OK) return st;
        if (!gated) { G = Ga_d; gated = true; }
    }

    // With a second stream the weight gradient is enqueued there, after G exists, and runs beside the dX product.
    StreamFork fk;
    void *wstream = a.stream;
    if (a.aux && a.aux != a.stream && !ws.dry) {
        if ((st = fk.fork(a.stream, a.aux)) != TT_OK) return st;
        wstream = a.aux;
    }
    auto wgrad = [&]() -> tt_status {
        // dW = X^T G : M = n_in, K = b, N = n_out; first operand is X transposed; dW stored like W
        uint8_t f[TT_MAX_K];
        const tt_tiling tXt = transpose_tiling(a.tX, k);
        st = pick_forms(a.forms_b, f, k, {ni, b, 1}, {b, no, 1}, {ni, no, 1}, ni, b, no, tXt, a.tdY, a.tW);
        if (st != TT_OK) return st;
        tt_tiling aXt, aG;
        aligned_tilings(f, k, &aXt, &aG, nullptr);
        const tt_tiling aX = transpose_tiling(aXt, k);
        int k1, k2, k3;
        form_counts(f, k, &k1, &k2, &k3);
        Sharded Xa, Ga;
        if ((st = prepare_operand(X, aX, k, esz, nullptr, a.dtype, ws, wstream, &Xa)) != TT_OK) return st;
        if ((st = prepare_operand(G, aG, k, esz, gated ? nullptr : &Y, a.dtype, ws, wstream, &Ga)) != TT_OK) return st;
        OutputPlan op;
        if ((st = plan_output(f, a.tW, a.dW, ni, no, k, a.dtype, TT_ACT_NONE, ws, &op)) != TT_OK) return st;
        if (!ws.dry) {
            // X shard is (b/..) x (n_in/..) row-major = K x M: trans_a
            st = launch_gemm(n, Xa.ptr, Ga.ptr, op.gemm_out, ni >> k1, no >> k2, b >> k3, 1, 0, a.dtype, op.gemm_dtype,
                             op.gemm_act, 1, wstream);
            if (st != TT_OK) return st;
            if ((st = finish_output(op, a.tW, a.dW, ni, no, k, a.dtype, TT_ACT_NONE, wstream)) != TT_OK) return st;
        }
        return TT_OK;
    };
    auto dgrad = [&]() -> tt_status {
        if (!a.with_dx) return TT_OK;
        Sharded Wa;
        if ((st = prepare_operand(W, aW_d, k, esz, nullptr, a.dtype, ws, a.stream, &Wa)) != TT_OK) return st;
        OutputPlan op;
        const int64_t Ms = b >> d1, Ns = ni >> d2, Ks = no >> d3;
        const int ksplit = pick_ksplit(Ms, Ns, Ks, n, a.dtype, Ks % 8 == 0, Ks % 8 == 0);
        if ((st = plan_output(fd, a.tdX, a.dX, b, ni, k, a.dtype, TT_ACT_NONE, ws, &op, ksplit)) != TT_OK) return st;
        if (!ws.dry) {
            // W shard is (n_in/..) x (n_out/..) row-major = N x K: trans_b
            st = launch_gemm(n, Ga_d.ptr, Wa.ptr, op.gemm_out, Ms, Ns, Ks, 0, 1, a.dtype, op.gemm_dtype, op.gemm_act, ksplit,
                             a.stream);
            if (st != TT_OK) return st;
            if ((st = finish_output(op, a.tdX, a.dX, b, ni, k, a.dtype, TT_ACT_NONE, a.stream)) != TT_OK) return st;
        }
        return TT_OK;
    };
    // One stream: dX product first, then the weight gradient.  Two streams: the weight gradient is enqueued first so
    // that it is already running on the side stream while the dX product is being launched.
    if (fk.forked) {
        if ((st = wgrad()) != TT_OK) return st;
        if ((st = dgrad()) != TT_OK) return st;
    } else {
        if ((st = dgrad()) != TT_OK) return st;
        if ((st = wgrad()) != TT_OK) return st;
    }
    return fk.join();
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

extern "C" tt_status tt_fc_workspace_bytes(const tt_layer *layer, int64_t batch, int k, int dtype, int op, tt_tiling tX,
                                           tt_tiling tW, tt_tiling tY, tt_tiling tdY, tt_tiling tdX,
                                           const uint8_t *forms_a, const uint8_t *forms_b, int with_dx, size_t *bytes)
{
    if (!bytes) return TT_EINVAL;
    tt::FcArgs a{layer, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_a, forms_b, nullptr, nullptr, nullptr, nullptr,
                 nullptr, nullptr, nullptr, with_dx != 0, nullptr};
    tt_status st = tt::check_common(a);
    if (st != TT_OK) return st;
    tt::Workspace ws;
    ws.dry = true;
    if (op == TT_OP_FWD) st = tt::forward(a, ws);
    else if (op == TT_OP_DGRAD) st = tt::backward(a, ws);
    else return TT_EINVAL;
    if (st != TT_OK) return st;
    *bytes = tt::align_up(ws.used, 256);
    return TT_OK;
}

extern "C" tt_status tt_fc_forward(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                                   tt_tiling tY, const uint8_t *forms, const void *const *X, const void *const *W,
                                   void *const *Y, void *workspace, size_t ws_bytes, void *stream)
{
    tt::FcArgs a{layer, batch, k, dtype, tX, tW, tY, tY, tX, forms, nullptr, X, W, nullptr, nullptr, Y, nullptr, nullptr,
                 false, stream};
    tt_status st = tt::check_common(a);
    if (st != TT_OK) return st;
    const int n = 1 << k;
    if (tt::null_in(X, n) || tt::null_in(W, n) || tt::null_in(const_cast<const void *const *>(Y), n)) return TT_EINVAL;
    tt::Workspace ws;
    if ((st = tt::bind_workspace(ws, workspace, ws_bytes)) != TT_OK) return st;
    return tt::forward(a, ws);
}

extern "C" tt_status tt_fc_backward_overlapped(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX,
                                               tt_tiling tW, tt_tiling tY, tt_tiling tdY, tt_tiling tdX,
                                               const uint8_t *forms_dgrad, const uint8_t *forms_wgrad,
                                               const void *const *X, const void *const *W, const void *const *Y,
                                               const void *const *dY, void *const *dX, void *const *dW, void *workspace,
                                               size_t ws_bytes, void *stream, void *aux_stream);

extern "C" tt_status tt_fc_backward(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                                    tt_tiling tY, tt_tiling tdY, tt_tiling tdX, const uint8_t *forms_dgrad,
                                    const uint8_t *forms_wgrad, const void *const *X, const void *const *W,
                                    const void *const *Y, const void *const *dY, void *const *dX, void *const *dW,
                                    void *workspace, size_t ws_bytes, void *stream)
{
    tt::FcArgs a{layer, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_dgrad, forms_wgrad, X, W, Y, dY, nullptr, dX, dW,
                 dX != nullptr, stream};
    tt_status st = tt::check_common(a);
    if (st != TT_OK) return st;
    const int n = 1 << k;
    if (tt::null_in(X, n) || tt::null_in(W, n) || tt::null_in(dY, n) || tt::null_in(const_cast<const void *const *>(dW), n)) return TT_EINVAL;
    if (layer->act == TT_ACT_RELU && tt::null_in(Y, n)) return TT_EINVAL;
    if (dX && tt::null_in(const_cast<const void *const *>(dX), n)) return TT_EINVAL;
    tt::Workspace ws;
    if ((st = tt::bind_workspace(ws, workspace, ws_bytes)) != TT_OK) return st;
    return tt::backward(a, ws);
}

extern "C" tt_status tt_fc_backward_overlapped(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX,
                                               tt_tiling tW, tt_tiling tY, tt_tiling tdY, tt_tiling tdX,
                                               const uint8_t *forms_dgrad, const uint8_t *forms_wgrad,
                                               const void *const *X, const void *const *W, const void *const *Y,
                                               const void *const *dY, void *const *dX, void *const *dW, void *workspace,
                                               size_t ws_bytes, void *stream, void *aux_stream)
{
    tt::FcArgs a{layer, batch, k, dtype, tX, tW, tY, tdY, tdX, forms_dgrad, forms_wgrad, X, W, Y, dY, nullptr, dX, dW,
                 dX != nullptr, stream};
    a.aux = aux_stream;
    tt_status st = tt::check_common(a);
    if (st != TT_OK) return st;
    const int n = 1 << k;
    if (tt::null_in(X, n) || tt::null_in(W, n) || tt::null_in(dY, n) || tt::null_in(const_cast<const void *const *>(dW), n)) return TT_EINVAL;
    if (layer->act == TT_ACT_RELU && tt::null_in(Y, n)) return TT_EINVAL;
    if (dX && tt::null_in(const_cast<const void *const *>(dX), n)) return TT_EINVAL;
    tt::Workspace ws;
    if ((st = tt::bind_workspace(ws, workspace, ws_bytes)) != TT_OK) return st;
    return tt::backward(a, ws);
}
