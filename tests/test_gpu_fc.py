"""Parity of the FC execute calls with the untiled fp64 oracle, per operation (each op is fed the stored operands,
so tolerances do not compound along the chain)."""
import itertools

import numpy as np
import pytest
import torch

import paper_1805_04170_amd as tt
from oracle import layers as ly
from oracle import tiling as tl
from oracle import execute as ex
from synthetic import CONFIGS, bf16_bits_to_f64, normal_f32, to_bf16_bits

from gpu_util import DEV, alloc_shards, dev_to_np, np_to_dev, shards_to_dev, shards_to_np

pytestmark = pytest.mark.gpu


def tdtype(dt):
    return torch.bfloat16 if dt == "bf16" else torch.float32


def to_store(v, dt):
    return to_bf16_bits(v) if dt == "bf16" else v.astype(np.float32)


def f64(a, dt):
    return bf16_bits_to_f64(a) if dt == "bf16" else a.astype(np.float64)


def workspace(nbytes):
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV)


def assert_close(got_shards, t, rows, cols, want, mag, dt, what):
    got = tl.untile(shards_to_np(got_shards), t, rows, cols)      # also checks replicas are identical
    gf = f64(got, dt)
    tol = (1e-2 if dt == "bf16" else 1e-5) * mag                   # the stated bound, nothing added
    err = np.abs(gf - want)
    assert np.all(np.isfinite(gf)), what
    assert np.all(err <= tol + 1e-30), (what, float(err.max()), float((err / (tol + 1e-30)).max()))


def run_layer(b, ni, no, k, dt, relu, tX, tW, tY, tdY, tdX, f_fwd, f_dg, f_wg, seed, with_dx=True):
    lay = tt.layer("fc", "relu" if relu else "none", ni, no)
    X = to_store(normal_f32(seed, 0, (b, ni), 1.0), dt)
    W = to_store(normal_f32(seed, 1, (ni, no), 0.05), dt)
    dY = to_store(normal_f32(seed, 2, (b, no), 1.0), dt)
    bf = dt == "bf16"
    Xs, Ws, dYs = shards_to_dev(X, tX, bf), shards_to_dev(W, tW, bf), shards_to_dev(dY, tdY, bf)
    Ys = alloc_shards(b, no, tY, tdtype(dt), fill=float("nan"))
    nb = tt.tt_fc_workspace_bytes(lay, b, k, dt, tt.TT_OP_FWD, tX, tW, tY, forms_a=f_fwd)
    ws = workspace(nb)
    tt.tt_fc_forward(lay, b, k, dt, tX, tW, tY, f_fwd, Xs, Ws, Ys, ws)
    torch.cuda.synchronize()
    Xf, Wf = f64(X, dt), f64(W, dt)
    want_Y = ly.fc_forward(Xf, Wf, relu)
    assert_close(Ys, tY, b, no, want_Y, ly.abs_product(Xf, Wf), dt, ("fwd", tX, tW, tY, f_fwd))
    # backward consumes the stored Y the GPU produced (so the gate decision is taken on identical values)
    Y_stored = f64(tl.untile(shards_to_np(Ys), tY, b, no), dt)
    dXs = alloc_shards(b, ni, tdX, tdtype(dt), fill=float("nan")) if with_dx else None
    dWs = alloc_shards(ni, no, tW, tdtype(dt), fill=float("nan"))
    nb = tt.tt_fc_workspace_bytes(lay, b, k, dt, tt.TT_OP_DGRAD, tX, tW, tY, tdY, tdX, f_dg, f_wg, with_dx)
    ws = workspace(nb)
    tt.tt_fc_backward(lay, b, k, dt, tX, tW, tY, tdY, tdX, f_dg, f_wg, Xs, Ws, Ys, dYs, dXs, dWs, ws)
    torch.cuda.synchronize()
    dYf = f64(dY, dt)
    want_dX, want_dW = ly.fc_backward(dYf, Xf, Wf, Y_stored, relu)
    G = dYf * (Y_stored > 0) if relu else dYf
    if with_dx:
        assert_close(dXs, tdX, b, ni, want_dX, ly.abs_product(G, Wf.T), dt, ("dgrad", tdY, tW, tdX, f_dg))
    assert_close(dWs, tW, ni, no, want_dW, ly.abs_product(Xf.T, G), dt, ("wgrad", tX, tdY, tW, f_wg))


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_named_tilings_one_and_two_cuts(dt, golden_loader):
    g = golden_loader("paper_tilings.txt")
    # T_data, T_model (one cut) and T_hybrid (two cuts) of Sec. 4.1: weight / activation / gradient tilings
    for name in ["T_data", "T_model", "T_hybrid"]:
        tW, tA, tG = g[name]
        k = len(tW)
        run_layer(32, 64, 48, k, dt, True, tA, tW, tA, tG, tG, None, None, None, 50 + k)


@pytest.mark.parametrize("relu", [False, True])
def test_every_form_sequence_two_cuts(relu):
    # fixed stored tilings, every aligned form sequence for each of the three products
    seqs = ["".join(p) for p in itertools.product("123", repeat=2)]
    for f in seqs:
        run_layer(16, 32, 24, 2, "bf16", relu, "RC", "Cr", "rR", "CR", "RR", f, f, f, 60)


def test_random_stored_tilings_default_forms():
    rng = np.random.default_rng(5)
    ts = tl.all_tilings(2)
    for i in range(25):
        tX, tW, tY, tdY, tdX = (ts[j] for j in rng.integers(0, 9, 5))
        run_layer(16, 40, 24, 2, "bf16" if i % 2 else "f32", bool(i % 3), tX, tW, tY, tdY, tdX, None, None, None, 70 + i)


def test_three_cuts_ragged_width_and_skip_dx():
    run_layer(64, 96, 1000, 3, "bf16", False, "CCC", "RRR", "RRR", "rrr", "CCC", "333", "222", "111", 80)
    run_layer(64, 96, 1000, 3, "bf16", True, "RRR", "rrr", "RRC", "RCR", "RRR", None, None, None, 81, with_dx=False)
    run_layer(64, 1000, 40, 3, "bf16", True, "rCr", "CRC", "CrC", "CrC", "RCR", "232", "323", "212", 82)


def _backward_once(fn, lay, b, k, dt, t, forms, Xs, Ws, Ys, dYs, ni, no, **kw):
    dXs = alloc_shards(b, ni, t["dX"], tdtype(dt), fill=float("nan"))
    dWs = alloc_shards(ni, no, t["W"], tdtype(dt), fill=float("nan"))
    nb = tt.tt_fc_workspace_bytes(lay, b, k, dt, tt.TT_OP_DGRAD, t["X"], t["W"], t["Y"], t["dY"], t["dX"], forms[0], forms[1])
    ws = workspace(nb)
    fn(lay, b, k, dt, t["X"], t["W"], t["Y"], t["dY"], t["dX"], forms[0], forms[1], Xs, Ws, Ys, dYs, dXs, dWs, ws, **kw)
    return dXs, dWs, ws


@pytest.mark.parametrize("relu", [False, True])
def test_backward_overlapped_equals_backward(relu):
    # the two-stream variant must produce the very same bits, eagerly and as a captured graph replayed several times
    b, ni, no, k, dt = 64, 512, 384, 3, "bf16"
    t = dict(X="CCr", W="RRC", Y="CCC", dY="CrC", dX="CCr")
    forms = ("233", "112")
    lay = tt.layer("fc", "relu" if relu else "none", ni, no)
    X = to_store(normal_f32(90, 0, (b, ni), 1.0), dt)
    W = to_store(normal_f32(90, 1, (ni, no), 0.05), dt)
    Y = to_store(normal_f32(90, 3, (b, no), 1.0), dt)
    dY = to_store(normal_f32(90, 2, (b, no), 1.0), dt)
    Xs, Ws, Ys, dYs = (shards_to_dev(a, tt_, True) for a, tt_ in ((X, t["X"]), (W, t["W"]), (Y, t["Y"]), (dY, t["dY"])))
    ref_dX, ref_dW, _ = _backward_once(tt.tt_fc_backward, lay, b, k, dt, t, forms, Xs, Ws, Ys, dYs, ni, no)
    torch.cuda.synchronize()
    aux = torch.cuda.Stream()
    got_dX, got_dW, _ = _backward_once(tt.tt_fc_backward_overlapped, lay, b, k, dt, t, forms, Xs, Ws, Ys, dYs, ni, no, aux_stream=aux)
    torch.cuda.synchronize()
    for g, r in zip(got_dX + got_dW, ref_dX + ref_dW):
        assert torch.equal(g.view(torch.int16), r.view(torch.int16))
    # captured: outputs and workspace allocated outside the capture, work launched on the capturing stream
    dXs = alloc_shards(b, ni, t["dX"], tdtype(dt), fill=float("nan"))
    dWs = alloc_shards(ni, no, t["W"], tdtype(dt), fill=float("nan"))
    ws = workspace(tt.tt_fc_workspace_bytes(lay, b, k, dt, tt.TT_OP_DGRAD, t["X"], t["W"], t["Y"], t["dY"], t["dX"], forms[0], forms[1]))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        tt.tt_fc_backward_overlapped(lay, b, k, dt, t["X"], t["W"], t["Y"], t["dY"], t["dX"], forms[0], forms[1], Xs, Ws, Ys,
                                     dYs, dXs, dWs, ws, aux_stream=aux)
    for rep in range(3):
        for d in dXs + dWs:
            d.fill_(float("nan"))                                 # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for g, r in zip(dXs + dWs, ref_dX + ref_dW):
            assert torch.equal(g.view(torch.int16), r.view(torch.int16)), rep


def test_whole_step_as_replayed_graph_equals_eager():
    # what bench.py times: one forward + backward step of a planned chain captured into a HIP graph and replayed; every
    # replay must reproduce the eager step bit for bit (eager work and synchronisations between the replays)
    from synthetic.configs import FcChain
    cfg = FcChain("graph_small", 256, (2048, 1024, 1024, 1000), 3, "bf16", 0.02, 2006)
    plan = plan_for(cfg)
    dt, k, b, L = cfg.dtype, cfg.k, cfg.batch, cfg.n_layers
    x0, Ws, gL = chain_tensors(cfg)
    tx, tg, tw = plan.x(), plan.g(), plan.w()
    layers = [tt.layer("fc", "relu" if cfg.act(l) else "none", cfg.widths[l - 1], cfg.widths[l]) for l in range(1, L + 1)]
    xs = [shards_to_dev(x0, tx[0], True)] + [alloc_shards(b, cfg.widths[l], tx[l], torch.bfloat16, fill=float("nan")) for l in range(1, L + 1)]
    gs = [alloc_shards(b, cfg.widths[l], tg[l], torch.bfloat16, fill=float("nan")) for l in range(L)] + [shards_to_dev(gL, tg[L], True)]
    wsh = [shards_to_dev(Ws[l], tw[l], True) for l in range(L)]
    dws = [alloc_shards(cfg.widths[l], cfg.widths[l + 1], tw[l], torch.bfloat16, fill=float("nan")) for l in range(L)]
    need = 256
    for l in range(1, L + 1):
        f = [plan.forms(l, op) for op in range(3)]
        need = max(need, tt.tt_fc_workspace_bytes(layers[l - 1], b, k, dt, tt.TT_OP_FWD, tx[l - 1], tw[l - 1], tx[l], forms_a=f[0]),
                   tt.tt_fc_workspace_bytes(layers[l - 1], b, k, dt, tt.TT_OP_DGRAD, tx[l - 1], tw[l - 1], tx[l], tg[l], tg[l - 1], f[1], f[2]))
    ws = workspace(need)

    def step():
        for l in range(1, L + 1):
            tt.tt_fc_forward(layers[l - 1], b, k, dt, tx[l - 1], tw[l - 1], tx[l], plan.forms(l, tt.TT_OP_FWD), xs[l - 1], wsh[l - 1], xs[l], ws)
        for l in range(L, 0, -1):
            tt.tt_fc_backward(layers[l - 1], b, k, dt, tx[l - 1], tw[l - 1], tx[l], tg[l], tg[l - 1], plan.forms(l, tt.TT_OP_DGRAD),
                              plan.forms(l, tt.TT_OP_WGRAD), xs[l - 1], wsh[l - 1], xs[l], gs[l], gs[l - 1], dws[l - 1], ws)

    outputs = [t for l in range(1, L + 1) for t in xs[l]] + [t for l in range(L) for t in gs[l]] + [t for l in range(L) for t in dws[l]]
    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outputs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in outputs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, r in zip(outputs, ref):
            assert torch.equal(t.view(torch.int16), r.view(torch.int16)), rep


def test_uneven_and_bad_workspace_are_refused():
    lay = tt.layer("fc", "none", 10, 6)
    x = [torch.zeros(8, dtype=torch.bfloat16, device=DEV)] * 4
    with pytest.raises(tt.TilingError) as e:
        tt.tt_fc_forward(lay, 8, 2, "bf16", "RR", "rr", "CC", "22", x, x, x)
    assert e.value.status == 2
    lay = tt.layer("fc", "none", 16, 16)
    with pytest.raises(tt.TilingError) as e:                     # K-split needs partial-sum workspace
        tt.tt_fc_forward(lay, 8, 2, "bf16", "CC", "RR", "RR", "33", x, x, x)
    assert e.value.status == 6


def chain_tensors(cfg):
    return cfg.x0(), [cfg.weight(l) for l in range(1, cfg.n_layers + 1)], cfg.grad_out()


def run_chain(cfg, plan):
    """Forward and backward of a whole chain under a plan; every element of every activation, activation gradient and
    weight gradient is compared with the oracle applied to the operands the GPU actually stored (per operation, so
    tolerances do not compound along the chain).  Returns the largest error / bound ratio seen per kind of product."""
    dt, k, b, L = cfg.dtype, cfg.k, cfg.batch, cfg.n_layers
    bf = dt == "bf16"
    x0, Ws, gL = chain_tensors(cfg)
    tx, tg, tw = plan.x(), plan.g(), plan.w()
    layers = [tt.layer("fc", "relu" if cfg.act(l) else "none", cfg.widths[l - 1], cfg.widths[l]) for l in range(1, L + 1)]
    xs = [shards_to_dev(x0, tx[0], bf)]
    wsh = [shards_to_dev(Ws[l], tw[l], bf) for l in range(L)]
    for l in range(1, L + 1):
        f = plan.forms(l, tt.TT_OP_FWD)
        ys = alloc_shards(b, cfg.widths[l], tx[l], tdtype(dt), fill=float("nan"))
        nb = tt.tt_fc_workspace_bytes(layers[l - 1], b, k, dt, tt.TT_OP_FWD, tx[l - 1], tw[l - 1], tx[l], forms_a=f)
        tt.tt_fc_forward(layers[l - 1], b, k, dt, tx[l - 1], tw[l - 1], tx[l], f, xs[l - 1], wsh[l - 1], ys, workspace(nb))
        xs.append(ys)
    torch.cuda.synchronize()
    tol_c = 1e-2 if bf else 1e-5                                   # the stated bounds, nothing added
    worst = {"fwd": 0.0, "dgrad": 0.0, "wgrad": 0.0}

    def compare(kind, l, got, want, mag):
        err = np.abs(got - want)
        assert np.all(np.isfinite(got)), (kind, l)
        bound = tol_c * mag + 1e-30
        assert np.all(err <= bound), (kind, l, float(err.max()), np.argwhere(err > bound)[:5])
        worst[kind] = max(worst[kind], float((err / bound).max()))

    full_x = [f64(tl.untile(shards_to_np(xs[l]), tx[l], b, cfg.widths[l]), dt) for l in range(L + 1)]
    Wf = [f64(w, dt) for w in Ws]
    for l in range(1, L + 1):
        compare("fwd", l, full_x[l], ly.fc_forward(full_x[l - 1], Wf[l - 1], bool(cfg.act(l))),
                ly.abs_product(full_x[l - 1], Wf[l - 1]))
    gs = [None] * (L + 1)
    gs[L] = shards_to_dev(gL, tg[L], bf)
    dws = [None] * L
    for l in range(L, 0, -1):
        fd, fw = plan.forms(l, tt.TT_OP_DGRAD), plan.forms(l, tt.TT_OP_WGRAD)
        gs[l - 1] = alloc_shards(b, cfg.widths[l - 1], tg[l - 1], tdtype(dt), fill=float("nan"))
        dws[l - 1] = alloc_shards(cfg.widths[l - 1], cfg.widths[l], tw[l - 1], tdtype(dt), fill=float("nan"))
        nb = tt.tt_fc_workspace_bytes(layers[l - 1], b, k, dt, tt.TT_OP_DGRAD, tx[l - 1], tw[l - 1], tx[l], tg[l], tg[l - 1], fd, fw)
        tt.tt_fc_backward(layers[l - 1], b, k, dt, tx[l - 1], tw[l - 1], tx[l], tg[l], tg[l - 1], fd, fw, xs[l - 1], wsh[l - 1],
                          xs[l], gs[l], gs[l - 1], dws[l - 1], workspace(nb))
    torch.cuda.synchronize()
    full_g = [f64(tl.untile(shards_to_np(gs[l]), tg[l], b, cfg.widths[l]), dt) for l in range(L + 1)]
    for l in range(L, 0, -1):
        relu = bool(cfg.act(l))
        G = full_g[l] * (full_x[l] > 0) if relu else full_g[l]
        want_dx, want_dw = ly.fc_backward(full_g[l], full_x[l - 1], Wf[l - 1], full_x[l], relu)
        compare("dgrad", l, full_g[l - 1], want_dx, ly.abs_product(G, Wf[l - 1].T))
        ni = cfg.widths[l - 1]
        dW = f64(tl.untile(shards_to_np(dws[l - 1]), tw[l - 1], ni, cfg.widths[l]), dt)
        dws[l - 1] = None
        compare("wgrad", l, dW, want_dw, ly.abs_product(full_x[l - 1].T, G))
        del dW, want_dx, want_dw
    worst["chain"] = end_to_end(cfg, f64(x0, dt), Wf, f64(gL, dt), full_x[L], full_g[0], tol_c)
    print("chain %s: per product err / bound fwd %.3f dgrad %.3f wgrad %.3f; end to end x_L %.2e g_0 %.2e of the magnitude chain, "
          "rms error / rms value x_L %.2e g_0 %.2e" % (cfg.name, worst["fwd"], worst["dgrad"], worst["wgrad"], worst["chain"]["x_L"],
                                                       worst["chain"]["g_0"], worst["chain"]["x_L_rms"], worst["chain"]["g_0_rms"]))
    return worst


def end_to_end(cfg, x0, Wf, gL, got_xL, got_g0, tol_c):
    """The chain as a whole, reported separately from the per-product checks: the oracle runs forward and backward
    untiled in fp64 from the same inputs, never seeing a GPU intermediate, so the GPU's rounding of every stored tensor
    compounds along the chain.  The scale is the chain of magnitude products (|x_0| |W_1| ... |W_L| and
    |g_L| |W_L|^T ... |W_1|^T).  Forward: every layer adds at most one product's error, and ReLU does not stretch
    differences, so L times the per-product bound holds and is asserted.  Backward: where a stored activation and the
    oracle's differ in sign (both within rounding of zero) the gate passes a gradient on one side only; that difference
    is bounded by the scale, not by a rounding error, so the figure is reported and only checked to be finite."""
    L = cfg.n_layers
    xo, mag = [x0], np.abs(x0)
    for l in range(1, L + 1):
        xo.append(ly.fc_forward(xo[l - 1], Wf[l - 1], bool(cfg.act(l))))
        mag = ly.abs_product(mag, Wf[l - 1])
    fwd = np.abs(got_xL - xo[L]) / (mag + 1e-30)
    assert np.all(fwd <= L * tol_c), ("whole chain forward", float(fwd.max()))
    go, gmag = gL, np.abs(gL)
    for l in range(L, 0, -1):
        go, _ = ly.fc_backward(go, xo[l - 1], Wf[l - 1], xo[l], bool(cfg.act(l)))
        gmag = ly.abs_product(gmag, Wf[l - 1].T)
    bwd = np.abs(got_g0 - go) / (gmag + 1e-30)
    assert np.all(np.isfinite(got_g0))
    rms = lambda a: float(np.sqrt(np.mean(np.square(a))))
    return {"x_L": float(fwd.max()), "g_0": float(bwd.max()), "x_L_rms": rms(got_xL - xo[L]) / (rms(xo[L]) + 1e-300),
            "g_0_rms": rms(got_g0 - go) / (rms(go) + 1e-300)}


def plan_for(cfg, mode=tt.TT_PLAN_EXACT, **pins):
    layers = [tt.layer("fc", "none", cfg.widths[l], cfg.widths[l + 1]) for l in range(cfg.n_layers)]
    return tt.tt_plan_chain(layers, cfg.batch, cfg.k, mode, **pins)


def test_config_tiny_mlp_fp32_planned_and_recursive():
    cfg = CONFIGS["tiny_mlp"]
    run_chain(cfg, plan_for(cfg))
    run_chain(cfg, plan_for(cfg, tt.TT_PLAN_RECURSIVE))
    run_chain(cfg, plan_for(cfg, pin_x0="RR", pin_g0="RR"))


@pytest.mark.parametrize("name", ["alexnet_fc", "vgg16_fc"])
def test_config_fc_stacks_full_size(name):
    cfg = CONFIGS[name]
    run_chain(cfg, plan_for(cfg))


class ForcedPlan:
    """A fixed graph tiling with the accessors of a planner result."""

    def __init__(self, L, tx, tg, tw, forms):
        self._x, self._g, self._w, self._f = [tx] * (L + 1), [tg] * (L + 1), [tw] * L, forms

    def x(self):
        return self._x

    def g(self):
        return self._g

    def w(self):
        return self._w

    def forms(self, layer_index, op):
        return self._f[op]


def test_config_wide_mlp_full_size_forced_tiling():
    # 8 x (8192 -> 8192), batch 512, 16 shards; every tensor stored as a 4 x 4 grid (RRCC); the forward and dgrad
    # products split the reduction dimension twice (4-way partial-sum reduce) and need a real conversion of their
    # first operand; the weight gradient lands directly in the stored grid.
    cfg = CONFIGS["wide_mlp"]
    plan = ForcedPlan(cfg.n_layers, "RRCC", "RRCC", "RRCC", ["3322", "2233", "1122"])
    run_chain(cfg, plan)


def test_wide_mlp_shapes_sixteen_way_reduce():
    # the variant with all four cuts on the reduction dimension (16 partial sums), at reduced width
    from synthetic.configs import FcChain
    cfg = FcChain("wide_small", 128, (1024, 1024, 1024), 4, "bf16", 0.01, 2005)
    plan = ForcedPlan(cfg.n_layers, "CCCC", "rrrr", "RRRR", ["3333", "2222", "1111"])
    run_chain(cfg, plan)
