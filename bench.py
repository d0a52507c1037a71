#!/usr/bin/env python3
"""Benchmark of the tiled execution hot path on one MI355X.

One step = forward and backward of the whole FC stack (all 3 products per layer, with their input conversions,
output conversions and partial-sum reductions) under the planner's minimum-communication k-cut tiling, all 2^k
shards living in this GPU's HBM.  Inputs are resident in HBM before the timed region.  The timed region replays a
HIP graph of one step K times; a second, eager pass of K steps brackets every kernel with HIP events (on the launch
stream) to get per-kernel durations for the roofline line.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM traffic per launch (read + write bytes) of the large shard products from the rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs summarised in profiles/vgg16_fc_step_hbm_traffic_pmc.txt (counters scaled by what the same counters
# read for the W_1 retile, a copy of known size).  Keyed by workload, kernel and per-shard M x N x K; None if not measured.
MEASURED_TRAFFIC_BYTES = {
    "vgg16_fc:gemm_tn:3136x4096x256": int((30.10 + 205.61) * 1e6),
    "vgg16_fc:gemm_nn:256x4096x3136": int((218.66 + 67.11) * 1e6),
    "vgg16_fc:gemm_nt:256x3136x4096": int((222.41 + 51.44) * 1e6),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vgg16_fc",
                    choices=["vgg16_fc", "alexnet_fc", "wide_mlp", "tiny_mlp", "vgg16_conv4", "shape_study"])
    ap.add_argument("--conv-split", default="planner", choices=["planner", "batch", "out_channel"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a HIP graph replay")
    ap.add_argument("--overlap", action="store_true",
                    help="weight-gradient products on a second stream (tt_fc_backward_overlapped); default: one stream, "
                         "which measured faster on the batch-256 workloads, whose large products are all bound by HBM")
    return ap.parse_args()


class Chain:
    """Device state of one FC chain under a plan: shards of x_l, g_l, W_l, dW_l and one workspace."""

    def __init__(self, cfg, tt, torch, tilings=None):
        import numpy as np
        from synthetic import CONFIGS  # noqa: F401
        self.cfg, self.tt, self.torch = cfg, tt, torch
        self.k, self.b, self.L, self.dt = cfg.k, cfg.batch, cfg.n_layers, cfg.dtype
        self.layers = [tt.layer("fc", "relu" if cfg.act(l) else "none", cfg.widths[l - 1], cfg.widths[l])
                       for l in range(1, self.L + 1)]
        if tilings is None:
            plan = tt.tt_plan_chain([tt.layer("fc", "none", cfg.widths[l], cfg.widths[l + 1]) for l in range(self.L)],
                                    self.b, self.k, tt.TT_PLAN_EXACT)
            self.tx, self.tg, self.tw = plan.x(), plan.g(), plan.w()
            self.forms = [[plan.forms(l, op) for op in range(3)] for l in range(1, self.L + 1)]
            self.plan_cost = plan.cost
        else:
            self.tx, self.tg, self.tw, self.forms = tilings
            self.plan_cost = None
        tdt = torch.bfloat16 if self.dt == "bf16" else torch.float32
        dev = "cuda:0"

        def upload(T, t):
            out = []
            rows, cols = T.shape
            sr, sc = tt.tt_shard_shape(rows, cols, t)
            n = 1 << self.k
            for s in range(n):
                rb, cb = block_of(t, s)
                piece = np.ascontiguousarray(T[rb * sr:(rb + 1) * sr, cb * sc:(cb + 1) * sc])
                if self.dt == "bf16":
                    out.append(torch.from_numpy(piece.view(np.int16)).to(dev).view(torch.bfloat16))
                else:
                    out.append(torch.from_numpy(piece).to(dev))
            return out

        def empty(rows, cols, t):
            sr, sc = tt.tt_shard_shape(rows, cols, t)
            return [torch.zeros((sr, sc), dtype=tdt, device=dev) for _ in range(1 << self.k)]

        w = cfg.widths
        self.x = [upload(cfg.x0(), self.tx[0])] + [empty(self.b, w[l], self.tx[l]) for l in range(1, self.L + 1)]
        self.g = [empty(self.b, w[l], self.tg[l]) for l in range(self.L)] + [upload(cfg.grad_out(), self.tg[self.L])]
        self.W = [upload(cfg.weight(l), self.tw[l - 1]) for l in range(1, self.L + 1)]
        self.dW = [empty(w[l - 1], w[l], self.tw[l - 1]) for l in range(1, self.L + 1)]
        need = 256
        for l in range(1, self.L + 1):
            f = self.forms[l - 1]
            need = max(need, tt.tt_fc_workspace_bytes(self.layers[l - 1], self.b, self.k, self.dt, tt.TT_OP_FWD,
                                                      self.tx[l - 1], self.tw[l - 1], self.tx[l], forms_a=f[0]))
            need = max(need, tt.tt_fc_workspace_bytes(self.layers[l - 1], self.b, self.k, self.dt, tt.TT_OP_DGRAD,
                                                      self.tx[l - 1], self.tw[l - 1], self.tx[l], self.tg[l], self.tg[l - 1],
                                                      f[1], f[2]))
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)
        self.ws_bytes = need
        self.aux = None  # second stream for the weight-gradient products (set by main unless --no-overlap)

    def step(self):
        tt = self.tt
        for l in range(1, self.L + 1):
            tt.tt_fc_forward(self.layers[l - 1], self.b, self.k, self.dt, self.tx[l - 1], self.tw[l - 1], self.tx[l],
                             self.forms[l - 1][0], self.x[l - 1], self.W[l - 1], self.x[l], self.ws)
        for l in range(self.L, 0, -1):
            tt.tt_fc_backward_overlapped(self.layers[l - 1], self.b, self.k, self.dt, self.tx[l - 1], self.tw[l - 1],
                                         self.tx[l], self.tg[l], self.tg[l - 1], self.forms[l - 1][1],
                                         self.forms[l - 1][2], self.x[l - 1], self.W[l - 1], self.x[l], self.g[l],
                                         self.g[l - 1], self.dW[l - 1], self.ws, aux_stream=self.aux)


class ConvLayerBench:
    """Device state of one convolution layer (forward + backward) under a tiling."""

    def __init__(self, cfg, tt, torch, split):
        import numpy as np
        self.cfg, self.tt = cfg, tt
        N, C, K, k = cfg.N, cfg.C, cfg.K, cfg.k
        self.lay = tt.layer("conv", "none", C, K, H=cfg.H, W=cfg.W, R=cfg.R, S=cfg.S, pad=cfg.pad)
        if split == "planner":
            p = tt.tt_plan_chain([self.lay], N, k)
            self.t = dict(X=p.x()[0], Y=p.x()[1], W=p.w()[0], dY=p.g()[1], dX=p.g()[0])
            self.f = [p.forms(1, o) for o in range(3)]
            self.plan_cost = p.cost
        elif split == "batch":
            self.t = dict(X="R" * k, Y="R" * k, W="r" * k, dY="R" * k, dX="R" * k)
            self.f = ["1" * k, "1" * k, "3" * k]
            self.plan_cost = None
        else:
            self.t = dict(X="r" * k, Y="C" * k, W="C" * k, dY="C" * k, dX="r" * k)
            self.f = ["2" * k, "3" * k, "2" * k]
            self.plan_cost = None
        tWs = self.t["W"].translate(str.maketrans("RC", "CR"))    # letters on the (K*R*S) x C storage matrix
        self.tWs = tWs
        dev = "cuda:0"

        def upload(M2, t):
            rows, cols = M2.shape
            sr, sc = tt.tt_shard_shape(rows, cols, t)
            out = []
            for s in range(1 << k):
                rb, cb = block_of(t, s)
                piece = np.ascontiguousarray(M2[rb * sr:(rb + 1) * sr, cb * sc:(cb + 1) * sc])
                out.append(torch.from_numpy(piece.view(np.int16)).to(dev).view(torch.bfloat16))
            return out

        def empty(rows, cols, t):
            sr, sc = tt.tt_shard_shape(rows, cols, t)
            return [torch.zeros((sr, sc), dtype=torch.bfloat16, device=dev) for _ in range(1 << k)]

        x = cfg.x().transpose(0, 2, 3, 1).reshape(N * cfg.H * cfg.W, C)
        w = cfg.weight().transpose(0, 2, 3, 1).reshape(K * cfg.R * cfg.S, C)
        g = cfg.grad_out().transpose(0, 2, 3, 1).reshape(N * cfg.P * cfg.Q, K)
        self.X, self.Wt, self.dY = upload(x, self.t["X"]), upload(w, tWs), upload(g, self.t["dY"])
        self.Y = empty(N * cfg.P * cfg.Q, K, self.t["Y"])
        self.dX = empty(N * cfg.H * cfg.W, C, self.t["dX"])
        self.dW = empty(K * cfg.R * cfg.S, C, tWs)
        t = self.t
        need = max(256, tt.tt_conv_workspace_bytes(self.lay, N, k, "bf16", tt.TT_OP_FWD, t["X"], t["W"], t["Y"], forms_a=self.f[0]),
                   tt.tt_conv_workspace_bytes(self.lay, N, k, "bf16", tt.TT_OP_DGRAD, t["X"], t["W"], t["Y"], t["dY"], t["dX"],
                                              self.f[1], self.f[2]))
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)
        self.tx, self.tg, self.tw = [t["X"], t["Y"]], [t["dX"], t["dY"]], [t["W"]]

    def step(self):
        tt, t, c = self.tt, self.t, self.cfg
        tt.tt_conv_forward(self.lay, c.N, c.k, "bf16", t["X"], t["W"], t["Y"], self.f[0], self.X, self.Wt, self.Y, self.ws)
        tt.tt_conv_backward(self.lay, c.N, c.k, "bf16", t["X"], t["W"], t["Y"], t["dY"], t["dX"], self.f[1], self.f[2],
                            self.X, self.Wt, self.Y, self.dY, self.dX, self.dW, self.ws)


def block_of(t, s):
    """(row block, column block) of shard s under tiling string t (host-side placement of synthetic inputs)."""
    k = len(t)
    rb = cb = 0
    for j, ch in enumerate(t):
        bit = (s >> (k - 1 - j)) & 1
        if ch == "R":
            rb = 2 * rb + bit
        elif ch == "C":
            cb = 2 * cb + bit
    return rb, cb


def aggregate(records):
    agg = {}
    for r in records:
        key = (r["kernel"], r["count"], r["d0"], r["d1"], r["d2"])
        a = agg.setdefault(key, dict(kernel=r["kernel"], count=r["count"], d0=r["d0"], d1=r["d1"], d2=r["d2"],
                                     bytes=r["bytes"], flops=r["flops"], ms=0.0, launches=0))
        a["ms"] += r["ms"]
        a["launches"] += 1
    return sorted(agg.values(), key=lambda a: -a["ms"])


def cpu_baseline(cfg, budget_gflop=250.0):
    """The oracle's plain-loop layer operators (oracle/layers_plain.c: fp64, untiled, OpenMP over output rows) timed on
    this host on a bounded sample of the same workload: whole fwd+bwd steps of the first layers of an FC chain until
    about budget_gflop is spent (the whole step where it fits), or a few images of a convolution layer."""
    import numpy as np
    from oracle import layers_plain as lp
    from synthetic import bf16_bits_to_f64
    cores = lp.threads()
    conv = (lambda a: bf16_bits_to_f64(a)) if cfg.dtype == "bf16" else (lambda a: a.astype(np.float64))
    if not hasattr(cfg, "widths"):
        ns = 1      # the seven-loop convolution is slow: one image is 11 GFLOP at conv4
        X, Wt, G = conv(cfg.x()[:ns]), conv(cfg.weight()), conv(cfg.grad_out()[:ns])
        t0 = time.perf_counter()
        lp.conv_forward(X, Wt, cfg.pad)
        lp.conv_dgrad(G, Wt, cfg.pad, cfg.H, cfg.W)
        lp.conv_wgrad(X, G, cfg.pad, cfg.R, cfg.S)
        dt = time.perf_counter() - t0
        fl = cfg.flops() * ns / cfg.N
        return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
                "sample": "fwd+dgrad+wgrad of %d of the %d images of %s, fp64 plain loops (%.1f GFLOP, %.2f s)" % (
                    ns, cfg.N, cfg.name, fl / 1e9, dt)}
    # layers 1..n: as many as fit the budget (at least one); each layer's forward and both backward products
    n, spent = 0, 0.0
    while n < cfg.n_layers and (n == 0 or spent + 6e-9 * cfg.batch * cfg.widths[n] * cfg.widths[n + 1] <= budget_gflop):
        spent += 6e-9 * cfg.batch * cfg.widths[n] * cfg.widths[n + 1]
        n += 1
    x = [conv(cfg.x0())]
    Ws = [conv(cfg.weight(l)) for l in range(1, n + 1)]
    g = conv(normal_like(cfg, n))
    t0 = time.perf_counter()
    for l in range(1, n + 1):
        x.append(lp.fc_forward(x[l - 1], Ws[l - 1], bool(cfg.act(l))))
    for l in range(n, 0, -1):
        g, _dw = lp.fc_backward(g, x[l - 1], Ws[l - 1], x[l], bool(cfg.act(l)))
    dt = time.perf_counter() - t0
    return {"value": spent * 1e9 / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": "untiled fwd+bwd of layers 1..%d of the %d of %s, fp64 plain loops (%.1f GFLOP, %.2f s)" % (
                n, cfg.n_layers, cfg.name, spent, dt)}


def normal_like(cfg, layer):
    """incoming gradient of `layer`'s output for the CPU sample: the workload's own dC/dx_L when the sample covers the
    whole chain, else a tensor of the same recipe at that layer's width"""
    if layer == cfg.n_layers:
        return cfg.grad_out()
    from synthetic import normal_f32, to_bf16_bits
    v = normal_f32(cfg.seed, 1, (cfg.batch, cfg.widths[layer]), 1.0)
    return to_bf16_bits(v) if cfg.dtype == "bf16" else v


def counted_cross_shard_elems(tt, cfg, chain, is_conv):
    """What the step's conversions and reductions really move between shards (flat count, block by block), next to the
    planner's cost, which is the paper's recursive model of the same traffic; the two are equal at one cut only."""
    if is_conv or any(f is None for layer_forms in chain.forms for f in layer_forms):
        return None
    return tt.tt_fc_chain_cross_elems(chain.layers, cfg.batch, cfg.k, chain.tx, chain.tg, chain.tw, chain.forms)


def shape_study(args, tt, torch):
    """Sec. 6.3 / Table 1 of the paper asked again on one MI355X: a 4-layer MLP with 8K x 8K weights, one step untiled
    (k = 0) against the same step cut into 8 shards under the planner's tiling, all shards on this GPU.  Same flops."""
    from synthetic.configs import FcChain
    paper = {512: (0.31, 0.19), 1024: (0.56, 0.39), 2048: (1.13, 0.73)}  # seconds per batch, the paper's GPU and fp32
    rows = []
    for b in (512, 1024, 2048):
        res = {}
        for k in (0, 3):
            cfg = FcChain("mlp4_8k", b, (8192,) * 5, k, "bf16", 0.01, 1006)
            chain = Chain(cfg, tt, torch)
            for _ in range(max(args.warmup, 1)):
                chain.step()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                chain.step()
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.steps
            res[k] = dict(ms=ms, tflops=cfg.flops() / (ms * 1e-3) / 1e12, tiling_w=chain.tw, tiling_x=chain.tx,
                          plan_cost_elems=chain.plan_cost)
            del chain, graph
            torch.cuda.empty_cache()
        rows.append({"batch": b, "untiled_ms": res[0]["ms"], "tiled_ms": res[3]["ms"],
                     "untiled_TFLOPs": res[0]["tflops"], "tiled_TFLOPs": res[3]["tflops"],
                     "tiled_over_untiled_time": res[3]["ms"] / res[0]["ms"], "tiling_w": res[3]["tiling_w"],
                     "tiling_x": res[3]["tiling_x"], "paper_untiled_s": paper[b][0], "paper_tiled_s": paper[b][1],
                     "paper_tiled_over_untiled_time": paper[b][1] / paper[b][0]})
    print(json.dumps({"metric": "fwd+bwd time per batch of a 4-layer 8K x 8K MLP: untiled vs cut into 8 shards on one GPU",
                      "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "dtype": "bf16",
                      "data": "synthetic", "config": {"workload": "shape_study: 8192->8192 x4, k=0 vs k=3 planner EXACT"},
                      "rows": rows}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all 2^k shards are simulated in one HBM); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_1805_04170_amd as tt
    from synthetic import CONFIGS
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    tt.binding.lib()
    torch.cuda.set_device(0)
    if args.workload == "shape_study":
        shape_study(args, tt, torch)
        return
    cfg = CONFIGS[args.workload]
    is_conv = not hasattr(cfg, "widths")
    if is_conv:
        chain = ConvLayerBench(cfg, tt, torch, args.conv_split)
    elif args.workload == "wide_mlp":
        # forced tiling: every tensor stored as a 4 x 4 grid; forward / dgrad split the reduction dimension twice
        L = cfg.n_layers
        chain = Chain(cfg, tt, torch, tilings=(["RRCC"] * (L + 1), ["RRCC"] * (L + 1), ["RRCC"] * L,
                                               [["3322", "2233", "1122"]] * L))
    else:
        chain = Chain(cfg, tt, torch)
    K, W = args.steps, args.warmup
    if not is_conv and args.overlap:
        chain.aux = torch.cuda.Stream()

    for _ in range(max(W, 1)):
        chain.step()
    torch.cuda.synchronize()

    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            chain.step()
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()

    run = graph.replay if graph is not None else chain.step
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / K
    tflops = cfg.flops() / (elapsed / K) / 1e12

    # per-kernel durations: eager pass on ONE stream (so that durations do not overlap), HIP events around every launch
    if not is_conv:
        chain.aux = None
    tt.tt_profile_begin()
    for _ in range(K):
        chain.step()
    records = tt.tt_profile_end()
    agg = aggregate(records)
    is_product = lambda a: a["kernel"].startswith("gemm") or a["kernel"].startswith("conv_")
    gemm_ms = sum(a["ms"] for a in agg if is_product(a)) / K
    conv_ms = sum(a["ms"] for a in agg if not is_product(a)) / K
    dom = agg[0]
    dom_ms = dom["ms"] / dom["launches"]
    key = "%s:%s:%dx%dx%d" % (args.workload, dom["kernel"], dom["d0"], dom["d1"], dom["d2"])
    # Which roof bounds the dominant kernel: the larger of its two lower bounds on time (flops at the dense bf16 MFMA
    # peak, algorithmic bytes at the HBM peak).  The batch-256 products have fewer than 312 flop per byte and sit under
    # the HBM roof; both fractions are reported.
    d_tflops = dom["flops"] / (dom_ms * 1e-3) / 1e12
    d_gbps = dom["bytes"] / (dom_ms * 1e-3) / 1e9
    hbm_bound = dom["bytes"] / (PEAK_HBM_GBS * 1e9) >= dom["flops"] / (PEAK_BF16_TFLOPS * 1e12)
    roofline = {
        "bound": "hbm" if hbm_bound else "mfma",
        "kernel": "%s count=%d M=%d N=%d K=%d" % (dom["kernel"], dom["count"], dom["d0"], dom["d1"], dom["d2"]),
        "achieved": d_gbps if hbm_bound else d_tflops, "peak": PEAK_HBM_GBS if hbm_bound else PEAK_BF16_TFLOPS,
        "unit": "GB/s" if hbm_bound else "TFLOP/s",
        "frac": d_gbps / PEAK_HBM_GBS if hbm_bound else d_tflops / PEAK_BF16_TFLOPS,
        "traffic": MEASURED_TRAFFIC_BYTES.get(key),
        "avg_ms": dom_ms, "launches": dom["launches"],
        "algorithmic_bytes": dom["bytes"], "flops": dom["flops"],
        "flop_per_byte": dom["flops"] / dom["bytes"] if dom["bytes"] else None,
        "mfma_TFLOPs": d_tflops, "mfma_frac": d_tflops / PEAK_BF16_TFLOPS,
        "hbm_GBps": d_gbps, "hbm_frac": d_gbps / PEAK_HBM_GBS,
    }
    kernels = [{"kernel": a["kernel"], "count": a["count"], "d": [a["d0"], a["d1"], a["d2"]], "launches_per_step": a["launches"] / K,
                "avg_ms": a["ms"] / a["launches"],
                "TFLOPs": (a["flops"] / (a["ms"] / a["launches"] * 1e-3) / 1e12) if a["flops"] else None,
                "GBps": a["bytes"] / (a["ms"] / a["launches"] * 1e-3) / 1e9} for a in agg]

    # partial-sum reduce headline: the reduction launch that moves the most bytes in this step
    red = [a for a in agg if a["kernel"] == "reduce"]
    reduce_line = None
    if red:
        rb = max(red, key=lambda a: a["bytes"])
        rb_ms = rb["ms"] / rb["launches"]
        reduce_line = {"rows": rb["d0"], "cols": rb["d1"], "bytes": rb["bytes"], "avg_ms": rb_ms,
                       "GBps": rb["bytes"] / (rb_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                       "frac": rb["bytes"] / (rb_ms * 1e-3) / 1e9 / PEAK_HBM_GBS}

    # retile headline: the largest tensor of the workload between two non-replicated tilings
    rows, cols = (cfg.widths[0], cfg.widths[1]) if not is_conv else (cfg.K * cfg.R * cfg.S, cfg.C)
    ka = cfg.k
    A, B = "R" * ka, "C" * ka
    esz = 2 if cfg.dtype == "bf16" else 4
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    sr, sc = tt.tt_shard_shape(rows, cols, A)
    src = [torch.zeros((sr, sc), dtype=tdt, device="cuda:0") for _ in range(1 << ka)]
    sr, sc = tt.tt_shard_shape(rows, cols, B)
    dst = [torch.zeros((sr, sc), dtype=tdt, device="cuda:0") for _ in range(1 << ka)]
    for _ in range(3):
        tt.tt_retile(dst, B, src, A, rows, cols, esz)
    # back-to-back launches between one pair of HIP events on the launch stream
    n_rt = 50
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(n_rt):
        tt.tt_retile(dst, B, src, A, rows, cols, esz)
    ev1.record()
    torch.cuda.synchronize()
    r_ms = ev0.elapsed_time(ev1) / n_rt
    r_bytes = 2 * rows * cols * esz
    r_gbs = r_bytes / (r_ms * 1e-3) / 1e9
    rrec = [{"bytes": r_bytes}]
    retile = {"tensor": "W_1 %dx%d %s" % (rows, cols, cfg.dtype), "from": A, "to": B, "bytes": rrec[0]["bytes"],
              "avg_ms": r_ms, "GBps": r_gbs, "peak": PEAK_HBM_GBS, "frac": r_gbs / PEAK_HBM_GBS}
    del src, dst

    try:
        counted = counted_cross_shard_elems(tt, cfg, chain, is_conv)
    except Exception:  # a report line must not take the measurement down
        counted = None
    out = {
        "metric": "tiled fwd+bwd TFLOP/s at VGG-16 FC shapes (% MFMA peak); retile GB/s (% HBM)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": ("%s: batch %d, %s, k=%d (%d shards), %s tiling" % (
            cfg.name, cfg.batch, "->".join(str(w) for w in cfg.widths), cfg.k, 1 << cfg.k,
            "planner EXACT" if chain.plan_cost is not None else "forced RRCC grid")) if not is_conv else (
            "%s: N=%d C=%d K=%d %dx%d %dx%d pad %d, k=%d (%d shards), %s split" % (
                cfg.name, cfg.N, cfg.C, cfg.K, cfg.H, cfg.W, cfg.R, cfg.S, cfg.pad, cfg.k, 1 << cfg.k, args.conv_split)),
            "tiling_x": chain.tx, "tiling_g": chain.tg, "tiling_w": chain.tw, "plan_cost_elems": chain.plan_cost,
            "counted_cross_shard_elems": counted,
            "timed": "hip graph replay" if graph is not None else "eager launches",
            "streams": 2 if (not is_conv and args.overlap) else 1},
        "frac_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "roofline": roofline,
        "retile": retile,
        "reduce": reduce_line,
        "breakdown_ms_per_step": {"products": gemm_ms, "conversions_and_reductions": conv_ms},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
