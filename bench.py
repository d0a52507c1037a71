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

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def measured_traffic(workload, rec):
    """HBM bytes per launch (read + written) of one launch shape, as the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
    this workload measured them (profiles/hbm_traffic.json, written by profile_summary.py from those runs; the counters
    are scaled by what they read for a retile of known size).  None if that shape was not measured."""
    try:
        with open(TRAFFIC_FILE) as fh:
            table = json.load(fh)
    except (OSError, ValueError):
        return None
    key = "%s count=%d %dx%dx%d" % (rec["kernel"], rec["count"], rec["d0"], rec["d1"], rec["d2"])
    hit = table.get(workload, {}).get("launches", {}).get(key)
    return None if hit is None else int(hit["read_bytes"] + hit["write_bytes"])


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vgg16_fc",
                    choices=["vgg16_fc", "alexnet_fc", "wide_mlp", "wide_mlp_f3", "tiny_mlp", "vgg16_conv4", "shape_study"])
    ap.add_argument("--conv-split", default="planner", choices=["planner", "batch", "out_channel"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="measure only --workload; default: the headline workload plus one block per other configuration")
    ap.add_argument("--other-steps", type=int, default=10, help="timed steps of each of the other configurations")
    ap.add_argument("--launch-log", default=None,
                    help="write the launches of one step (kernel, shape, algorithmic bytes and flops, in launch order) to "
                         "this JSON file: what profile_summary.py needs to attribute profiler dispatches to launches")
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
    """launch shapes of a profiled pass, most time first (time summed over the launches of a shape)"""
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


def shape_study(args, tt, torch, steps=None):
    """Sec. 6.3 / Table 1 of the paper asked again on one MI355X: a 4-layer MLP with 8K x 8K weights, one step untiled
    (k = 0) against the same step cut into 8 shards under the planner's tiling, all shards on this GPU.  Same flops."""
    from synthetic.configs import FcChain
    paper = {512: (0.31, 0.19), 1024: (0.56, 0.39), 2048: (1.13, 0.73)}  # seconds per batch, the paper's GPU and fp32
    rows = []
    steps = steps or args.steps
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
            for _ in range(steps):
                graph.replay()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
            res[k] = dict(ms=ms, tflops=cfg.flops() / (ms * 1e-3) / 1e12, tiling_w=chain.tw, tiling_x=chain.tx,
                          plan_cost_elems=chain.plan_cost)
            del chain, graph
            torch.cuda.empty_cache()
        rows.append({"batch": b, "untiled_ms": res[0]["ms"], "tiled_ms": res[3]["ms"],
                     "untiled_TFLOPs": res[0]["tflops"], "tiled_TFLOPs": res[3]["tflops"],
                     "tiled_over_untiled_time": res[3]["ms"] / res[0]["ms"], "tiling_w": res[3]["tiling_w"],
                     "tiling_x": res[3]["tiling_x"], "paper_untiled_s": paper[b][0], "paper_tiled_s": paper[b][1],
                     "paper_tiled_over_untiled_time": paper[b][1] / paper[b][0]})
    return {"metric": "fwd+bwd time per batch of a 4-layer 8K x 8K MLP: untiled vs cut into 8 shards on one GPU",
            "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": args.warmup, "dtype": "bf16",
            "data": "synthetic", "config": {"workload": "shape_study: 8192->8192 x4, k=0 vs k=3 planner EXACT"},
            "rows": rows}


def build_workload(name, args, tt, torch, conv_split):
    """(cfg, device state, description of the tiling) of one workload"""
    from synthetic import CONFIGS
    cfg = CONFIGS["wide_mlp" if name == "wide_mlp_f3" else name]
    if not hasattr(cfg, "widths"):
        return cfg, ConvLayerBench(cfg, tt, torch, conv_split), "%s split" % conv_split
    L = cfg.n_layers
    if name == "wide_mlp":
        # forced tiling: every tensor stored as a 4 x 4 grid; forward / dgrad split the reduction dimension twice
        return cfg, Chain(cfg, tt, torch, tilings=(["RRCC"] * (L + 1), ["RRCC"] * (L + 1), ["RRCC"] * L,
                                                   [["3322", "2233", "1122"]] * L)), "forced RRCC grid"
    if name == "wide_mlp_f3":
        # all four cuts on the reduction dimension of the forward product: 16 partial sums of 512 x 8192 fp32 per layer
        return cfg, Chain(cfg, tt, torch, tilings=(["CCCC"] * (L + 1), ["rrrr"] * (L + 1), ["RRRR"] * L,
                                                   [["3333", "2222", "1111"]] * L)), "forced x:CCCC W:RRRR, forward forms F3 x 4"
    return cfg, Chain(cfg, tt, torch), "planner EXACT"


def kernel_line(a, steps):
    ms = a["ms"] / a["launches"]
    tf = a["flops"] / (ms * 1e-3) / 1e12 if a["flops"] else None
    gb = a["bytes"] / (ms * 1e-3) / 1e9
    return {"kernel": a["kernel"], "count": a["count"], "d": [a["d0"], a["d1"], a["d2"]], "launches_per_step": a["launches"] / steps,
            "avg_ms": ms, "TFLOPs": tf, "GBps": gb}


def roofline_of(workload, a):
    """Which roof bounds a launch shape: the larger of its two lower bounds on time (flops at the dense bf16 MFMA peak,
    algorithmic bytes at the HBM peak); both fractions are reported next to it."""
    ms = a["ms"] / a["launches"]
    tf = a["flops"] / (ms * 1e-3) / 1e12
    gb = a["bytes"] / (ms * 1e-3) / 1e9
    hbm_bound = a["bytes"] / (PEAK_HBM_GBS * 1e9) >= a["flops"] / (PEAK_BF16_TFLOPS * 1e12)
    return {
        "bound": "hbm" if hbm_bound else "mfma",
        "kernel": "%s count=%d M=%d N=%d K=%d" % (a["kernel"], a["count"], a["d0"], a["d1"], a["d2"]),
        "achieved": gb if hbm_bound else tf, "peak": PEAK_HBM_GBS if hbm_bound else PEAK_BF16_TFLOPS,
        "unit": "GB/s" if hbm_bound else "TFLOP/s",
        "frac": gb / PEAK_HBM_GBS if hbm_bound else tf / PEAK_BF16_TFLOPS,
        "traffic": measured_traffic(workload, a),
        "avg_ms": ms, "launches": a["launches"],
        "algorithmic_bytes": a["bytes"], "flops": a["flops"],
        "flop_per_byte": a["flops"] / a["bytes"] if a["bytes"] else None,
        "mfma_TFLOPs": tf, "mfma_frac": tf / PEAK_BF16_TFLOPS, "hbm_GBps": gb, "hbm_frac": gb / PEAK_HBM_GBS,
    }


def hbm_line(a):
    ms = a["ms"] / a["launches"]
    gb = a["bytes"] / (ms * 1e-3) / 1e9
    return {"kernel": a["kernel"], "rows": a["d0"], "cols": a["d1"], "bytes": a["bytes"], "avg_ms": ms, "GBps": gb,
            "peak": PEAK_HBM_GBS, "frac": gb / PEAK_HBM_GBS}


def measure(name, args, tt, torch, steps, warmup, conv_split="planner", with_cpu=True, full=False):
    """One workload: K timed steps (HIP graph replay unless --no-graph), then an eager pass of the same K steps with every
    kernel bracketed by HIP events on the launch stream.  Returns the report block of the workload."""
    cfg, chain, tiling_desc = build_workload(name, args, tt, torch, conv_split)
    is_conv = not hasattr(cfg, "widths")
    if not is_conv and args.overlap:
        chain.aux = torch.cuda.Stream()
    for _ in range(max(warmup, 1)):
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
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / steps
    flops = cfg.flops()
    tflops = flops / (elapsed / steps) / 1e12

    # per-kernel durations: eager pass on ONE stream (so that durations do not overlap), HIP events around every launch
    if not is_conv:
        chain.aux = None
    tt.tt_profile_begin()
    for _ in range(steps):
        chain.step()
    records = tt.tt_profile_end()
    agg = aggregate(records)
    is_product = lambda a: a["kernel"].startswith("gemm") or a["kernel"].startswith("conv_")
    products = [a for a in agg if is_product(a)]
    others = [a for a in agg if not is_product(a)]
    gemm_ms = sum(a["ms"] for a in products) / steps
    conv_ms = sum(a["ms"] for a in others) / steps
    # the dominant kernel: the product launch shape with the most time per step; the conversions and reductions are
    # reported separately (the one that moves the most bytes of each kind)
    wl_key = name if not is_conv else "%s_%s" % (name, conv_split)
    dom = products[0]
    out = {
        "workload": ("%s: batch %d, %s, k=%d (%d shards), %s" % (
            name, cfg.batch, "->".join(str(w) for w in cfg.widths) if len(cfg.widths) < 6 else "%d x (%d->%d)" % (
                cfg.n_layers, cfg.widths[0], cfg.widths[1]), cfg.k, 1 << cfg.k, tiling_desc)) if not is_conv else (
            "%s: N=%d C=%d K=%d %dx%d %dx%d pad %d, k=%d (%d shards), %s" % (
                name, cfg.N, cfg.C, cfg.K, cfg.H, cfg.W, cfg.R, cfg.S, cfg.pad, cfg.k, 1 << cfg.k, tiling_desc)),
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "ms_per_step": ms_per_step, "TFLOPs": tflops, "frac_mfma_peak": tflops / PEAK_BF16_TFLOPS, "steps": steps,
        "timed": "hip graph replay" if graph is not None else "eager launches",
        "tiling_x": chain.tx, "tiling_g": chain.tg, "tiling_w": chain.tw, "plan_cost_elems": chain.plan_cost,
        "roofline": roofline_of(wl_key, dom),
        "breakdown_ms_per_step": {"products": gemm_ms, "conversions_and_reductions": conv_ms},
    }
    red = [a for a in others if a["kernel"] == "reduce"]
    cvt = [a for a in others if a["kernel"] in ("convert", "gate")]
    out["reduce"] = hbm_line(max(red, key=lambda a: a["bytes"])) if red else None
    out["conversion"] = hbm_line(max(cvt, key=lambda a: a["bytes"])) if cvt else None
    if full:
        out["kernels"] = [kernel_line(a, steps) for a in agg]
        try:
            out["counted_cross_shard_elems"] = counted_cross_shard_elems(tt, cfg, chain, is_conv)
        except Exception:  # a report line must not take the measurement down
            out["counted_cross_shard_elems"] = None
        out["streams"] = 2 if (not is_conv and args.overlap) else 1
        out["_launches"] = (wl_key, records[:len(records) // steps])
    else:
        out["products"] = [kernel_line(a, steps) for a in products[:3]]
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg)
    del chain, graph
    torch.cuda.empty_cache()
    return out, cfg


def retile_headline(cfg, tt, torch):
    """retile of the workload's largest tensor between two non-replicated tilings: back-to-back launches between one pair
    of HIP events on the launch stream"""
    is_conv = not hasattr(cfg, "widths")
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
    return {"tensor": "W_1 %dx%d %s" % (rows, cols, cfg.dtype), "from": A, "to": B, "bytes": r_bytes,
            "avg_ms": r_ms, "GBps": r_gbs, "peak": PEAK_HBM_GBS, "frac": r_gbs / PEAK_HBM_GBS}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all 2^k shards are simulated in one HBM); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_1805_04170_amd as tt
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    tt.binding.lib()
    torch.cuda.set_device(0)
    if args.workload == "shape_study":
        print(json.dumps(shape_study(args, tt, torch)))
        return
    K, W = args.steps, args.warmup
    head, cfg = measure(args.workload, args, tt, torch, K, W, args.conv_split, with_cpu=not args.no_cpu_baseline, full=True)
    retile = retile_headline(cfg, tt, torch)
    wl_key, step_launches = head.pop("_launches")
    if args.launch_log:
        with open(args.launch_log, "w") as fh:
            json.dump({"workload": wl_key, "launches": step_launches, "retile_bytes_each_way": retile["bytes"] // 2}, fh)
    out = {
        "metric": "tiled fwd+bwd TFLOP/s at VGG-16 FC shapes (% MFMA peak); retile GB/s (% HBM)",
        "value": head["TFLOPs"], "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"], "tiling_x": head["tiling_x"], "tiling_g": head["tiling_g"],
                   "tiling_w": head["tiling_w"], "plan_cost_elems": head["plan_cost_elems"],
                   "counted_cross_shard_elems": head["counted_cross_shard_elems"], "timed": head["timed"],
                   "streams": head["streams"]},
        "frac_mfma_peak": head["frac_mfma_peak"],
        "roofline": head["roofline"],
        "retile": retile,
        "reduce": head["reduce"],
        "conversion": head["conversion"],
        "breakdown_ms_per_step": head["breakdown_ms_per_step"],
        "kernels": head["kernels"],
    }
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    if not args.headline_only and args.workload == "vgg16_fc":
        # the other configurations, one compact block each (fewer timed steps; each with its own CPU sample)
        others = []
        for name, split in (("alexnet_fc", None), ("wide_mlp", None), ("wide_mlp_f3", None), ("vgg16_conv4", "planner"),
                            ("vgg16_conv4", "batch"), ("vgg16_conv4", "out_channel"), ("tiny_mlp", None)):
            cpu = not args.no_cpu_baseline and name != "wide_mlp_f3" and split in (None, "planner")
            blk, _ = measure(name, args, tt, torch, args.other_steps, min(W, 2), split or "planner", with_cpu=cpu)
            others.append(blk)
        out["others"] = others
        study = shape_study(args, tt, torch, steps=max(3, args.other_steps // 2))
        out["shape_study"] = {"workload": study["config"]["workload"], "rows": study["rows"]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
