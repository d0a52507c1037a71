"""Pins for oracle/graph.py (tiling search on a general dataflow graph, Sec. 4.2-4.5).

The paper prints no value for a general graph, so the pins are: physical element counts by explicit index sets for
the element-wise and batch-only operators, equality with the layer-chain oracle (C code, pinned in
test_oracle_cost.py) on chains written as graphs - random tilings, optima, convolutions -, closed forms, and Theorem 1."""
import itertools
import random

import pytest

from oracle import cost as oc
from oracle import graph as og
from oracle import tiling as tl

L2 = {"R": 0, "C": 1, "r": "r"}


def held(rows, cols, letter, d):
    name = {0: "R", 1: "C", "r": "r"}[letter]
    rs, cs = tl.shard_slices(rows, cols, name, d)
    return {(i, j) for i in range(rs.start, rs.stop) for j in range(cs.start, cs.stop)}


def test_elementwise_one_cut_is_ghost_minus_held():
    # c = a + b on 4 x 6 matrices: for each aligned dimension count what every device fetches for its inputs and
    # what has to travel so that the output ends up stored as asked; the operator takes the cheaper dimension
    rows, cols = 4, 6
    tensors = [{"shape": (rows, cols), "same_as": None} for _ in range(3)]
    ops = [{"kind": "elementwise", "ins": [0, 1], "out": 2}]
    for la, lb, lc in itertools.product([0, 1, "r"], repeat=3):
        best = None
        for dim in (0, 1):
            cnt = 0
            for d in range(2):
                cnt += len(held(rows, cols, dim, d) - held(rows, cols, la, d))
                cnt += len(held(rows, cols, dim, d) - held(rows, cols, lb, d))
                cnt += len(held(rows, cols, lc, d) - held(rows, cols, dim, d))
            best = cnt if best is None else min(best, cnt)
        assert og.graph_cost(tensors, ops, 1, {0: (la,), 1: (lb,), 2: (lc,)}) == best


def test_batch_only_operator_forces_the_batch_cut():
    # any operator that is neither a product nor element-wise runs data parallel (Sec. 4.5)
    tensors = [{"shape": (8, 10), "same_as": None}, {"shape": (8, 1), "same_as": None}, {"shape": (8, 1), "same_as": None}]
    ops = [{"kind": "batch", "ins": [0, 1], "out": 2}]
    assert og.graph_cost(tensors, ops, 1, {0: (0,), 1: (0,), 2: (0,)}) == 0
    assert og.graph_cost(tensors, ops, 1, {0: (1,), 1: (0,), 2: (0,)}) == 40          # column cut -> row cut: A / 2
    assert og.graph_cost(tensors, ops, 1, {0: ("r",), 1: ("r",), 2: ("r",)}) == 8      # only the output is gathered
    # second cut works on the tiles of the first and weighs double (Theorem 1)
    assert og.graph_cost(tensors, ops, 2, {0: (0, 1), 1: (0, 0), 2: (0, 0)}) == 2 * (40 // 2)
    # a batch of 2 cannot be cut twice
    small = [{"shape": (2, 4), "same_as": None}, {"shape": (2, 4), "same_as": None}]
    assert og.graph_cost(small, [{"kind": "batch", "ins": [0], "out": 1}], 2, {0: ("r", "r"), 1: ("r", "r")}) == og.INF


def test_sample_channel_operator_is_ghost_minus_held():
    # a per-(sample, channel) operator with a narrower output (4 x 6 -> 4 x 2: three columns per channel pooled into
    # one): device d needs the input block of its aligned cut and hands over what the stored output tiling asks for
    tensors = [{"shape": (4, 6), "same_as": None}, {"shape": (4, 2), "same_as": None}]
    ops = [{"kind": "sample_channel", "ins": [0], "out": 1}]
    for li, lo in itertools.product([0, 1, "r"], repeat=2):
        best = None
        for dim in (0, 1):
            cnt = 0
            for d in range(2):
                cnt += len(held(4, 6, dim, d) - held(4, 6, li, d))
                cnt += len(held(4, 2, lo, d) - held(4, 2, dim, d))
            best = cnt if best is None else min(best, cnt)
        assert og.graph_cost(tensors, ops, 1, {0: (li,), 1: (lo,)}) == best
    # one channel left: only the sample cut remains
    one = [{"shape": (4, 3), "same_as": None}, {"shape": (4, 1), "same_as": None}]
    assert og.graph_cost(one, ops, 1, {0: (0,), 1: (0,)}) == 0
    assert [f[2] for f in og.forms_of(ops[0], one)] == [4, 1]


def chain_tilings(idx, x, g, w):
    t = {}
    for l, s in enumerate(x):
        t[idx["x"][l]] = tuple(L2[c] for c in s)
    for l, s in enumerate(g):
        t[idx["g"][l]] = tuple(L2[c] for c in s)
    for l, s in enumerate(w):
        t[idx["w"][l]] = tuple(L2[c] for c in s)
    return t


@pytest.mark.parametrize("k", [1, 2, 3])
def test_chain_written_as_graph_prices_like_the_chain_oracle(k):
    rnd = random.Random(100 + k)
    for trial in range(40):
        L = rnd.choice([1, 2, 3])
        batch = rnd.choice([8, 12, 16, 6])
        widths = [rnd.choice([8, 16, 24, 10, 4]) for _ in range(L + 1)]
        tensors, ops, idx = og.mlp_graph(batch, widths)
        chain = oc.make_chain(batch, widths)
        x = ["".join(rnd.choice("RCr") for _ in range(k)) for _ in range(L + 1)]
        g = ["".join(rnd.choice("RCr") for _ in range(k)) for _ in range(L + 1)]
        w = ["".join(rnd.choice("RCr") for _ in range(k)) for _ in range(L)]
        want = oc.chain_cost(chain, k, x, g, w)[0]
        got = og.graph_cost(tensors, ops, k, chain_tilings(idx, x, g, w))
        assert (got == og.INF and want == oc.INF) or got == want, (batch, widths, x, g, w)


def test_chain_optimum_equals_the_chain_oracles():
    for batch, widths, k in [(8, [6, 4], 1), (8, [6, 4], 2), (4, [8, 12, 6], 1), (12, [4, 4], 2)]:
        tensors, ops, idx = og.mlp_graph(batch, widths)
        want = oc.bruteforce(oc.make_chain(batch, widths), k)[0]
        got, arg = og.bruteforce(tensors, ops, k)
        assert got == want
        assert og.graph_cost(tensors, ops, k, arg) == got


def test_data_parallel_closed_form_with_residual_adds():
    # x1 = x0 W1 ; x2 = x1 W2 + x0 (a residual block) with its backward pass; every activation cut along the batch,
    # weights replicated: the only traffic is the all-reduce of the two weight gradients; a replicated tensor keeps its
    # size from cut to cut, so cut j moves 2 |W| per weight in each of its 2^j groups: 2 |W| (2^k - 1) in all
    # (batch much larger than the layers, or a deep cut finds a model-parallel form cheaper for the small tiles)
    b, n = 64, 6
    T = lambda shape, same=None: {"shape": shape, "same_as": same}
    names = ["x0", "x1", "h2", "x2", "g2", "gh2", "g1", "g0a", "g0", "W1", "W2", "dW1", "dW2"]
    ix = {s: i for i, s in enumerate(names)}
    tensors = [T((b, n)) for _ in range(9)] + [T((n, n)), T((n, n)), T((n, n), ix["W1"]), T((n, n), ix["W2"])]
    ops = [og.matmul(ix["x0"], ix["W1"], ix["x1"]), og.matmul(ix["x1"], ix["W2"], ix["h2"]),
           {"kind": "elementwise", "ins": [ix["h2"], ix["x0"]], "out": ix["x2"]},
           {"kind": "elementwise", "ins": [ix["g2"]], "out": ix["gh2"]},
           og.matmul(ix["gh2"], ix["W2"], ix["g1"], tb=True), og.matmul(ix["x1"], ix["gh2"], ix["dW2"], ta=True),
           og.matmul(ix["g1"], ix["W1"], ix["g0a"], tb=True), og.matmul(ix["x0"], ix["g1"], ix["dW1"], ta=True),
           {"kind": "elementwise", "ins": [ix["g0a"], ix["g2"]], "out": ix["g0"]}]
    for k in (1, 2, 3):
        t = {i: (0,) * k for i in range(9)}
        t[ix["W1"]] = t[ix["W2"]] = ("r",) * k
        assert og.graph_cost(tensors, ops, k, t) == 2 * (2 * n * n) * (2 ** k - 1)


def test_convolution_as_contraction_prices_like_the_chain_oracle():
    # X[N,C,H,W] * W[K,C,R,S]: image and filter extents only multiply the areas (Sec. 4.5)
    rnd = random.Random(7)
    N, H, R = 8, 5, 3
    chans = [4, 8, 6]
    for k in (1, 2):
        chain = oc.make_chain(N, chans, xmult=[H * H] * 3, wmult=[1, R * R, R * R])
        T = lambda shape, same=None: {"shape": shape, "same_as": same}
        tensors, ops = [], []
        x = [len(tensors) + i for i in range(3)]; tensors += [T((N, c, H, H)) for c in chans]
        g = [len(tensors) + i for i in range(3)]; tensors += [T((N, c, H, H)) for c in chans]
        w = [len(tensors) + i for i in range(2)]; tensors += [T((chans[l + 1], chans[l], R, R)) for l in range(2)]
        dw = [len(tensors) + i for i in range(2)]; tensors += [T((chans[l + 1], chans[l], R, R), w[l]) for l in range(2)]
        for l in range(2):
            ops.append({"kind": "contract", "ins": [x[l], w[l]], "out": x[l + 1], "m": (0, 0), "n": (0, 1), "k": (1, 1)})
            ops.append({"kind": "contract", "ins": [g[l + 1], w[l]], "out": g[l], "m": (0, 0), "n": (1, 1), "k": (1, 0)})
            ops.append({"kind": "contract", "ins": [x[l], g[l + 1]], "out": dw[l], "m": (1, 1), "n": (1, 0), "k": (0, 0)})
        for trial in range(30):
            xs = ["".join(rnd.choice("RCr") for _ in range(k)) for _ in range(3)]
            gs = ["".join(rnd.choice("RCr") for _ in range(k)) for _ in range(3)]
            ws = ["".join(rnd.choice("RCr") for _ in range(k)) for _ in range(2)]
            want = oc.chain_cost(chain, k, xs, gs, ws)[0]
            t = {}
            for l in range(3):
                t[x[l]] = tuple(L2[c] for c in xs[l])       # activations: R = batch (dim 0), C = channel (dim 1)
                t[g[l]] = tuple(L2[c] for c in gs[l])
            for l in range(2):                                # filters [K,C,R,S]: the chain's R = in-channel = dim 1
                t[w[l]] = tuple({"R": 1, "C": 0, "r": "r"}[c] for c in ws[l])
            got = og.graph_cost(tensors, ops, k, t)
            assert (got == og.INF and want == oc.INF) or got == want, (xs, gs, ws)


def test_greedy_checker_accepts_a_greedy_plan_and_rejects_others():
    batch, widths, k = 8, [8, 8], 2
    tensors, ops, idx = og.mlp_graph(batch, widths)
    cost, x, g, w, delta = oc.recursive(oc.make_chain(batch, widths), k)
    t = chain_tilings(idx, x, g, w)
    forms = [list(og.op_cost(op, tensors, t, k, want_forms=True)[1]) for op in ops]
    # the chain oracle's greedy plan, re-priced cut by cut, is a valid run of Algorithm 1 ...
    if og.greedy_is_valid(tensors, ops, k, t, forms, delta):
        assert sum(d << j for j, d in enumerate(delta)) == cost
    else:  # ... unless the per-operator form sequence that prices it best is not the level-wise cheapest one
        assert og.graph_cost(tensors, ops, k, t) <= cost
    # a plan whose first cut is not a one-cut optimum is rejected
    bad = dict(t)
    bad[idx["x"][0]] = (1, 1)
    bad[idx["w"][0]] = (1, 0)
    assert not og.greedy_is_valid(tensors, ops, k, bad, forms, delta)
