"""Pins for oracle/execute.py: the aligned forms are correct, non-redundant and
balanced block products (Sec. 4.2.1), and the three phases reproduce the untiled product."""
import itertools

import numpy as np
import pytest

from oracle import execute as ex
from oracle import tiling as tl


def all_forms(k):
    return ["".join(p) for p in itertools.product("123", repeat=k)]


def test_aligned_letters_as_in_paper():
    # Sec. 4.2.1: form 1 = row-partitioned x replicated -> row; form 2 = replicated x column -> column;
    # form 3 = column x row -> partial sums
    assert ex.aligned_tilings("1") == ("R", "r")
    assert ex.aligned_tilings("2") == ("r", "C")
    assert ex.aligned_tilings("3") == ("C", "R")
    assert ex.aligned_tilings("132") == ("RCr", "rRC")


@pytest.mark.parametrize("k", [1, 2, 3])
def test_concat_and_sum_reproduce_untiled(k):
    rng = np.random.default_rng(10 + k)
    M, K, N = 8, 16, 24
    X = rng.integers(-4, 5, size=(M, K)).astype(np.float64)     # small integers: exact sums in any order
    Y = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    Z = X @ Y
    for f in all_forms(k):
        parts = ex.shard_products(X, Y, f)
        assert len(parts) == 2 ** k                                # balanced: one product per device
        assert np.array_equal(ex.assemble(parts, f, M, N), Z)     # correct
        shapes = {p.shape for p in parts}
        assert shapes == {(M >> f.count("1"), N >> f.count("2"))}


@pytest.mark.parametrize("forms", ["1", "2", "3", "13", "32", "231", "333", "123"])
def test_every_scalar_product_covered_once(forms):
    # non-redundant: each (m, k, n) term of the sum is computed by exactly one shard
    M, K, N = 8, 8, 8
    aX, aY = ex.aligned_tilings(forms)
    cover = np.zeros((M, K, N), dtype=np.int64)
    for s in range(2 ** len(forms)):
        mr, kc = tl.shard_slices(M, K, aX, s)
        kr, nc = tl.shard_slices(K, N, aY, s)
        assert (kc.start, kc.stop) == (kr.start, kr.stop)          # inner ranges agree: a valid block product
        cover[mr, kc, nc] += 1
    assert (cover == 1).all()


def test_three_phases_from_any_stored_tiling():
    rng = np.random.default_rng(3)
    M, K, N = 8, 8, 16
    X = rng.integers(-3, 4, size=(M, K)).astype(np.float64)
    Y = rng.integers(-3, 4, size=(K, N)).astype(np.float64)
    Z = X @ Y
    k = 2
    tilings = tl.all_tilings(k)
    for tX, tY, tZ, f in itertools.product(tilings[::2], tilings[1::2], tilings[::3], all_forms(k)):
        out = ex.tiled_matmul(tl.tile(X, tX), tX, tl.tile(Y, tY), tY, tZ, f, M, K, N)
        assert np.array_equal(tl.untile(out, tZ, M, N), Z)


def test_relu_after_the_sum():
    # partial sums of opposite sign: ReLU of the sum is not the sum of ReLUs
    X = np.array([[1.0, -2.0]]); Y = np.array([[1.0], [1.0]])
    parts = ex.shard_products(X, Y, "3")
    assert [p[0, 0] for p in parts] == [1.0, -2.0]
    out = ex.reduce_to(parts, "3", "r", 1, 1, relu=True)
    assert out[0][0, 0] == 0.0 and out[1][0, 0] == 0.0


def test_named_tilings_run_without_conversion(golden_loader):
    # Sec. 4.1: under T_data / T_model / T_hybrid the forward product finds its operands aligned
    g = golden_loader("paper_tilings.txt")
    for name, fwd_forms in [("T_data", "1"), ("T_model", "3"), ("T_hybrid", "13")]:
        tW, tAct, _ = g[name]
        aX, aY = ex.aligned_tilings(fwd_forms)
        assert (aX, aY) == (tAct, tW)


def test_transpose_tiling():
    assert ex.transpose_tiling("RCr") == "CRr"
    T = np.arange(32).reshape(4, 8)
    for t in tl.all_tilings(2):
        a = [s.T for s in tl.tile(T, t)]
        b = tl.tile(T.T, ex.transpose_tiling(t))
        assert all(np.array_equal(x, y) for x, y in zip(a, b))
