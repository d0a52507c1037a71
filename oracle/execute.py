"""Tiled execution of one matrix product, by the three-phase scheme of
Sec. 4.2.1 / Sec. 5.2: convert inputs to an aligned tiling, multiply locally on
each of the 2^k shards, convert (and, for the third aligned form, reduce) the
outputs.  fp64 throughout.

A form sequence is a string over "123", one aligned form per cut:
  form 1:  X:R  Y:r  ->  Z:R      (rows of X split;   M-split)
  form 2:  X:r  Y:C  ->  Z:C      (columns of Y split; N-split)
  form 3:  X:C  Y:R  ->  Z:red    (inner dimension split; partial sums)
"""
import numpy as np

from . import tiling as tl

ALIGNED_X = {"1": "R", "2": "r", "3": "C"}
ALIGNED_Y = {"1": "r", "2": "C", "3": "R"}


def aligned_tilings(forms):
    """(a_X, a_Y) for a form sequence."""
    return ("".join(ALIGNED_X[f] for f in forms), "".join(ALIGNED_Y[f] for f in forms))


def output_grid_tiling(forms):
    """Tiling of the temporary outputs seen as a grid: form 1 -> R, form 2 -> C,
    form 3 -> 'r' positions that hold *different partial sums* (not replicas)."""
    return "".join({"1": "R", "2": "C", "3": "r"}[f] for f in forms)


def transpose_tiling(t):
    return t.translate(str.maketrans("RC", "CR"))


def shard_products(X, Y, forms):
    """Phase 2: the 2^k local products on aligned tiles."""
    aX, aY = aligned_tilings(forms)
    Xs, Ys = tl.tile(X, aX), tl.tile(Y, aY)
    return [np.matmul(a.astype(np.float64), b.astype(np.float64)) for a, b in zip(Xs, Ys)]


def assemble(partials, forms, M, N):
    """Concatenate over the form-1/2 cuts and sum over the form-3 cuts."""
    grid = output_grid_tiling(forms)
    Z = np.zeros((M, N))
    for s, part in enumerate(partials):
        Z[tl.shard_slices(M, N, grid, s)] += part
    return Z


def reduce_to(partials, forms, tZ, M, N, relu=False):
    """Phase 3 with a reduction: sum partials, then the element-wise function,
    then cut into the stored tiling tZ."""
    Z = assemble(partials, forms, M, N)
    if relu:
        Z = np.maximum(Z, 0.0)
    return tl.tile(Z, tZ)


def tiled_matmul(X_shards, tX, Y_shards, tY, tZ, forms, M, K, N, relu=False):
    """All three phases from stored shards to stored shards."""
    aX, aY = aligned_tilings(forms)
    Xa = tl.retile(X_shards, tX, aX, M, K)
    Ya = tl.retile(Y_shards, tY, aY, K, N)
    parts = [np.matmul(a.astype(np.float64), b.astype(np.float64)) for a, b in zip(Xa, Ya)]
    return reduce_to(parts, forms, tZ, M, N, relu)


def forms_feasible(forms, M, K, N):
    return (M % (1 << forms.count("1")) == 0 and N % (1 << forms.count("2")) == 0
            and K % (1 << forms.count("3")) == 0)
