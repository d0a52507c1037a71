"""k-cut tiling geometry (Sec. 4.1 Def. 1; flattening theorem, Sec. 4.4).

A k-cut tiling of a matrix is a string over {R, C, r}: cut j (j = 0 is the
first, outermost cut) halves the rows (R), halves the columns (C) or
replicates (r).  Shard s in [0, 2^k) chooses side bit_j(s) at cut j, with the
outermost cut as the most significant bit.  By the flattening theorem the
2^k shards form a regular grid: 2^kR row blocks by 2^kC column blocks, each
held 2^kr times.
"""
import itertools

import numpy as np

LETTERS = "RCr"


def all_tilings(k):
    """T^k of Def. 1 as strings, in the order the definition composes them."""
    return ["".join(p) for p in itertools.product(LETTERS, repeat=k)]


def flattened(t):
    """(kR, kC, kr) of a tiling: its class under the flattening theorem."""
    return (t.count("R"), t.count("C"), t.count("r"))


def bit(s, j, k):
    return (s >> (k - 1 - j)) & 1


def block_index(t, s):
    """(row block, col block) held by shard s: the side bits at the R cuts
    (resp. C cuts) read outermost-first as a binary number."""
    k = len(t)
    rho = gam = 0
    for j, letter in enumerate(t):
        b = bit(s, j, k)
        if letter == "R":
            rho = 2 * rho + b
        elif letter == "C":
            gam = 2 * gam + b
        elif letter != "r":
            raise ValueError("bad tiling letter %r" % letter)
    return rho, gam


def shard_shape(rows, cols, t):
    kR, kC, _ = flattened(t)
    if rows % (1 << kR) or cols % (1 << kC):
        raise ValueError("uneven tiling %s of %dx%d" % (t, rows, cols))
    return rows >> kR, cols >> kC


def shard_slices(rows, cols, t, s):
    sr, sc = shard_shape(rows, cols, t)
    rho, gam = block_index(t, s)
    return slice(rho * sr, (rho + 1) * sr), slice(gam * sc, (gam + 1) * sc)


def tile(T, t):
    """Split a full 2-D array into its 2^k shards (copies)."""
    rows, cols = T.shape
    return [np.ascontiguousarray(T[shard_slices(rows, cols, t, s)]) for s in range(1 << len(t))]


def untile(shards, t, rows, cols):
    """Reassemble the full array; every replica must be bit-identical."""
    out = np.empty((rows, cols), dtype=shards[0].dtype)
    seen = np.zeros((rows, cols), dtype=bool)
    for s, sh in enumerate(shards):
        rs, cs = shard_slices(rows, cols, t, s)
        if seen[rs, cs].all():
            if not np.array_equal(out[rs, cs].view(np.uint8), np.ascontiguousarray(sh).view(np.uint8)):
                raise AssertionError("replicas differ at shard %d" % s)
        out[rs, cs] = sh
        seen[rs, cs] = True
    assert seen.all()
    return out


def retile(shards, A, B, rows, cols):
    """Tiling conversion A -> B (Sec. 5.2 step 1): by definition the B-tiles of
    the tensor whose A-tiles are given."""
    return tile(untile(shards, A, rows, cols), B)


# ---- 4-D (convolution) tensors: only dim 0 and dim 1 are ever cut (Sec. 4.5) ----

def tile4(T, t):
    """R cuts dim 0 (batch / input channel), C cuts dim 1 (channel / output channel)."""
    d0, d1 = T.shape[:2]
    return [np.ascontiguousarray(T[shard_slices(d0, d1, t, s)]) for s in range(1 << len(t))]


def untile4(shards, t, shape):
    out = np.empty(shape, dtype=shards[0].dtype)
    for s, sh in enumerate(shards):
        out[shard_slices(shape[0], shape[1], t, s)] = sh
    return out


# ---- between a convolution and a fully-connected layer ----

def flatten_images(T):
    """[batch, channel, h, w] -> batch x (channel * h * w), channels major: the matrix a fully-connected layer
    multiplies.  With this column order the first half of the columns is the first half of the channels, so a column
    cut of the matrix is a channel cut of the images (Sec. 4.5 allows no other cut of an image tensor)."""
    return np.ascontiguousarray(T).reshape(T.shape[0], -1)


def unflatten_images(Mx, shape):
    """inverse of flatten_images: batch x (channel * h * w) -> [batch, channel, h, w]"""
    return np.ascontiguousarray(Mx).reshape(shape)
