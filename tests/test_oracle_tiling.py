"""Pins for oracle/tiling.py: the sets the paper prints, hand-placed blocks,
and the invariants of Def. 1 and the flattening theorem."""
import itertools

import numpy as np
import pytest

from oracle import tiling as tl


def test_T2_as_printed(golden_loader):
    g = golden_loader("paper_tilings.txt")
    assert tl.all_tilings(2) == g["T2"]                      # Sec. 4.1, listing after Def. 1
    classes = {tl.flattened(t) for t in tl.all_tilings(2)}
    assert classes == {tl.flattened(t) for t in g["T2_flat"]}  # Sec. 4.4: six classes
    assert len(classes) == 6


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_counts(k):
    assert len(tl.all_tilings(k)) == 3 ** k
    assert len({tl.flattened(t) for t in tl.all_tilings(k)}) == (k + 1) * (k + 2) // 2


def test_hand_placed_blocks():
    # Fig. 4(b): RR = four row strips; RC = 2x2 blocks.  First cut = most significant bit.
    T = np.arange(32).reshape(4, 8)
    rr = tl.tile(T, "RR")
    assert [s[0, 0] for s in rr] == [0, 8, 16, 24] and rr[0].shape == (1, 8)
    rc = tl.tile(T, "RC")
    assert rc[0].shape == (2, 4)
    assert [int(s[0, 0]) for s in rc] == [0, 4, 16, 20]        # s=1 flips the inner (C) cut
    cr = tl.tile(T, "CR")
    assert [int(s[0, 0]) for s in cr] == [0, 16, 4, 20]        # s=1 flips the inner (R) cut
    rr_ = tl.tile(T, "Rr")
    assert np.array_equal(rr_[0], rr_[1]) and np.array_equal(rr_[2], rr_[3])
    assert np.array_equal(rr_[0], T[:2]) and np.array_equal(rr_[2], T[2:])
    r_R = tl.tile(T, "rR")
    assert np.array_equal(r_R[0], T[:2]) and np.array_equal(r_R[1], T[2:]) and np.array_equal(r_R[2], T[:2])


@pytest.mark.parametrize("k", [1, 2, 3])
def test_tile_untile_identity_and_sizes(k):
    rng = np.random.default_rng(k)
    T = rng.integers(0, 1 << 30, size=(16, 24)).astype(np.int64)
    for t in tl.all_tilings(k):
        shards = tl.tile(T, t)
        assert len(shards) == 2 ** k
        assert sum(s.size for s in shards) == 2 ** t.count("r") * T.size
        assert all(s.shape == tl.shard_shape(16, 24, t) for s in shards)
        assert np.array_equal(tl.untile(shards, t, 16, 24), T)


def test_flattening_same_tile_set():
    # any reordering of a cut sequence yields the same multiset of tiles (Sec. 4.4)
    T = np.arange(8 * 8).reshape(8, 8)
    for t in ["RCr", "RRC", "Crr", "RCC"]:
        ref = sorted(s.tobytes() for s in tl.tile(T, t))
        for p in set(itertools.permutations(t)):
            assert sorted(s.tobytes() for s in tl.tile(T, "".join(p))) == ref


def test_uneven_rejected():
    with pytest.raises(ValueError):
        tl.shard_shape(10, 6, "RR")
    assert tl.shard_shape(10, 6, "RC") == (5, 3)


def test_retile_roundtrip_and_copy():
    rng = np.random.default_rng(5)
    T = rng.standard_normal((8, 16)).astype(np.float32)
    for A in tl.all_tilings(2):
        a = tl.tile(T, A)
        same = tl.retile(a, A, A, 8, 16)
        assert all(np.array_equal(x, y) for x, y in zip(a, same))
        for B in tl.all_tilings(2):
            back = tl.retile(tl.retile(a, A, B, 8, 16), B, A, 8, 16)
            assert all(np.array_equal(x, y) for x, y in zip(a, back))


def test_untile_detects_bad_replica():
    T = np.arange(16.0).reshape(4, 4)
    sh = tl.tile(T, "r")
    sh[1] = sh[1] + 1
    with pytest.raises(AssertionError):
        tl.untile(sh, "r", 4, 4)


def test_tile4_matches_2d_rule():
    T = np.arange(4 * 8 * 2 * 3).reshape(4, 8, 2, 3)
    for t in ["RC", "CR", "rR", "CC"]:
        sh = tl.tile4(T, t)
        flat = tl.tile(T[:, :, 0, 0], t)
        for a, b in zip(sh, flat):
            assert np.array_equal(a[:, :, 0, 0], b)
        assert np.array_equal(tl.untile4(sh, t, T.shape), T)


def test_flattened_images_column_cut_is_a_channel_cut():
    # Sec. 4.5: image tensors are cut along batch and channel only.  With channel-major columns the tiles of the
    # flattened matrix are the flattened tiles of the 4-D tensor, for every tiling (so no other cut ever appears).
    rng = np.random.default_rng(11)
    T = rng.integers(0, 1000, size=(4, 8, 3, 5))
    Mx = tl.flatten_images(T)
    assert Mx.shape == (4, 120)
    assert Mx[2, 3 * 15 + 1 * 5 + 4] == T[2, 3, 1, 4]                     # column = (channel, row, column of the image)
    for t in tl.all_tilings(2) + ["CCC", "RCr"]:
        for a, b in zip(tl.tile(Mx, t), tl.tile4(T, t)):
            assert np.array_equal(a, tl.flatten_images(b)), t
    assert np.array_equal(tl.unflatten_images(Mx, T.shape), T)
