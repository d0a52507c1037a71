"""Parity of the conversion kernels (retile, gated retile, partial-sum reduce) with the oracle: bit-exact for
copies, relative error <= 1e-5 for the fp32 sums."""
import itertools

import numpy as np
import pytest
import torch

import paper_1805_04170_amd as tt
from oracle import execute as ex
from oracle import tiling as tl
from synthetic import CONFIGS, bf16_bits_to_f32, to_bf16_bits, normal_f32

from gpu_util import DEV, alloc_shards, dev_to_np, np_to_dev, shards_to_dev, shards_to_np

pytestmark = pytest.mark.gpu

NP_OF = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}
TORCH_OF = {1: torch.uint8, 2: torch.int16, 4: torch.int32, 8: torch.int64}


def run_retile(T, A, B, e):
    rows, cols = T.shape
    src = [torch.from_numpy(s.view(NP_OF[e]).view({1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}[e])).to(DEV)
           for s in tl.tile(T, A)]
    dst = alloc_shards(rows, cols, B, TORCH_OF[e], fill=0)
    tt.tt_retile(dst, B, src, A, rows, cols, e)
    torch.cuda.synchronize()
    got = [d.cpu().numpy().view(NP_OF[e]) for d in dst]
    want = tl.tile(T, B)
    for s, (g, w) in enumerate(zip(got, want)):
        assert np.array_equal(g, w), (A, B, e, s)
    return dst


@pytest.mark.parametrize("e", [1, 2, 4, 8])
def test_retile_all_pairs_two_cuts(e):
    rng = np.random.default_rng(e)
    T = rng.integers(0, 256, size=(24, 40 * e), dtype=np.uint8).view(NP_OF[e]).reshape(24, 40)
    for A, B in itertools.product(tl.all_tilings(2), repeat=2):
        run_retile(T, A, B, e)


def test_retile_three_cuts_ragged_shapes():
    # 1000 columns: shard widths 500 / 250 / 125 fall back to 8-, 4- and 2-byte vectors; 200 rows of 25 each
    rng = np.random.default_rng(7)
    T = rng.integers(0, 1 << 16, size=(200, 1000), dtype=np.uint16)
    ts = tl.all_tilings(3)
    pick = rng.choice(len(ts), size=(40, 2))
    for ia, ib in pick:
        run_retile(T, ts[ia], ts[ib], 2)
    run_retile(T, "CCC", "RRR", 2)
    run_retile(T, "RRR", "CCC", 2)
    run_retile(T, "rrr", "CCC", 2)
    run_retile(T, "CCC", "rrr", 2)


def test_retile_k0_k4_and_roundtrip():
    rng = np.random.default_rng(8)
    T = rng.integers(0, 1 << 32, size=(64, 96), dtype=np.uint32)
    run_retile(T, "", "", 4)
    run_retile(T, "RRCC", "CCrR", 4)
    run_retile(T, "RCRC", "CRCR", 4)
    # A -> B -> A is the identity
    A, B = "RCr", "CCR"
    src = shards_to_dev(T.view(np.int32), A)
    mid = alloc_shards(64, 96, B, torch.int32)
    back = alloc_shards(64, 96, A, torch.int32)
    tt.tt_retile(mid, B, src, A, 64, 96, 4)
    tt.tt_retile(back, A, mid, B, 64, 96, 4)
    torch.cuda.synchronize()
    for a, b in zip(src, back):
        assert torch.equal(a, b)


def test_retile_six_cuts():
    rng = np.random.default_rng(9)
    T = rng.integers(0, 1 << 16, size=(128, 256), dtype=np.uint16)
    run_retile(T, "RRRCCC", "CCCRRR", 2)
    run_retile(T, "RCrRCr", "rrCCRR", 2)


def test_retile_full_size_weight():
    # VGG-16 first classifier weight, 25088 x 4096 bf16 (205.5 MB), the launch shape the benchmark times
    rows, cols = 25088, 4096
    g = torch.Generator(device="cpu").manual_seed(11)
    T = torch.randint(-32768, 32767, (rows, cols), dtype=torch.int16, generator=g)
    for A, B in [("RRR", "CCC"), ("RRR", "CRC")]:
        src = [T[tl.shard_slices(rows, cols, A, s)].contiguous().to(DEV) for s in range(8)]
        dst = alloc_shards(rows, cols, B, torch.int16, fill=0)
        tt.tt_retile(dst, B, src, A, rows, cols, 2)
        torch.cuda.synchronize()
        for s in range(8):
            assert torch.equal(dst[s].cpu(), T[tl.shard_slices(rows, cols, B, s)]), (A, B, s)
        del src, dst


@pytest.mark.parametrize("rows,cols", [(512, 4096), (1024, 8192), (520, 1032)])
def test_retile_and_gate_medium_tensors(rows, cols):
    # activation-sized tensors (2 and 8 M elements and a ragged one): the launches with two and four vectors per lane
    # and a tail of partly filled workgroups
    rng = np.random.default_rng(rows)
    T = rng.integers(0, 1 << 16, size=(rows, cols), dtype=np.uint16)
    for A, B in [("RC", "CR"), ("RRC", "Crr"), ("rC", "RR")]:
        run_retile(T, A, B, 2)
    v = rng.standard_normal((rows, cols)).astype(np.float32)
    m = rng.standard_normal((rows, cols)).astype(np.float32)
    V, Mk = to_bf16_bits(v), to_bf16_bits(m)
    want_full = np.where(bf16_bits_to_f32(Mk) > 0, V, np.zeros_like(V))
    for A, Am, B in [("RC", "CR", "RR"), ("Cr", "RC", "CC")]:
        src = shards_to_dev(V, A, True)
        msk = shards_to_dev(Mk, Am, True)
        dst = alloc_shards(rows, cols, B, torch.bfloat16)
        tt.tt_retile_gate(dst, B, src, A, msk, Am, rows, cols, "bf16")
        torch.cuda.synchronize()
        got = tl.untile(shards_to_np(dst), B, rows, cols)
        assert np.array_equal(got.view(np.uint16), want_full.view(np.uint16)), (A, Am, B)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_gated_retile(dtype):
    rng = np.random.default_rng(12)
    rows, cols = 48, 80
    v = rng.standard_normal((rows, cols)).astype(np.float32)
    m = rng.standard_normal((rows, cols)).astype(np.float32)
    m[rng.random((rows, cols)) < 0.3] = 0.0
    m[0, 0] = -0.0
    bf = dtype == "bf16"
    V = to_bf16_bits(v) if bf else v
    Mk = to_bf16_bits(m) if bf else m
    mf = bf16_bits_to_f32(Mk) if bf else Mk
    want_full = np.where(mf > 0, V, np.zeros_like(V))
    tdt = torch.bfloat16 if bf else torch.float32
    for A, Am, B in [("RR", "CC", "Rr"), ("Cr", "rR", "CC"), ("rr", "RC", "RC"), ("RC", "RC", "RC")]:
        src = shards_to_dev(V, A, bf)
        msk = shards_to_dev(Mk, Am, bf)
        dst = alloc_shards(rows, cols, B, tdt)
        tt.tt_retile_gate(dst, B, src, A, msk, Am, rows, cols, dtype)
        torch.cuda.synchronize()
        got = tl.untile(shards_to_np(dst), B, rows, cols)
        assert np.array_equal(got.view(np.uint16 if bf else np.uint32), want_full.view(np.uint16 if bf else np.uint32))


@pytest.mark.parametrize("forms,B,out,relu", [
    ("3", "r", "f32", False), ("33", "RR", "bf16", True), ("13", "CR", "f32", True), ("32", "rC", "bf16", False),
    ("333", "RRR", "bf16", False), ("231", "rCr", "f32", False), ("12", "CR", "bf16", True), ("3333", "RRCC", "f32", False),
])
def test_reduce_against_oracle(forms, B, out, relu):
    rng = np.random.default_rng(len(forms) * 7 + len(B))
    rows, cols = 64, 96
    k = len(forms)
    k1, k2 = forms.count("1"), forms.count("2")
    parts = [rng.standard_normal((rows >> k1, cols >> k2)).astype(np.float32) for _ in range(1 << k)]
    want = ex.reduce_to([p.astype(np.float64) for p in parts], forms, B, rows, cols, relu)
    dparts = [np_to_dev(p) for p in parts]
    dst = alloc_shards(rows, cols, B, torch.bfloat16 if out == "bf16" else torch.float32)
    tt.tt_reduce(dst, B, out, dparts, forms, rows, cols, tt.TT_ACT_RELU if relu else tt.TT_ACT_NONE)
    torch.cuda.synchronize()
    # scale of the sum: sum of |partials| over the reduced cuts
    mag = ex.assemble([np.abs(p).astype(np.float64) for p in parts], forms, rows, cols)
    for s, (d, w) in enumerate(zip(dst, want)):
        g = dev_to_np(d)
        gf = bf16_bits_to_f32(g).astype(np.float64) if out == "bf16" else g.astype(np.float64)
        sl = tl.shard_slices(rows, cols, B, s)
        tol = 1e-5 * mag[sl] + (2.0 ** -8 * np.abs(w) if out == "bf16" else 0.0)   # + half-ulp of the bf16 store
        assert np.all(np.abs(gf - w) <= tol + 1e-30), (forms, B, s)


def test_reduce_ragged_columns_scalar_path():
    rng = np.random.default_rng(21)
    rows, cols = 32, 250            # 125-wide blocks: no 16-byte vectors
    forms, B = "23", "Cr"
    parts = [rng.standard_normal((rows, cols // 2)).astype(np.float32) for _ in range(4)]
    want = ex.reduce_to([p.astype(np.float64) for p in parts], forms, B, rows, cols, False)
    dst = alloc_shards(rows, cols, B, torch.float32)
    tt.tt_reduce(dst, B, "f32", [np_to_dev(p) for p in parts], forms, rows, cols)
    torch.cuda.synchronize()
    for d, w in zip(dst, want):
        np.testing.assert_allclose(dev_to_np(d).astype(np.float64), w, rtol=1e-5, atol=1e-6)
