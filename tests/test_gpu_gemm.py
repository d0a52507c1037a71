"""Parity of the shard-product kernels with the fp64 oracle.
bf16 inputs / fp32 accumulate: |gpu - oracle| <= 1e-2 * (|A| |B|)_ij  (+ half an ulp of a bf16 store);
fp32: <= 1e-5 * (|A| |B|)_ij."""
import numpy as np
import pytest
import torch

import paper_1805_04170_amd as tt
from oracle import layers as ly
from synthetic import bf16_bits_to_f64, normal_f32, to_bf16_bits

from gpu_util import DEV, dev_to_np, np_to_dev

pytestmark = pytest.mark.gpu


def check(count, M, N, K, ta, tb, in_dt, out_dt, relu, seed):
    bf = in_dt == "bf16"
    As, Bs, Cs, want, mags = [], [], [], [], []
    for s in range(count):
        a = normal_f32(seed, 2 * s, (M, K), 1.0)
        b = normal_f32(seed, 2 * s + 1, (K, N), 0.05)
        if bf:
            a, b = to_bf16_bits(a), to_bf16_bits(b)
        af = bf16_bits_to_f64(a) if bf else a.astype(np.float64)
        bfl = bf16_bits_to_f64(b) if bf else b.astype(np.float64)
        z = af @ bfl
        want.append(np.maximum(z, 0) if relu else z)
        mags.append(ly.abs_product(af, bfl))
        As.append(np_to_dev(a.T if ta else a, bf))
        Bs.append(np_to_dev(b.T if tb else b, bf))
        Cs.append(torch.full((M, N), float("nan"), dtype=torch.bfloat16 if out_dt == "bf16" else torch.float32, device=DEV))
    tt.tt_shard_gemm(As, Bs, Cs, M, N, K, ta, tb, in_dt, out_dt, tt.TT_ACT_RELU if relu else tt.TT_ACT_NONE)
    torch.cuda.synchronize()
    for s in range(count):
        got = dev_to_np(Cs[s])
        gf = bf16_bits_to_f64(got) if out_dt == "bf16" else got.astype(np.float64)
        tol = (1e-2 if bf else 1e-5) * mags[s]                      # the stated bound, nothing added
        err = np.abs(gf - want[s])
        assert np.all(np.isfinite(gf)), (s, "non-finite output")
        assert np.all(err <= tol + 1e-30), (s, float(err.max()), float((err / (tol + 1e-30)).max()))
        # the bound is loose for fp32 accumulation; also require a tight typical error so a dropped k-tile cannot hide:
        # 1e-4 of the magnitude product, plus the rounding of the stored result where that is bf16 (8 significant bits,
        # round to nearest: at most 2^-8 of the value)
        if bf:
            tight = 1e-4 * mags[s] + (2.0 ** -8 * np.abs(want[s]) if out_dt == "bf16" else 0.0)
            assert np.all(err <= tight + 1e-30), (s, float((err / (tight + 1e-30)).max()))


LAYOUTS = [(0, 0), (0, 1), (1, 0), (1, 1)]


@pytest.mark.parametrize("ta,tb", LAYOUTS)
@pytest.mark.parametrize("out_dt", ["bf16", "f32"])
def test_bf16_mfma_tiles_and_tails(ta, tb, out_dt):
    # several 128/256 tiles plus ragged tails in M, N and K (all multiples of 8 along contiguous dims)
    check(3, 264, 200, 328, ta, tb, "bf16", out_dt, False, 31)
    check(2, 128, 136, 64, ta, tb, "bf16", out_dt, True, 32)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_bf16_small_and_tall(ta, tb):
    check(8, 32, 512, 1024, ta, tb, "bf16", "f32", False, 33)      # batch-split shard: few rows
    check(1, 520, 72, 40, ta, tb, "bf16", "bf16", False, 34)        # three row tiles, one short K tile


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_bf16_unaligned_falls_back(ta, tb):
    check(2, 37, 125, 50, ta, tb, "bf16", "bf16", True, 35)         # 125-wide rows: no 16-byte vectors
    check(2, 33, 10, 17, ta, tb, "bf16", "f32", False, 36)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_fp32(ta, tb):
    check(4, 32, 10, 256, ta, tb, "f32", "f32", False, 37)
    check(2, 70, 130, 65, ta, tb, "f32", "f32", True, 38)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_bf16_large_launch_eight_wave_tiles(ta, tb):
    # enough 256 x 256 tiles for the eight-wave kernels (both tile engines, chosen by layout), ragged M, N and K
    check(8, 1000, 1016, 200, ta, tb, "bf16", "bf16", True, 39)
    check(8, 1024, 1024, 192, ta, tb, "bf16", "f32", False, 40)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
@pytest.mark.parametrize("out_dt", ["bf16", "f32"])
def test_bf16_persistent_engine(ta, tb, out_dt):
    # K a multiple of 64 and more 256 x 256 tiles than CUs: the persistent pipelined engine, several output tiles per
    # workgroup (prefetch runs across tile boundaries), ragged M and N, K loops of one, two and five tiles
    check(8, 1544, 1528, 128, ta, tb, "bf16", out_dt, True, 42)
    check(8, 1032, 1544, 64, ta, tb, "bf16", out_dt, False, 43)
    check(3, 2056, 1800, 320, ta, tb, "bf16", out_dt, False, 44)
    # three output tiles per workgroup and a K loop of four tiles: a full tile's write-out rides along the next one
    check(8, 2056, 2312, 256, ta, tb, "bf16", out_dt, True, 48)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
@pytest.mark.parametrize("out_dt", ["bf16", "f32"])
def test_bf16_two_workgroups_per_cu_engine(ta, tb, out_dt):
    # launches with few 256 x 256 tiles, K a multiple of 32: the 256 x 128 engine (three-stage ring of 32-deep K tiles);
    # ragged M and N, K loops of 3 (the ring is deeper than one of the loops is long) and 16 tiles
    check(2, 520, 520, 96, ta, tb, "bf16", out_dt, True, 45)
    check(8, 256, 1024, 512, ta, tb, "bf16", out_dt, False, 46)
    check(1, 136, 264, 32, ta, tb, "bf16", out_dt, False, 47)


@pytest.mark.parametrize("out_dt", ["bf16", "f32"])
def test_bf16_line_wide_k_tiles_engine(out_dt):
    # skinny A B^T products with at most one 256 x 128 tile per CU and K a multiple of 64 (the data gradients at batch
    # 256): the 256 x 128 engine with K tiles of 64 (two stages of A, three of B); ragged N, ragged M, K loops of 8, 4
    # and 64 tiles, the last at the shape of the VGG-16 first data gradient
    check(16, 256, 1064, 512, 0, 1, "bf16", out_dt, True, 49)
    check(32, 200, 392, 256, 0, 1, "bf16", out_dt, False, 50)
    check(6, 256, 3136, 4096, 0, 1, "bf16", out_dt, False, 51)


@pytest.mark.parametrize("K", [256, 128, 512])
def test_bf16_panel_in_registers_engine(K):
    # weight-gradient shaped products (both operands stored K-major, K = 128 / 256, large bf16 result): the engine that
    # keeps the left operand's panel in registers; 8 shards x 5 panels (the last with 8 of 256 rows) x 52 column tiles
    # on 512 resident workgroups, so runs change panel and shard mid-way
    check(8, 1032, 3328, K, 1, 0, "bf16", "bf16", K == 128, 48)


def test_k_zero_and_empty():
    C = [torch.full((8, 8), 5.0, dtype=torch.float32, device=DEV)]
    A = [torch.zeros((8, 1), dtype=torch.bfloat16, device=DEV)]
    tt.tt_shard_gemm(A, A, C, 8, 8, 0, 0, 0, "bf16", "f32")
    torch.cuda.synchronize()
    assert torch.all(C[0] == 0)
    tt.tt_shard_gemm(A, A, C, 0, 8, 4, 0, 0, "bf16", "f32")          # nothing to do


def test_vgg_shard_shape_every_element():
    # the K-split shard product of the VGG-16 first classifier layer: 256 x 3136 x 4096, fp32 partial output
    M, K, N = 256, 3136, 4096
    a = to_bf16_bits(normal_f32(41, 0, (M, K), 1.0)); b = to_bf16_bits(normal_f32(41, 1, (K, N), 0.005))
    A = [np_to_dev(a, True)]; B = [np_to_dev(b, True)]
    C = [torch.empty((M, N), dtype=torch.float32, device=DEV)]
    tt.tt_shard_gemm(A, B, C, M, N, K, 0, 0, "bf16", "f32")
    torch.cuda.synchronize()
    got = dev_to_np(C[0]).astype(np.float64)
    af, bfl = bf16_bits_to_f64(a), bf16_bits_to_f64(b)
    want = af @ bfl
    mag = ly.abs_product(af, bfl)
    assert np.all(np.abs(got - want) <= 1e-2 * mag)
    assert float(np.max(np.abs(got - want) / mag)) < 1e-4
