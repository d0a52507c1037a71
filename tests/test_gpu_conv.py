"""Parity of the convolution execute calls (implicit GEMM) with the fp64 oracle (textbook definition in
oracle/layers.py, pinned against torch's CPU conv2d in the non-GPU tests).
Storage: activations NHWC seen as (N*H*W) x C matrices, filters [K][R][S][C] seen as (K*R*S) x C."""
import itertools

import numpy as np
import pytest
import torch

import paper_1805_04170_amd as tt
from oracle import execute as ex
from oracle import layers as ly
from oracle import tiling as tl
from synthetic import CONFIGS, bf16_bits_to_f64, normal_f32, to_bf16_bits

from gpu_util import DEV, alloc_shards, np_to_dev, shards_to_np

pytestmark = pytest.mark.gpu


def act_matrix(T):            # logical NCHW -> (N*H*W) x C
    n, c, h, w = T.shape
    return np.ascontiguousarray(T.transpose(0, 2, 3, 1)).reshape(n * h * w, c)


def act_from_matrix(Mx, n, c, h, w):
    return Mx.reshape(n, h, w, c).transpose(0, 3, 1, 2)


def filt_matrix(Wt):          # logical K C R S -> (K*R*S) x C
    k, c, r, s = Wt.shape
    return np.ascontiguousarray(Wt.transpose(0, 2, 3, 1)).reshape(k * r * s, c)


def filt_from_matrix(Mx, k, c, r, s):
    return Mx.reshape(k, r, s, c).transpose(0, 3, 1, 2)


def up(Mx, t):
    return [np_to_dev(s, Mx.dtype == np.uint16) for s in tl.tile(Mx, t)]


def ws(nbytes):
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV)


def close(got, want, mag, what, rel=1e-2):
    tol = rel * mag                                                # the stated bound, nothing added
    err = np.abs(got - want)
    assert np.all(np.isfinite(got)), what
    assert np.all(err <= tol + 1e-30), (what, float(err.max()), float((err / (tol + 1e-30)).max()))


def conv_mag_fwd(X, W, pad):
    return ly.conv_forward(np.abs(X), np.abs(W), pad)


def run_conv(N, C, K, H, Wd, R, S, pad, k, relu, tX, tW, tY, tdY, tdX, f_fwd, f_dg, f_wg, seed, with_dx=True, dt="bf16"):
    lay = tt.layer("conv", "relu" if relu else "none", C, K, H=H, W=Wd, R=R, S=S, pad=pad)
    P, Q = H + 2 * pad - R + 1, Wd + 2 * pad - S + 1
    bf = dt == "bf16"
    store = to_bf16_bits if bf else (lambda a: a.astype(np.float32))
    wide = bf16_bits_to_f64 if bf else (lambda a: a.astype(np.float64))
    tdt, rel = (torch.bfloat16, 1e-2) if bf else (torch.float32, 1e-5)
    Xb = store(normal_f32(seed, 0, (N, C, H, Wd), 1.0))
    Wb = store(normal_f32(seed, 1, (K, C, R, S), 0.05))
    dYb = store(normal_f32(seed, 2, (N, K, P, Q), 1.0))
    X, W, dY = wide(Xb), wide(Wb), wide(dYb)
    tWs = ex.transpose_tiling(tW)                      # letters on the filter storage matrix
    Xs, Ws_, dYs = up(act_matrix(Xb), tX), up(filt_matrix(Wb), tWs), up(act_matrix(dYb), tdY)
    Ys = alloc_shards(N * P * Q, K, tY, tdt, fill=float("nan"))
    nb = tt.tt_conv_workspace_bytes(lay, N, k, dt, tt.TT_OP_FWD, tX, tW, tY, forms_a=f_fwd)
    tt.tt_conv_forward(lay, N, k, dt, tX, tW, tY, f_fwd, Xs, Ws_, Ys, ws(nb))
    torch.cuda.synchronize()
    Ym = wide(tl.untile(shards_to_np(Ys), tY, N * P * Q, K))
    Yg = act_from_matrix(Ym, N, K, P, Q)
    want = ly.conv_forward(X, W, pad)
    if relu:
        want = np.maximum(want, 0)
    close(Yg, want, conv_mag_fwd(X, W, pad), ("fwd", tX, tW, tY, f_fwd), rel)
    dXs = alloc_shards(N * H * Wd, C, tdX, tdt, fill=float("nan")) if with_dx else None
    dWs = alloc_shards(K * R * S, C, tWs, tdt, fill=float("nan"))
    nb = tt.tt_conv_workspace_bytes(lay, N, k, dt, tt.TT_OP_DGRAD, tX, tW, tY, tdY, tdX, f_dg, f_wg, with_dx)
    tt.tt_conv_backward(lay, N, k, dt, tX, tW, tY, tdY, tdX, f_dg, f_wg, Xs, Ws_, Ys, dYs, dXs, dWs, ws(nb))
    torch.cuda.synchronize()
    G = dY * (Yg > 0) if relu else dY
    if with_dx:
        dXg = act_from_matrix(wide(tl.untile(shards_to_np(dXs), tdX, N * H * Wd, C)), N, C, H, Wd)
        close(dXg, ly.conv_dgrad(G, W, pad, H, Wd), ly.conv_dgrad(np.abs(G), np.abs(W), pad, H, Wd), ("dgrad", tdY, tW, tdX, f_dg), rel)
    dWg = filt_from_matrix(wide(tl.untile(shards_to_np(dWs), tWs, K * R * S, C)), K, C, R, S)
    close(dWg, ly.conv_wgrad(X, G, pad, R, S), ly.conv_wgrad(np.abs(X), np.abs(G), pad, R, S), ("wgrad", tX, tdY, tW, f_wg), rel)


def test_single_shard_and_one_cut():
    run_conv(2, 16, 24, 6, 5, 3, 3, 1, 0, False, "", "", "", "", "", "", "", "", 100)
    # data parallel (batch split), model parallel on output channels, on input channels
    run_conv(4, 16, 32, 6, 6, 3, 3, 1, 1, True, "R", "r", "R", "R", "R", "1", "1", "3", 101)
    run_conv(4, 16, 32, 6, 6, 3, 3, 1, 1, True, "r", "C", "C", "C", "r", "2", "3", "2", 102)
    run_conv(4, 16, 32, 6, 6, 3, 3, 1, 1, False, "C", "R", "r", "r", "C", "3", "2", "1", 103)


@pytest.mark.parametrize("relu", [False, True])
def test_every_form_sequence_two_cuts(relu):
    for f in ["".join(p) for p in itertools.product("123", repeat=2)]:
        run_conv(4, 32, 32, 5, 6, 3, 3, 1, 2, relu, "RC", "Cr", "rR", "CR", "RR", f, f, f, 110)


def test_random_stored_tilings_default_forms():
    rng = np.random.default_rng(6)
    ts = tl.all_tilings(2)
    for i in range(12):
        tX, tW, tY, tdY, tdX = (ts[j] for j in rng.integers(0, 9, 5))
        run_conv(4, 32, 64, 4, 4, 3, 3, 1, 2, bool(i % 2), tX, tW, tY, tdY, tdX, None, None, None, 120 + i)


def test_other_filter_shapes():
    run_conv(4, 64, 32, 7, 7, 1, 1, 0, 2, True, "RR", "rr", "RR", "RR", "RR", None, None, None, 130)     # 1x1
    run_conv(2, 16, 16, 9, 8, 5, 5, 2, 1, False, "R", "r", "R", "R", "R", None, None, None, 131)          # 5x5 "same"
    run_conv(2, 16, 16, 8, 8, 3, 3, 0, 1, False, "C", "R", "r", "r", "C", None, None, None, 132, False)   # no padding, no dX
    run_conv(8, 8, 8, 3, 3, 3, 3, 1, 3, True, "RRR", "rrr", "RRR", "RRR", "RRR", "111", "111", "333", 133)  # 8 channels: K tail
    run_conv(8, 64, 128, 6, 6, 3, 3, 1, 1, True, "r", "C", "C", "C", "r", "2", "3", "2", 134)           # 64 output channels per shard: 256 x 64 tiles


def test_weight_gradient_with_the_reduction_range_cut_evenly():
    # more than 128 output channels per shard and a multiple of 64 pixels per shard: the pixels of all shards that add up
    # into one filter block are cut into equal runs, which may start in one shard and end in the next
    run_conv(8, 16, 160, 8, 8, 3, 3, 1, 3, False, "RRR", "rrr", "RRR", "RRR", "RRR", "111", "111", "333", 140)     # batch split: one block, eight shards
    run_conv(8, 32, 320, 8, 8, 3, 3, 1, 2, True, "RC", "Cr", "rR", "CR", "RR", "13", "31", "32", 141)             # two blocks of two shards each
    run_conv(4, 64, 136, 8, 16, 3, 3, 1, 2, True, "rr", "RR", "rr", "rr", "CC", "33", "22", "11", 142)            # no F3 cut: the range of one shard cut into parts
    run_conv(16, 16, 264, 4, 4, 1, 1, 0, 1, False, "R", "r", "R", "R", "R", "1", "1", "3", 143)                    # 1x1 filters, 16 pixels per image, two row tiles


def test_shards_that_share_their_left_operand_run_as_one_product():
    # 64 or 128 columns per shard and the left operand replicated over the cuts that split them: forward and data gradient
    # run one product per group of shards, every wave writing into its own shard's result
    run_conv(4, 256, 256, 6, 6, 3, 3, 1, 2, True, "rr", "RR", "CC", "rr", "CC", "22", "22", "11", 180)    # the planner's kind of tiling
    run_conv(4, 64, 256, 5, 7, 3, 3, 1, 1, False, "r", "C", "C", "C", "r", "2", "3", "2", 181)            # 128 columns per shard, forward only fused
    run_conv(8, 128, 128, 4, 4, 3, 3, 1, 2, True, "Rr", "rC", "RC", "Rr", "RC", "12", "12", "31", 182)    # two groups of two members
    run_conv(4, 128, 256, 4, 4, 1, 1, 0, 2, False, "rC", "RC", "Cr", "rr", "CC", "23", "22", "12", 183)   # partial sums per member (F3 beside F2), 1 x 1 filters


def test_weight_gradient_of_shards_that_share_the_images_runs_as_one_product():
    # at most 128 output channels per shard and X replicated over the cuts that split them: the weight gradient runs as
    # one product over all output channels of a group (dY converted with those cuts replicated), its pixel range cut evenly
    run_conv(4, 64, 256, 8, 8, 3, 3, 1, 2, True, "rr", "CC", "CC", "CC", "rr", "22", "33", "22", 185)    # the output-channel split: one group
    run_conv(8, 32, 256, 8, 8, 3, 3, 1, 2, False, "Rr", "rC", "RC", "RC", "Rr", "12", "13", "32", 186)   # a batch cut beside it: two shards add up
    run_conv(4, 64, 512, 8, 8, 3, 3, 1, 2, True, "Cr", "RC", "rC", "rC", "Cr", "32", "23", "12", 187)    # an input-channel cut beside it: two blocks
    run_conv(4, 16, 384, 4, 16, 1, 1, 0, 3, False, "rrR", "CCr", "CCR", "CCR", "rrR", "221", "331", "223", 188)  # 96 channels per shard, three cuts
    run_conv(4, 64, 256, 6, 8, 1, 3, 1, 2, False, "rr", "CC", "CC", "CC", "rr", "22", "33", "22", 192)    # 1 x 3 taps: the merged data gradient on the kernel that reads the filters as they are
    # ... and the mirror case, at most 128 input channels per shard with dY replicated over the cuts that split them
    run_conv(4, 256, 256, 8, 8, 3, 3, 1, 2, True, "rr", "RR", "CC", "rr", "CC", "22", "22", "11", 189)   # the planner's kind of tiling: one group
    run_conv(4, 256, 256, 8, 8, 3, 3, 1, 2, False, "Cr", "RC", "rC", "rC", "Cr", "32", "23", "12", 190)  # both kinds of cut: one product is left
    run_conv(8, 256, 192, 8, 8, 3, 3, 1, 2, True, "CR", "Rr", "rR", "rR", "CR", "31", "21", "13", 191)   # a batch cut beside it: two shards add up


def test_fp32_convolutions():
    # fp32 operands and results on the plain kernels: no cut, every form at one cut, mixed forms and stored tilings at
    # two cuts (partial sums, gate, conversions as for bf16), odd channel counts (no 16-byte vectors needed), 5 x 3 taps
    run_conv(2, 5, 7, 6, 5, 3, 3, 1, 0, True, "", "", "", "", "", "", "", "", 170, dt="f32")
    run_conv(4, 6, 10, 5, 5, 3, 3, 1, 1, True, "R", "r", "R", "R", "R", "1", "1", "3", 171, dt="f32")
    run_conv(4, 6, 10, 5, 5, 3, 3, 1, 1, False, "r", "C", "C", "C", "r", "2", "3", "2", 172, dt="f32")
    run_conv(4, 6, 10, 5, 5, 3, 3, 1, 1, True, "C", "R", "r", "r", "C", "3", "2", "1", 173, dt="f32")
    for i, f in enumerate(["12", "31", "23", "33"]):
        run_conv(4, 12, 8, 4, 6, 5, 3, 2, 2, bool(i % 2), "RC", "Cr", "rR", "CR", "RR", f, f, f, 174 + i, dt="f32")
    run_conv(8, 16, 16, 4, 4, 3, 3, 1, 3, True, "RRR", "rrr", "RRR", "RRR", "RRR", None, None, None, 179, dt="f32")


def test_refusals():
    lay = tt.layer("conv", "none", 12, 16, H=4, W=4, R=3, S=3, pad=1)       # 12 channels: no 16-byte channel vectors
    x = [torch.zeros(4096, dtype=torch.bfloat16, device=DEV)]
    with pytest.raises(tt.TilingError) as e:
        tt.tt_conv_forward(lay, 2, 0, "bf16", "", "", "", "", x, x, x)
    assert e.value.status == 3
    lay = tt.layer("conv", "none", 16, 16, H=4, W=4, R=3, S=3, pad=1)
    with pytest.raises(tt.TilingError) as e:                                  # batch 2 cannot be cut twice
        tt.tt_conv_forward(lay, 2, 2, "bf16", "RR", "rr", "RR", "11", x * 4, x * 4, x * 4)
    assert e.value.status == 2


_CONV4_ORACLE = {}


def conv4_oracle(cfg):
    """the untiled fp64 results of the full-size layer and their magnitude products (the same for every split: no
    activation, so the gated gradient is the incoming one); computed once per session, about half a minute of host time"""
    if not _CONV4_ORACLE:
        X, W, dY = bf16_bits_to_f64(cfg.x()), bf16_bits_to_f64(cfg.weight()), bf16_bits_to_f64(cfg.grad_out())
        aX, aW, adY = np.abs(X), np.abs(W), np.abs(dY)
        _CONV4_ORACLE.update(
            Y=(ly.conv_forward(X, W, cfg.pad), ly.conv_forward(aX, aW, cfg.pad)),
            dX=(ly.conv_dgrad(dY, W, cfg.pad, cfg.H, cfg.W), ly.conv_dgrad(adY, aW, cfg.pad, cfg.H, cfg.W)),
            dW=(ly.conv_wgrad(X, dY, cfg.pad, cfg.R, cfg.S), ly.conv_wgrad(aX, adY, cfg.pad, cfg.R, cfg.S)))
    return _CONV4_ORACLE


@pytest.mark.parametrize("split", ["planner", "batch", "out_channel"])
def test_config_vgg_conv4_full_size_every_element(split):
    cfg = CONFIGS["vgg16_conv4"]
    N, C, K, H, Wd, R, S, pad, k = cfg.N, cfg.C, cfg.K, cfg.H, cfg.W, cfg.R, cfg.S, cfg.pad, cfg.k
    P, Q = cfg.P, cfg.Q
    lay = tt.layer("conv", "none", C, K, H=H, W=Wd, R=R, S=S, pad=pad)
    if split == "planner":
        p = tt.tt_plan_chain([lay], N, k)
        tX, tY, tW, tdY, tdX = p.x()[0], p.x()[1], p.w()[0], p.g()[1], p.g()[0]
        f = [p.forms(1, o) for o in range(3)]
    elif split == "batch":
        tX = tY = tdY = tdX = "RRR"; tW = "rrr"; f = ["111", "111", "333"]
    else:
        tX = tdX = "rrr"; tY = tdY = "CCC"; tW = "CCC"; f = ["222", "333", "222"]
    Xb, Wb, dYb = cfg.x(), cfg.weight(), cfg.grad_out()
    tWs = ex.transpose_tiling(tW)
    Xs, Ws_, dYs = up(act_matrix(Xb), tX), up(filt_matrix(Wb), tWs), up(act_matrix(dYb), tdY)
    Ys = alloc_shards(N * P * Q, K, tY, torch.bfloat16, fill=float("nan"))
    dXs = alloc_shards(N * H * Wd, C, tdX, torch.bfloat16, fill=float("nan"))
    dWs = alloc_shards(K * R * S, C, tWs, torch.bfloat16, fill=float("nan"))
    nb = max(tt.tt_conv_workspace_bytes(lay, N, k, "bf16", tt.TT_OP_FWD, tX, tW, tY, forms_a=f[0]),
             tt.tt_conv_workspace_bytes(lay, N, k, "bf16", tt.TT_OP_DGRAD, tX, tW, tY, tdY, tdX, f[1], f[2]))
    w = ws(nb)
    tt.tt_conv_forward(lay, N, k, "bf16", tX, tW, tY, f[0], Xs, Ws_, Ys, w)
    tt.tt_conv_backward(lay, N, k, "bf16", tX, tW, tY, tdY, tdX, f[1], f[2], Xs, Ws_, Ys, dYs, dXs, dWs, w)
    torch.cuda.synchronize()
    Yg = act_from_matrix(bf16_bits_to_f64(tl.untile(shards_to_np(Ys), tY, N * P * Q, K)), N, K, P, Q)
    dXg = act_from_matrix(bf16_bits_to_f64(tl.untile(shards_to_np(dXs), tdX, N * H * Wd, C)), N, C, H, Wd)
    dWg = filt_from_matrix(bf16_bits_to_f64(tl.untile(shards_to_np(dWs), tWs, K * R * S, C)), K, C, R, S)
    o = conv4_oracle(cfg)                                  # all 64 images, all 512 x 512 x 3 x 3 filter gradients
    close(Yg, o["Y"][0], o["Y"][1], ("fwd", split))
    close(dXg, o["dX"][0], o["dX"][1], ("dgrad", split))
    close(dWg, o["dW"][0], o["dW"][1], ("wgrad", split))
