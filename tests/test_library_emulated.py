"""The whole library built for the host and run in lock step (tests/emu): every source file of the library as it is,
kernels included (tests/emu/emu_lockstep.h says how threads, barriers and the wave-wide instructions are stood in for),
loaded in place of the HIP build for the duration of a test.  The checks are the GPU parity tests' own functions, called
on host tensors at sizes the emulation finishes in seconds: the execute calls (planning of conversions, workspace
layout, launches, reductions) and the kernels produce, on the host, what the oracle says.  This is a test of the
product's sources; the product itself never loads this build.
"""
import ctypes
import os
import shutil
import subprocess

import numpy as np
import pytest
import torch

import paper_1805_04170_amd.binding as binding
from oracle import tiling as tl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = shutil.which("clang++", path="/opt/rocm/llvm/bin") or shutil.which("clang++")
pytestmark = pytest.mark.skipif(CLANG is None, reason="no host clang++ for the emulation build")


@pytest.fixture(scope="module")
def emulated_library(emulators):
    return emulators.get("library")


@pytest.fixture
def on_host(emulated_library, monkeypatch):
    """the binding and the GPU tests' helpers pointed at the emulated library and at host tensors"""
    import gpu_util
    import test_gpu_conv
    import test_gpu_convert
    import test_gpu_fc
    import test_gpu_gemm
    import test_gpu_net
    monkeypatch.setattr(binding, "LIB_PATH", emulated_library)
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_stream", lambda stream: ctypes.c_void_p(0))
    monkeypatch.setattr(torch.cuda, "synchronize", lambda *a, **k: None)
    for m in (gpu_util, test_gpu_fc, test_gpu_conv, test_gpu_convert, test_gpu_gemm, test_gpu_net):
        if hasattr(m, "DEV"):
            monkeypatch.setattr(m, "DEV", "cpu")

    def aligned_workspace(nbytes):      # device allocations are 256-byte aligned, which the library asks of a workspace
        n = max(int(nbytes), 256)
        raw = torch.empty(n + 256, dtype=torch.uint8)
        return raw[(-raw.data_ptr()) % 256:][:n]

    monkeypatch.setattr(test_gpu_fc, "workspace", aligned_workspace)
    monkeypatch.setattr(test_gpu_conv, "ws", aligned_workspace)
    monkeypatch.setattr(test_gpu_net, "workspace", aligned_workspace)
    return dict(fc=test_gpu_fc, conv=test_gpu_conv, convert=test_gpu_convert, gemm=test_gpu_gemm, net=test_gpu_net)


def test_every_declared_symbol_is_exported_by_the_host_build(emulated_library):
    L = ctypes.CDLL(emulated_library)
    for name in binding.EXPORTS:
        assert hasattr(L, name), name


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_fc_layer_named_tilings(on_host, golden_loader, dt):
    g = golden_loader("paper_tilings.txt")
    for name in ["T_data", "T_model", "T_hybrid"]:
        tW, tA, tG = g[name]
        k = len(tW)
        on_host["fc"].run_layer(32, 64, 48, k, dt, True, tA, tW, tA, tG, tG, None, None, None, 50 + k)


# ---- the GPU parity tests themselves, run on the host where their sizes allow

@pytest.mark.parametrize("relu", [False, True])
def test_fc_every_form_sequence_two_cuts(on_host, relu):
    on_host["fc"].test_every_form_sequence_two_cuts(relu)


def test_fc_random_stored_tilings(on_host):
    on_host["fc"].test_random_stored_tilings_default_forms()


def test_fc_three_cuts_ragged_width_and_skip_dx(on_host):
    on_host["fc"].test_three_cuts_ragged_width_and_skip_dx()


def test_fc_refusals(on_host):
    on_host["fc"].test_uneven_and_bad_workspace_are_refused()


def test_fc_tiny_mlp_planned_and_recursive(on_host):
    on_host["fc"].test_config_tiny_mlp_fp32_planned_and_recursive()


def test_conv_single_shard_and_one_cut(on_host):
    on_host["conv"].test_single_shard_and_one_cut()


@pytest.mark.parametrize("relu", [False, True])
def test_conv_every_form_sequence_two_cuts(on_host, relu):
    on_host["conv"].test_every_form_sequence_two_cuts(relu)


def test_conv_random_stored_tilings(on_host):
    on_host["conv"].test_random_stored_tilings_default_forms()


def test_conv_other_filter_shapes(on_host):
    on_host["conv"].test_other_filter_shapes()


@pytest.mark.parametrize("engine", [1, 2])
def test_conv_weight_gradient_with_the_reduction_range_cut_evenly(on_host, monkeypatch, engine):
    monkeypatch.setenv("TT_WGRAD_ENGINE", str(engine))
    on_host["conv"].test_weight_gradient_with_the_reduction_range_cut_evenly()


@pytest.mark.parametrize("engine", [1, 2])
@pytest.mark.parametrize("parts", [1, 3, 7])
def test_conv_weight_gradient_every_number_of_partial_sums(on_host, monkeypatch, parts, engine):
    # the development build lets the test choose how many runs the reduction range is cut into: runs of unequal length,
    # runs that start inside one shard and end inside another, one run over all four shards of a block; on both engines
    monkeypatch.setenv("TT_WGRAD_PARTS", str(parts))
    monkeypatch.setenv("TT_WGRAD_ENGINE", str(engine))
    on_host["conv"].run_conv(12, 16, 272, 8, 8, 3, 3, 1, 3, True, "RRC", "rrR", "RRr", "RRC", "RRr", "112", "113", "332", 150 + parts)


def test_conv_shards_that_share_their_left_operand(on_host):
    on_host["conv"].test_shards_that_share_their_left_operand_run_as_one_product()


def test_conv_weight_gradient_of_shards_that_share_the_images(on_host):
    on_host["conv"].test_weight_gradient_of_shards_that_share_the_images_runs_as_one_product()


def test_conv_fp32(on_host):
    on_host["conv"].test_fp32_convolutions()


def test_conv_refusals(on_host):
    on_host["conv"].test_refusals()


@pytest.mark.parametrize("e", [1, 2, 4, 8])
def test_retile_all_pairs_two_cuts(on_host, e):
    on_host["convert"].test_retile_all_pairs_two_cuts(e)


def test_retile_ragged_deep_and_gated(on_host):
    c = on_host["convert"]
    c.test_retile_three_cuts_ragged_shapes()
    c.test_retile_k0_k4_and_roundtrip()
    c.test_retile_six_cuts()
    c.test_gated_retile("bf16")
    c.test_gated_retile("f32")


def test_reduce(on_host):
    c = on_host["convert"]
    c.test_reduce_ragged_columns_scalar_path()
    for forms, B, out, relu in [("3", "r", "f32", False), ("33", "RR", "bf16", True), ("13", "CR", "f32", True), ("32", "rC", "bf16", False),
                                ("333", "RRR", "bf16", False), ("231", "rCr", "f32", False), ("3333", "RRCC", "f32", False)]:
        c.test_reduce_against_oracle(forms, B, out, relu)


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_shard_products_small(on_host, ta, tb):
    g = on_host["gemm"]
    g.test_bf16_unaligned_falls_back(ta, tb)
    g.test_fp32(ta, tb)
    g.test_k_zero_and_empty()


def test_fc_backward_with_a_k_split_that_does_not_divide_into_whole_chunks(on_host):
    # the data gradient here is a skinny product over K = 1664 = 26 x 64 per shard; cut eight ways inside the launch the
    # chunks (rounded up to the tile depth) would be 256 deep and the last one and a half empty: the split has to stop at four
    on_host["fc"].run_layer(128, 96, 1664, 3, "bf16", False, "CRR", "rCr", "RRR", "rrr", "CCR", None, "212", "313", 1134)


def test_random_fc_layers(on_host):
    # seeded random sizes, stored tilings and form sequences, one to three cuts; requests the library declines as
    # infeasible or unsupported are skipped, any other status or a wrong value fails
    rng = np.random.default_rng(77)
    ran = 0
    for case in range(20):
        k = int(rng.choice([1, 2, 3, 3]))
        ts = tl.all_tilings(k)
        t = [ts[int(i)] for i in rng.integers(0, len(ts), 5)]
        f = [None if rng.random() < 0.5 else "".join(str(int(v)) for v in rng.integers(1, 4, k)) for _ in range(3)]
        mult = 1 << k
        b, ni, no = (mult * int(rng.integers(1, 12)) * int(rng.choice([1, 8])) for _ in range(3))
        dt = "bf16" if rng.random() < 0.7 else "f32"
        try:
            on_host["fc"].run_layer(b, ni, no, k, dt, bool(rng.integers(0, 2)), *t, *f, 3000 + case, with_dx=rng.random() < 0.85)
            ran += 1
        except binding.TilingError as e:
            assert e.status in (2, 3), (case, b, ni, no, k, dt, t, f, str(e))
    assert ran >= 10


def test_random_conv_layers(on_host):
    rng = np.random.default_rng(78)
    ran = 0
    for case in range(7):
        k = int(rng.choice([1, 2, 2, 3]))
        ts = tl.all_tilings(k)
        t = [ts[int(i)] for i in rng.integers(0, len(ts), 5)]
        f = [None if rng.random() < 0.5 else "".join(str(int(v)) for v in rng.integers(1, 4, k)) for _ in range(3)]
        mult = 1 << k
        N, C, K = mult * int(rng.integers(1, 3)), 8 * mult * int(rng.integers(1, 4)), 8 * mult * int(rng.integers(1, 4))
        H, W, pad = int(rng.integers(3, 8)), int(rng.integers(3, 8)), int(rng.integers(0, 3))
        R, S = int(rng.choice([1, 3, 5])), int(rng.choice([1, 3, 5]))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        try:
            on_host["conv"].run_conv(N, C, K, H, W, R, S, pad, k, bool(rng.integers(0, 2)), *t, *f, 4000 + case, with_dx=rng.random() < 0.85)
            ran += 1
        except binding.TilingError as e:
            assert e.status in (2, 3), (case, N, C, K, H, W, R, S, pad, k, t, f, str(e))
    assert ran >= 4


@pytest.mark.parametrize("relu", [False, True])
def test_fc_backward_overlapped_equals_backward(on_host, monkeypatch, relu):
    # the two-stream variant's own path (fork, weight gradient first, join) gives the very same bits
    from synthetic import normal_f32
    fc = on_host["fc"]
    monkeypatch.setattr(binding, "_stream", lambda s: ctypes.c_void_p(s if isinstance(s, int) else 0))
    b, ni, no, k, dt = 64, 512, 384, 3, "bf16"
    t = dict(X="CCr", W="RRC", Y="CCC", dY="CrC", dX="CCr")
    forms = ("233", "112")
    lay = binding.layer("fc", "relu" if relu else "none", ni, no)
    X, W, Y, dY = (fc.to_store(normal_f32(90, i, shape, s), dt) for i, shape, s in
                   ((0, (b, ni), 1.0), (1, (ni, no), 0.05), (3, (b, no), 1.0), (2, (b, no), 1.0)))
    Xs, Ws, Ys, dYs = (fc.shards_to_dev(a, tt_, True) for a, tt_ in ((X, t["X"]), (W, t["W"]), (Y, t["Y"]), (dY, t["dY"])))
    ref_dX, ref_dW, _ = fc._backward_once(binding.tt_fc_backward, lay, b, k, dt, t, forms, Xs, Ws, Ys, dYs, ni, no)
    got_dX, got_dW, _ = fc._backward_once(binding.tt_fc_backward_overlapped, lay, b, k, dt, t, forms, Xs, Ws, Ys, dYs, ni, no, aux_stream=16)
    for g, r in zip(got_dX + got_dW, ref_dX + ref_dW):
        assert torch.equal(g.view(torch.int16), r.view(torch.int16))
        assert not torch.isnan(g.float()).any()


def test_forward_with_the_library_s_own_scratch(on_host):
    import test_zz_no_alloc as na
    na.test_static_scratch_forward_twice_second_smaller()
    na.test_static_scratch_refuses_what_does_not_fit()


def test_random_reductions_and_gated_retiles(on_host):
    # partial sums of random form sequences reduced into random stored tilings (fp32 and bf16 results, with and without
    # relu), and dY gated by Y > 0 on its way between random tilings: against the oracle, sizes with ragged vector tails
    import paper_1805_04170_amd as tt
    from gpu_util import alloc_shards, dev_to_np, np_to_dev, shards_to_dev, shards_to_np
    from oracle import execute as ex
    from synthetic import bf16_bits_to_f32, to_bf16_bits
    rng = np.random.default_rng(91)
    for case in range(30):
        k = int(rng.choice([1, 2, 3, 4]))
        forms = "".join(str(int(v)) for v in rng.integers(1, 4, k))
        B = "".join("RCr"[int(v)] for v in rng.integers(0, 3, k))
        mult = 1 << k
        rows, cols = mult * int(rng.integers(1, 9)), mult * int(rng.integers(1, 40))
        out, relu = ("bf16" if rng.integers(0, 2) else "f32"), bool(rng.integers(0, 2))
        k1, k2 = forms.count("1"), forms.count("2")
        parts = [rng.standard_normal((rows >> k1, cols >> k2)).astype(np.float32) for _ in range(mult)]
        want = ex.reduce_to([p.astype(np.float64) for p in parts], forms, B, rows, cols, relu)
        dst = alloc_shards(rows, cols, B, torch.bfloat16 if out == "bf16" else torch.float32)
        tt.tt_reduce(dst, B, out, [np_to_dev(p) for p in parts], forms, rows, cols, tt.TT_ACT_RELU if relu else tt.TT_ACT_NONE)
        mag = ex.assemble([np.abs(p).astype(np.float64) for p in parts], forms, rows, cols)
        for s, (d, w) in enumerate(zip(dst, want)):
            g = dev_to_np(d)
            gf = bf16_bits_to_f32(g).astype(np.float64) if out == "bf16" else g.astype(np.float64)
            tol = 1e-5 * mag[tl.shard_slices(rows, cols, B, s)] + (2.0 ** -8 * np.abs(w) if out == "bf16" else 0.0)
            assert np.all(np.abs(gf - w) <= tol + 1e-30), (case, forms, B, rows, cols, out, relu, s)
    for case in range(20):
        k = int(rng.choice([1, 2, 3]))
        tA, tM, tB = ("".join("RCr"[int(v)] for v in rng.integers(0, 3, k)) for _ in range(3))
        mult = 1 << k
        rows, cols = mult * int(rng.integers(1, 9)), mult * int(rng.integers(1, 40))
        bf = bool(rng.integers(0, 2))
        v = rng.standard_normal((rows, cols)).astype(np.float32)
        m = rng.standard_normal((rows, cols)).astype(np.float32)
        m[rng.random((rows, cols)) < 0.3] = 0.0
        if bf:
            v, m = to_bf16_bits(v), to_bf16_bits(m)
        mf = bf16_bits_to_f32(m) if bf else m
        want_full = np.where(mf > 0, v, np.zeros_like(v))
        dst = alloc_shards(rows, cols, tB, torch.bfloat16 if bf else torch.float32, fill=float("nan"))
        tt.tt_retile_gate(dst, tB, shards_to_dev(v, tA, bf), tA, shards_to_dev(m, tM, bf), tM, rows, cols, "bf16" if bf else "f32")
        got = tl.untile(shards_to_np(dst), tB, rows, cols)
        u = np.uint16 if bf else np.uint32
        assert np.array_equal(got.view(u), want_full.view(u)), (case, tA, tM, tB, rows, cols, bf)


def test_flatten_between_convolution_and_fully_connected(on_host):
    on_host["net"].test_flatten_every_tiling_pair_two_cuts()
    on_host["net"].test_flatten_tile_tails_and_sizes()
    on_host["net"].test_flatten_refusals()


def test_convolution_flatten_fully_connected_network(on_host):
    on_host["net"].test_conv_flatten_fc_fc_under_the_planners_tiling()
