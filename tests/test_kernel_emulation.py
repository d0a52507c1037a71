"""Memory-access check of the tile engines without a GPU: the kernels' own headers are compiled for the host (every
thread of every workgroup run in turn, tests/emu/), and every global read, global -> LDS load, LDS access and output
store must stay inside the buffers of the launch; every output element must be written.  The launch geometry comes from
the same host code the launchers use.  This checks index arithmetic, not values (the stand-in MFMA multiplies nothing)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = shutil.which("clang++", path="/opt/rocm/llvm/bin") or shutil.which("clang++")
pytestmark = pytest.mark.skipif(CLANG is None, reason="no host clang++ for the emulation build")


@pytest.fixture(scope="module")
def emu(emulators):
    return emulators.get("gemm3")


def run(exe, case, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([exe] + [str(v) for v in case], capture_output=True, text=True, env=e)


# engine, count, M, N, K, a_kc, b_kc, out_bf16, relu, ksplit
CASES = [
    (3, 8, 1544, 1528, 128, 1, 0, 1, 1, 1),     # the shapes of the GPU tests of the persistent engine, all four layouts
    (3, 8, 1032, 1544, 64, 1, 1, 0, 0, 1),
    (3, 3, 2056, 1800, 320, 0, 1, 1, 0, 1),
    (3, 8, 2056, 2312, 256, 0, 0, 1, 1, 1),
    # (the three products of the VGG-16 first classifier layer run below, through tt_shard_gemm and in the benchmark step)
    (3, 16, 512, 2048, 2048, 1, 1, 1, 0, 1),    # wide MLP shard product
    (3, 2, 520, 776, 64, 0, 0, 1, 0, 1),
    (3, 1, 264, 1000, 192, 1, 0, 1, 0, 1),      # 1000 columns: ragged last tile, 16-byte rows
    (3, 1, 264, 1004, 128, 1, 1, 0, 0, 1),      # fp32 rows of 1004
    (2, 8, 1000, 1016, 200, 0, 0, 1, 1, 1),     # ragged M, N and K (K tail read as zero chunks)
    (2, 8, 1024, 1024, 192, 0, 1, 0, 0, 1),
    (2, 1, 520, 264, 72, 1, 1, 1, 0, 1),
    (4, 2, 520, 520, 96, 1, 1, 1, 1, 1),        # the 256 x 128 engine: shapes of its GPU tests and of the hidden layers
    (4, 8, 256, 1024, 512, 0, 0, 0, 0, 1),
    (4, 1, 136, 264, 32, 1, 0, 1, 0, 1),
    (4, 8, 256, 2048, 1024, 1, 0, 0, 0, 1),
    (4, 8, 256, 1000, 512, 1, 0, 0, 0, 1),
    (4, 8, 512, 1000, 256, 0, 0, 1, 0, 1),
    (4, 4, 264, 520, 160, 0, 1, 0, 0, 2),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "e%d_%dx%dx%dx%d_%d%d%d_k%d" % (c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], c[9]))
def test_every_access_of_the_launch_stays_inside_its_buffers(emu, case):
    r = run(emu, case)
    assert r.returncode == 0, r.stdout[-400:] + r.stderr[-1200:]
    assert r.stdout.startswith("ok engine")


def test_the_checker_sees_an_access_past_the_end(emu):
    # the same launch with the last 16 bytes of every operand declared out of bounds must be reported
    r = run(emu, (3, 2, 520, 776, 64, 0, 0, 1, 0, 1), env={"EMU_SHRINK": "1"})
    assert r.returncode != 0 and "EMU FAULT: global read outside every operand" in r.stderr


def test_products_the_engines_do_not_take_are_refused_by_the_launch_code(emu):
    assert run(emu, (3, 1, 264, 264, 96, 1, 1, 1, 0, 1)).returncode == 2      # K not a multiple of 64
    assert run(emu, (4, 1, 264, 260, 64, 1, 0, 1, 0, 1)).returncode == 2      # row-contiguous B with N not a multiple of 8
    assert run(emu, (3, 1, 4, 264, 64, 1, 1, 1, 0, 1)).returncode == 2        # fewer than eight rows


# the register-staged engine: one kernel configuration per build
# (BM, BN, WM, WN, DEPTH, KMASK, A_KC, B_KC, BF16, VEC), (count, M, N, K, relu, ksplit)
CASES1 = [
    ((128, 128, 2, 2, 1, 1, 1, 1, 0, 1), (8, 256, 512, 1000, 0, 1)),     # data gradient of the last VGG-16 classifier layer
    ((128, 128, 2, 2, 1, 1, 0, 0, 1, 1), (1, 520, 72, 40, 0, 1)),        # three row tiles, one short K tile, both operands transposed in registers
    ((128, 128, 2, 2, 1, 0, 1, 1, 1, 0), (2, 128, 132, 64, 1, 1)),       # element-wise stores (rows of 132 bf16; both operands K-contiguous, as the launcher demands of a product whose N is no multiple of 8)
    ((256, 128, 2, 2, 2, 0, 1, 0, 1, 1), (1, 264, 264, 1024, 0, 1)),     # deep-prefetch variant
    ((256, 256, 2, 4, 1, 1, 1, 0, 1, 1), (8, 1000, 1016, 200, 1, 1)),    # eight waves, ragged everything
    ((128, 128, 2, 2, 0, 0, 0, 1, 0, 1), (2, 136, 264, 256, 0, 2)),      # single LDS buffer, in-shard K split
]


@pytest.mark.parametrize("cfg,case", CASES1, ids=lambda v: "x".join(str(i) for i in v))
def test_register_staged_engine_stays_inside_its_buffers(emulators, cfg, case):
    emulators.prefetch([("gemm1", c) for c, _ in CASES1])
    exe = emulators.get(("gemm1", cfg))
    r = run(exe, case)
    assert r.returncode == 0, r.stdout[-400:] + r.stderr[-1200:]


# ---- the conversion kernels with their launch code: tt_retile / tt_retile_gate / tt_reduce run on host buffers and are
# compared bit for bit with what the oracle expects (same cases as the GPU tests, plus sizes that take the launches with
# two and four vectors per lane)

import itertools

import numpy as np

from oracle import execute as ex
from oracle import tiling as tl
from synthetic import bf16_bits_to_f32, to_bf16_bits


@pytest.fixture(scope="module")
def emu_convert(emulators):
    return emulators.get("convert")


def _dump(d, stem, shards):
    for i, sh in enumerate(shards):
        np.ascontiguousarray(sh).tofile(os.path.join(d, "%s%d.bin" % (stem, i)))


def _call(exe, d, *args):
    r = subprocess.run([exe, str(d)] + [str(a) if a != "" else "-" for a in args], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-300:] + r.stderr[-1500:]
    return r.stdout


def test_retile_on_the_host_is_bit_exact(emu_convert, tmp_path):
    rng = np.random.default_rng(5)
    NP = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}
    cases = []
    for e in (1, 2, 4, 8):                                   # every pair of two-cut tilings, every element size
        T = rng.integers(0, 256, size=(24, 40 * e), dtype=np.uint8).view(NP[e]).reshape(24, 40)
        for A, B in itertools.product(tl.all_tilings(2), repeat=2):
            cases.append((T, A, B, e))
    T3 = rng.integers(0, 1 << 16, size=(200, 1000), dtype=np.uint16)   # 125-wide shards: 8-, 4- and 2-byte vectors
    ts = tl.all_tilings(3)
    for ia, ib in rng.choice(len(ts), size=(25, 2)):
        cases.append((T3, ts[ia], ts[ib], 2))
    big = rng.integers(0, 1 << 16, size=(512, 4096), dtype=np.uint16)   # 256 K vectors: two per lane
    cases += [(big, "RC", "CR", 2), (big, "RRC", "Crr", 2)]
    bigger = rng.integers(0, 1 << 16, size=(1024, 4104), dtype=np.uint16)  # four per lane, ragged tail of workgroups
    cases += [(bigger, "RC", "CR", 2)]
    cases += [(T3[:64, :96], "", "", 2), (T3[:64, :96].copy(), "RCRC", "CRrR", 2), (T3[:64, :64].copy(), "RCRCRC", "CRCRCR", 2)]
    for n, (T, A, B, e) in enumerate(cases):
        d = tmp_path / ("r%d" % n)
        d.mkdir()
        _dump(d, "src", tl.tile(T, A))
        _dump(d, "exp", tl.tile(T, B))
        _call(emu_convert, d, "retile", len(A), T.shape[0], T.shape[1], e, A, B)


def test_gated_retile_and_reduce_on_the_host(emu_convert, tmp_path):
    rng = np.random.default_rng(6)
    n = 0
    for rows, cols in ((48, 80), (512, 1032)):
        v = rng.standard_normal((rows, cols)).astype(np.float32)
        m = rng.standard_normal((rows, cols)).astype(np.float32)
        m[rng.random((rows, cols)) < 0.3] = 0.0
        for bf in (True, False):
            V = to_bf16_bits(v) if bf else v
            Mk = to_bf16_bits(m) if bf else m
            mf = bf16_bits_to_f32(Mk) if bf else Mk
            want = np.where(mf > 0, V, np.zeros_like(V))
            for A, Am, B in [("RR", "CC", "Rr"), ("Cr", "rR", "CC"), ("rr", "RC", "RC")]:
                d = tmp_path / ("g%d" % n)
                n += 1
                d.mkdir()
                _dump(d, "src", tl.tile(V, A))
                _dump(d, "msk", tl.tile(Mk, Am))
                _dump(d, "exp", tl.tile(want, B))
                _call(emu_convert, d, "gate", 2, rows, cols, 1 if bf else 0, A, Am, B)
    # partial-sum reduction: fp32 sums in the kernel's fixed order (increasing partial number), then ReLU, then the cast
    for forms, B, out_bf16, relu, rows, cols in [("31", "RC", True, True, 32, 48), ("33", "rR", False, False, 32, 48),
                                                 ("313", "CRr", True, False, 64, 64), ("12", "CR", True, True, 32, 48),
                                                 ("3", "R", False, True, 512, 4096), ("33", "RC", True, False, 1024, 4096)]:
        k = len(forms)
        grid = ex.output_grid_tiling(forms)
        parts = [rng.standard_normal(tl.shard_shape(rows, cols, grid)).astype(np.float32) for _ in range(1 << k)]
        Z = np.zeros((rows, cols), dtype=np.float32)
        for s, p in enumerate(parts):                      # shard s adds into its block; ids in increasing order
            sl = tl.shard_slices(rows, cols, grid, s)
            Z[sl] = Z[sl] + p
        if relu:
            Z = np.maximum(Z, np.float32(0))
        want = to_bf16_bits(Z) if out_bf16 else Z
        d = tmp_path / ("s%d" % n)
        n += 1
        d.mkdir()
        _dump(d, "src", parts)
        _dump(d, "exp", tl.tile(want, B))
        _call(emu_convert, d, "reduce", k, rows, cols, 1 if out_bf16 else 0, 1 if relu else 0, forms, B)


# ---- the convolution kernels with their launch code (tile choice, grids, the filter flip in front of the data gradient)

@pytest.fixture(scope="module")
def emu_conv(emulators):
    return emulators.get("conv")


# op (0 forward, 1 data gradient, 2 filter gradient), shards, images, in-channels, out-channels per shard, H, W, R, S, pad,
# bf16 output, relu, filters flipped first
CONV_CASES = [
    (0, 8, 8, 512, 512, 28, 28, 3, 3, 1, 1, 0, 0),     # VGG-16 conv4 cut along the batch: the three benchmark launches
    (1, 8, 8, 512, 512, 28, 28, 3, 3, 1, 1, 0, 1),
    (2, 8, 8, 512, 512, 28, 28, 3, 3, 1, 0, 0, 0),
    (0, 8, 64, 512, 64, 28, 28, 3, 3, 1, 1, 1, 0),     # ... cut along the output channels
    (1, 8, 64, 512, 64, 28, 28, 3, 3, 1, 0, 0, 1),     # (its data gradient splits the reduction: fp32 partial sums)
    (2, 8, 64, 512, 64, 28, 28, 3, 3, 1, 1, 0, 0),
    (1, 2, 2, 16, 24, 9, 9, 3, 3, 1, 1, 0, 0),         # data gradient on its own kernel (filters transposed in registers)
    (1, 2, 2, 16, 24, 9, 9, 3, 3, 1, 1, 0, 1),         # ... and through the element-wise flip (channel counts not multiples of 64)
    (0, 2, 3, 8, 16, 7, 5, 5, 1, 2, 0, 0, 0),          # 5 x 1 filter, padding 2, odd image
    (2, 2, 3, 8, 16, 7, 5, 1, 5, 2, 0, 0, 0),
    (0, 1, 1, 8, 8, 6, 6, 5, 5, 0, 1, 1, 0),           # 25 taps, no padding
    (0, 4, 2, 64, 64, 12, 12, 1, 1, 0, 1, 0, 0),       # 1 x 1 filter: the one-tap loader
    (1, 4, 2, 64, 64, 12, 12, 1, 1, 0, 1, 0, 1),
    # filter gradient with the reduction range of every block cut into equal runs (after pad: runs, shards per block,
    # tile engine):
    (3, 8, 8, 512, 512, 28, 28, 3, 3, 1, 7, 8, 1),     # conv4 cut along the batch: seven runs over the eight shards
    (3, 8, 8, 512, 512, 28, 28, 3, 3, 1, 7, 8, 2),
    (3, 8, 64, 64, 512, 28, 28, 3, 3, 1, 6, 1, 1),     # conv4 with the input channels cut: runs inside every shard
    (3, 8, 64, 64, 512, 28, 28, 3, 3, 1, 8, 1, 2),
    (3, 4, 3, 16, 136, 8, 8, 3, 3, 1, 5, 2, 1),        # runs of unequal length that cross from one shard into the next
    (3, 4, 3, 16, 136, 8, 8, 3, 3, 1, 5, 2, 2),
    (3, 8, 1, 8, 264, 8, 8, 3, 3, 1, 3, 8, 1),         # a run over three shards; two row tiles
    (3, 8, 1, 8, 264, 8, 8, 3, 3, 1, 3, 8, 2),
    (3, 2, 64, 8, 136, 7, 5, 5, 3, 2, 3, 2, 2),        # 7 x 5 images, 5 x 3 filter, padding 2: 49 output pixels per image
    (3, 2, 64, 8, 136, 7, 5, 5, 3, 2, 3, 2, 1),
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "op%d_%dx%dx%dx%d_%dx%d_%dx%d" % (c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], c[8]))
def test_convolution_launches_stay_inside_their_buffers(emu_conv, case):
    r = run(emu_conv, case)
    assert r.returncode == 0, r.stdout[-400:] + r.stderr[-1500:]


# ---- the shard-product entry point with its launch code: which engine and tile a shape gets is decided by the same
# ---- code as in the library, on a device with 256 compute units

@pytest.fixture(scope="module")
def emu_shard_gemm(emulators):
    return emulators.get("shard_gemm")


# shards, M, N, K, A transposed, B transposed, bf16 operands, bf16 result, relu, K split inside the launch;
# then the number of threads the launch must have run (which names the engine: workgroups x their size)
SHARD_CASES = [
    ((8, 256, 512, 4096, 0, 0, 1, 1, 1, 1), 32 * 256),      # hidden layer forward at batch 256: 256 x 128 tiles, two workgroups per CU
    ((8, 256, 3136, 4096, 0, 1, 1, 1, 0, 1), 200 * 256),    # VGG-16 first data gradient, not split: 200 tiles of 256 x 128, K tiles of 64
    ((8, 256, 1024, 2048, 0, 1, 1, 0, 0, 1), 64 * 256),     # ... second one, fp32 partial sums: too few tiles for that, K tiles of 32
    ((8, 256, 4608, 1024, 0, 1, 1, 1, 0, 1), 288 * 256),    # AlexNet first data gradient: more tiles than CUs, K tiles of 32, two workgroups per CU
    ((8, 256, 4096, 3136, 0, 0, 1, 0, 0, 1), 256 * 256),    # ... first forward product (fp32 partial sums of the F3 cuts): one workgroup per CU
    ((8, 3136, 4096, 256, 1, 0, 1, 1, 0, 1), 512 * 256),    # VGG-16 first weight gradient: the panel-in-registers engine, two workgroups of four waves per CU
    ((8, 1152, 4096, 128, 1, 0, 1, 1, 0, 1), 512 * 256),    # the same engine at a per-shard batch of 128
    ((8, 1024, 2048, 256, 1, 0, 1, 1, 0, 1), 512 * 256),    # ... and at the second VGG-16 weight gradient: two units per workgroup
    ((16, 1024, 2048, 512, 1, 0, 1, 1, 0, 1), 256 * 256),   # weight gradient at a per-shard batch of 512 (half a wide-MLP shard): the same engine, one workgroup per CU
    ((8, 1568, 4096, 192, 1, 0, 1, 1, 0, 1), 256 * 512),    # a batch it does not take: the persistent engine, one workgroup per CU
    ((16, 256, 4096, 512, 0, 1, 1, 0, 0, 1), 256 * 512),    # skinny data gradient: 256 x 256 tiles loaded straight into LDS
    ((16, 256, 2048, 512, 0, 0, 1, 0, 0, 1), 128 * 512),    # skinny NN product: the persistent engine, 128 tiles
    ((4, 256, 128, 1024, 0, 0, 1, 1, 0, 1), 8 * 256),       # one narrow column of tiles: register-staged 256 x 128
    ((3, 64, 64, 72, 0, 0, 1, 0, 1, 1), 8 * 256),           # small product, K not a multiple of the tile depth: 128 x 128 with K mask
    ((3, 50, 70, 33, 0, 1, 0, 0, 0, 1), 6 * 256),           # fp32 operands: the scalar kernel, 64 x 64 tiles
    ((2, 296, 264, 200, 1, 0, 1, 1, 0, 1), None),           # ragged tiles on every side
    ((8, 256, 512, 72, 0, 0, 1, 1, 0, 1), None),            # K the 256 x 128 engine refuses: falls through to the register-staged one
    ((4, 256, 512, 3136, 0, 0, 1, 0, 0, 4), 64 * 256),      # reduction split four ways inside one launch, sixteen partial products
    ((2, 40, 24, 300, 1, 1, 1, 1, 0, 3), None),             # the same on the smallest tile
]


@pytest.mark.parametrize("case,threads", SHARD_CASES, ids=lambda c: "x".join(map(str, c)) if isinstance(c, tuple) else None)
def test_shard_product_entry_point_stays_inside_its_buffers(emu_shard_gemm, case, threads):
    r = run(emu_shard_gemm, case)
    assert r.returncode == 0, r.stdout[-400:] + r.stderr[-1500:]
    assert r.stdout.startswith("ok shard_gemm")
    if threads is not None:
        assert int(r.stdout.split()[2]) == threads, r.stdout


def test_shard_product_entry_point_rejects_what_the_library_rejects(emu_shard_gemm):
    # a K split that would leave the last chunk empty (chunks are rounded up to the tile depth: two of 64 cover K = 128)
    r = run(emu_shard_gemm, (2, 64, 64, 128, 0, 0, 1, 0, 0, 3))
    assert r.returncode == 2 and "status" in r.stdout


# ---- a whole training step through the execute calls (planning of conversions, workspace layout, every launch of the
# ---- forward and backward pass), with shards and workspace of exactly the sizes the library asks for

import paper_1805_04170_amd as tt
from synthetic import CONFIGS


@pytest.fixture(scope="module")
def emu_step(emulators):
    return emulators.get("step")


def _t(s):
    return s if s else "-"


def fc_step_args(batch, k, dtype, widths, relus, tx, tg, tw, forms):
    L = len(widths) - 1
    return (["fc", batch, k, dtype, L] + list(widths) + [int(r) for r in relus] + [_t(t) for t in tx] + [_t(t) for t in tg] +
            [_t(t) for t in tw] + [_t(f) if f else "-" for lf in forms for f in lf])


def planned_fc_step(cfg, mode=tt.TT_PLAN_EXACT):
    L = cfg.n_layers
    plan = tt.tt_plan_chain([tt.layer("fc", "none", cfg.widths[l], cfg.widths[l + 1]) for l in range(L)], cfg.batch, cfg.k, mode)
    forms = [[plan.forms(l, op) for op in range(3)] for l in range(1, L + 1)]
    return fc_step_args(cfg.batch, cfg.k, cfg.dtype, cfg.widths, [cfg.act(l) for l in range(1, L + 1)], plan.x(), plan.g(), plan.w(), forms)


@pytest.mark.parametrize("name", ["tiny_mlp", "vgg16_fc", "alexnet_fc"])
def test_benchmark_step_stays_inside_its_buffers(emu_step, name):
    # the step bench.py times, at its full size: planner tilings and forms, overlapped backward
    r = run(emu_step, planned_fc_step(CONFIGS[name]))
    assert r.returncode == 0 and r.stdout.startswith("ok fc step"), r.stdout[-400:] + r.stderr[-1500:]


def test_the_step_checker_sees_a_workspace_that_is_too_short(emu_step):
    # a step that needs its workspace (a reduction-split product), told the truth and then given 256 bytes less
    args = fc_step_args(64, 2, "bf16", (72, 136, 40), (True, False), ["CC", "CC", "CC"], ["rr", "CC", "CC"], ["RR", "RR"], [[None] * 3] * 2)
    assert run(emu_step, args).returncode == 0
    r = run(emu_step, args, env={"EMU_WS_LIE": "256"})
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr


def test_steps_under_random_tilings_stay_inside_their_buffers(emu_step):
    # conversions in front of and behind every product, reductions of every depth: random stored tilings, default forms
    rng = np.random.default_rng(11)
    for k in (1, 2, 3):
        ts = tl.all_tilings(k)
        for _ in range(6):
            tx = [ts[i] for i in rng.integers(0, len(ts), 3)]
            tg = [ts[i] for i in rng.integers(0, len(ts), 3)]
            tw = [ts[i] for i in rng.integers(0, len(ts), 2)]
            dt = "bf16" if rng.integers(0, 2) else "f32"
            args = fc_step_args(64, k, dt, (96, 1000, 40) if k == 3 else (72, 136, 40), (True, False), tx, tg, tw, [[None] * 3] * 2)
            r = run(emu_step, args)
            assert r.returncode == 0 and r.stdout.startswith("ok fc step"), (args, r.stdout[-400:] + r.stderr[-1500:])


def conv_step_args(N, k, C, K, H, W, R, S, pad, relu, t, f):
    return ["conv", N, k, C, K, H, W, R, S, pad, int(relu)] + [_t(t[n]) for n in ("X", "W", "Y", "dY", "dX")] + [x if x else "-" for x in f]


@pytest.mark.parametrize("split", ["planner", "batch", "out_channel"])
def test_convolution_step_stays_inside_its_buffers(emu_step, split):
    # the three splits bench.py offers for a convolution layer, on a layer small enough for every split to run in seconds
    N, k, C, K, H, W = 16, 3, 64, 256 if split == "out_channel" else 128, 12, 12   # 256: the merged weight gradient
    lay = tt.layer("conv", "none", C, K, H=H, W=W, R=3, S=3, pad=1)
    if split == "planner":
        p = tt.tt_plan_chain([lay], N, k)
        t = dict(X=p.x()[0], Y=p.x()[1], W=p.w()[0], dY=p.g()[1], dX=p.g()[0])
        f = [p.forms(1, o) for o in range(3)]
    elif split == "batch":
        t = dict(X="R" * k, Y="R" * k, W="r" * k, dY="R" * k, dX="R" * k)
        f = ["1" * k, "1" * k, "3" * k]
    else:
        t = dict(X="r" * k, Y="C" * k, W="C" * k, dY="C" * k, dX="r" * k)
        f = ["2" * k, "3" * k, "2" * k]
    r = run(emu_step, conv_step_args(N, k, C, K, H, W, 3, 3, 1, True, t, f))
    assert r.returncode == 0 and r.stdout.startswith("ok conv step"), r.stdout[-400:] + r.stderr[-1500:]


def test_convolution_benchmark_step_stays_inside_its_buffers(emu_step):
    # vgg16_conv4 at full size under the planner's tiling, as bench.py runs it
    c = CONFIGS["vgg16_conv4"]
    lay = tt.layer("conv", "none", c.C, c.K, H=c.H, W=c.W, R=c.R, S=c.S, pad=c.pad)
    p = tt.tt_plan_chain([lay], c.N, c.k)
    t = dict(X=p.x()[0], Y=p.x()[1], W=p.w()[0], dY=p.g()[1], dX=p.g()[0])
    r = run(emu_step, conv_step_args(c.N, c.k, c.C, c.K, c.H, c.W, c.R, c.S, c.pad, False, t, [p.forms(1, o) for o in range(3)]))
    assert r.returncode == 0 and r.stdout.startswith("ok conv step"), r.stdout[-400:] + r.stderr[-1500:]


def test_convolution_steps_under_random_tilings_stay_inside_their_buffers(emu_step):
    rng = np.random.default_rng(12)
    ts = tl.all_tilings(2)
    for i in range(8):
        t = {n: ts[j] for n, j in zip(("X", "W", "Y", "dY", "dX"), rng.integers(0, len(ts), 5))}
        r = run(emu_step, conv_step_args(4, 2, 32, 64, 9, 9, 3, 3, 1, bool(i % 2), t, [None] * 3))
        assert r.returncode == 0 and r.stdout.startswith("ok conv step"), (t, r.stdout[-400:] + r.stderr[-1500:])
