"""The shard-product kernels run on the host in lock step (tests/emu/emu_lockstep.h: the threads of a workgroup as
cooperative fibers, barriers that hold, MFMA and the LDS transpose read computing what the instructions compute) and
their results compared with the oracle's, to the bar of the GPU tests.  The entry point is the library's own
(csrc/gemm.hip and csrc/gemm3.hip compiled for the host as they are), so every engine is reached the way the library
reaches it.  What this cannot show is what only the hardware decides (timing, instruction alignment rules); what it does
show without a GPU: tile and fragment indexing, LDS layouts, K tails, write-out, the K split inside a launch.
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import layers as ly
from synthetic import bf16_bits_to_f64, normal_f32, to_bf16_bits

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = shutil.which("clang++", path="/opt/rocm/llvm/bin") or shutil.which("clang++")
pytestmark = pytest.mark.skipif(CLANG is None, reason="no host clang++ for the emulation build")


@pytest.fixture(scope="module")
def lockstep_gemm(emulators):
    return emulators.get("shard_gemm_lockstep")


def check(exe, tmp, count, M, N, K, ta, tb, in_dt, out_dt, relu, seed, ksplit=1, env=None):
    bf = in_dt == "bf16"
    want, mags = [], []
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
        np.ascontiguousarray(a.T if ta else a).tofile(os.path.join(tmp, "a%d.bin" % s))
        np.ascontiguousarray(b.T if tb else b).tofile(os.path.join(tmp, "b%d.bin" % s))
    e = dict(os.environ)
    e.update(env or {})
    r = subprocess.run([exe] + [str(v) for v in (count, M, N, K, ta, tb, int(bf), int(out_dt == "bf16"), int(relu), ksplit, tmp)],
                       capture_output=True, text=True, env=e)
    assert r.returncode == 0, r.stdout[-400:] + r.stderr[-1500:]
    for s in range(count):
        # with a K split the launch leaves ksplit partial products per shard, to be summed
        gf = np.zeros((M, N))
        for q in range(ksplit):
            raw = np.fromfile(os.path.join(tmp, "c%d.bin" % (s * ksplit + q)), dtype=np.uint16 if out_dt == "bf16" else np.float32)
            gf += (bf16_bits_to_f64(raw) if out_dt == "bf16" else raw.astype(np.float64)).reshape(M, N)
        tol = (1e-2 if bf else 1e-5) * mags[s]
        err = np.abs(gf - want[s])
        assert np.all(np.isfinite(gf)), (s, "non-finite output")
        assert np.all(err <= tol + 1e-30), (s, float(err.max()), float((err / (tol + 1e-30)).max()), np.argwhere(err > tol + 1e-30)[:5])
        if bf and out_dt == "f32" and not relu:
            assert float(np.max(err / (mags[s] + 1e-30))) < 1e-4
    return r.stdout


LAYOUTS = [(0, 0), (0, 1), (1, 0), (1, 1)]


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_register_staged_engine_values(lockstep_gemm, tmp_path, ta, tb):
    check(lockstep_gemm, str(tmp_path), 2, 264, 200, 104, ta, tb, "bf16", "bf16", False, 31)   # ragged on every side, K mask
    check(lockstep_gemm, str(tmp_path), 1, 136, 72, 64, ta, tb, "bf16", "f32", True, 32)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
@pytest.mark.parametrize("out_dt", ["bf16", "f32"])
def test_two_workgroups_per_cu_engine_values(lockstep_gemm, tmp_path, ta, tb, out_dt):
    # few 256 x 256 tiles: the 256 x 128 engine; ragged M and N, a K loop shorter than its ring and a longer one
    out = check(lockstep_gemm, str(tmp_path), 1, 264, 392, 96, ta, tb, "bf16", out_dt, True, 45)
    assert int(out.split()[3]) == 8 * 256      # 2 x 4 tiles of 256 x 128, 256 threads each
    check(lockstep_gemm, str(tmp_path), 2, 136, 264, 32, ta, tb, "bf16", out_dt, False, 47)
    check(lockstep_gemm, str(tmp_path), 1, 256, 256, 256, ta, tb, "bf16", out_dt, False, 46)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
@pytest.mark.parametrize("out_dt", ["bf16", "f32"])
def test_persistent_engine_values(lockstep_gemm, tmp_path, ta, tb, out_dt):
    # on a stand-in device of 16 CUs, with the engine and tile forced the way the tuning switches allow: 24 ragged
    # tiles, one or two per workgroup (the operand ring runs across tile boundaries), K loops of one and three tiles
    env = {"EMU_CUS": "16", "TT_GEMM_ENGINE": "3", "TT_GEMM_TILE": "5"}
    out = check(lockstep_gemm, str(tmp_path), 2, 520, 776, 64, ta, tb, "bf16", out_dt, True, 42, env=env)
    assert int(out.split()[3]) == 16 * 512
    check(lockstep_gemm, str(tmp_path), 1, 264, 520, 192, ta, tb, "bf16", out_dt, False, 44, env=env)


@pytest.mark.parametrize("tb", [1, 0])
@pytest.mark.parametrize("out_dt", ["bf16", "f32"])
def test_line_wide_k_tiles_engine_values(lockstep_gemm, tmp_path, out_dt, tb):
    # the 256 x 128 engine with K tiles of 64 for A B^T products (two stages of A, three of B, waits that count loads):
    # ragged M and N, K loops of one tile (shorter than either ring), three and seven tiles, a K split inside the launch
    env = {"TT_GEMM_ENGINE": "6"}
    out = check(lockstep_gemm, str(tmp_path), 1, 264, 392, 192, 0, tb, "bf16", out_dt, True, 48, env=env)
    assert int(out.split()[3]) == 8 * 256      # 2 x 4 tiles of 256 x 128, 256 threads each
    check(lockstep_gemm, str(tmp_path), 2, 136, 264, 64, 0, tb, "bf16", out_dt, False, 49, env=env)
    check(lockstep_gemm, str(tmp_path), 1, 256, 256, 448, 0, tb, "bf16", out_dt, False, 50, env=env)
    if out_dt == "f32":
        check(lockstep_gemm, str(tmp_path), 2, 256, 136, 320, 0, tb, "bf16", "f32", False, 51, ksplit=2, env=env)   # chunks of 192 and 128


def test_line_wide_k_tiles_engine_as_the_library_chooses_it(lockstep_gemm, tmp_path):
    # a skinny data-gradient shaped product (one row of tiles, 128 of them for 256 CUs, K of four tiles): no switch set
    check(lockstep_gemm, str(tmp_path), 32, 256, 392, 256, 0, 1, "bf16", "bf16", False, 52)


def test_line_wide_k_tiles_engine_waits_exactly_as_long_as_it_must(lockstep_gemm, tmp_path):
    # with every wait letting two more loads stay in flight than the kernel asks for it must not get away with it; and
    # its results do not depend on which wave runs ahead
    env = {"TT_GEMM_ENGINE": "6"}
    shape = (1, 264, 392, 320, 0, 1, "bf16", "f32", False, 53)
    check(lockstep_gemm, str(tmp_path), *shape, env=env)
    with pytest.raises(AssertionError):
        check(lockstep_gemm, str(tmp_path), *shape, env=dict(env, EMU_VMCNT_SLACK="2"))
    check(lockstep_gemm, str(tmp_path), *shape, env=dict(env, EMU_ORDER="reverse"))


def test_persistent_engine_values_as_the_library_chooses_it(lockstep_gemm, tmp_path):
    # 240 tiles on 256 CUs: the weight-gradient layout, bf16 results (loads interleaved with the K steps)
    out = check(lockstep_gemm, str(tmp_path), 8, 1288, 1272, 64, 1, 0, "bf16", "bf16", False, 43)
    assert int(out.split()[3]) == 240 * 512


@pytest.mark.parametrize("relu", [False, True])
def test_panel_in_registers_engine_values(lockstep_gemm, tmp_path, relu):
    # the short-K engine of the weight gradients (left operand's panel in registers, stores left in flight over the next
    # unit's wait), forced on small products on a stand-in device of one CU (two workgroups): K = 256, two shards of two
    # panels (the second with 72 of its 256 rows: one wave full, one partly masked, two idle) by three column tiles, so
    # every workgroup changes panel and runs units behind stores that are still counted; then K = 128
    env = {"EMU_CUS": "1", "TT_GEMM_ENGINE": "5"}
    out = check(lockstep_gemm, str(tmp_path), 2, 328, 192, 256, 1, 0, "bf16", "bf16", relu, 81, env=env)
    assert int(out.split()[3]) == 2 * 256
    check(lockstep_gemm, str(tmp_path), 1, 264, 128, 128, 1, 0, "bf16", "bf16", relu, 82, env=env)
    # more workgroups than units to spare: runs of one unit, and a run that ends inside a panel
    check(lockstep_gemm, str(tmp_path), 1, 512, 320, 256, 1, 0, "bf16", "bf16", relu, 83, env={"EMU_CUS": "3", "TT_GEMM_ENGINE": "5"})


def test_panel_in_registers_engine_values_at_k_512(lockstep_gemm, tmp_path):
    # K = 512: the panel takes twice the registers and the two stages 128 KB, one workgroup per CU (stand-in device of two
    # CUs: two workgroups); two panels (the second with 40 rows) by five column tiles, so runs change panel mid-way
    env = {"EMU_CUS": "2", "TT_GEMM_ENGINE": "5"}
    out = check(lockstep_gemm, str(tmp_path), 1, 296, 320, 512, 1, 0, "bf16", "bf16", True, 85, env=env)
    assert int(out.split()[3]) == 2 * 256
    shape = (1, 256, 192, 512, 1, 0, "bf16", "bf16", False, 86)
    check(lockstep_gemm, str(tmp_path), *shape, env=dict(env, EMU_ORDER="reverse"))
    with pytest.raises(AssertionError):
        check(lockstep_gemm, str(tmp_path), *shape, env=dict(env, EMU_VMCNT_SLACK="2"))


def test_panel_in_registers_engine_counts_its_stores(lockstep_gemm, tmp_path):
    # its waits leave the previous unit's eight stores in flight; letting two more operations stay in flight than it
    # asks for must give stale operand tiles, and the order in which waves run must not matter
    env = {"EMU_CUS": "1", "TT_GEMM_ENGINE": "5"}
    shape = (1, 256, 512, 256, 1, 0, "bf16", "bf16", False, 84)
    check(lockstep_gemm, str(tmp_path), *shape, env=dict(env, EMU_ORDER="reverse"))
    with pytest.raises(AssertionError):
        check(lockstep_gemm, str(tmp_path), *shape, env=dict(env, EMU_VMCNT_SLACK="2"))


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_direct_to_lds_engine_values(lockstep_gemm, tmp_path, ta, tb):
    # the eight-wave 256 x 256 engine that loads tiles straight into LDS, forced by the tuning switches on small
    # products: ragged M and N, a K tail that is no multiple of the tile depth
    env = {"TT_GEMM_ENGINE": "1", "TT_GEMM_TILE": "8"}
    out = check(lockstep_gemm, str(tmp_path), 2, 264, 520, 72, ta, tb, "bf16", "bf16", True, 39, env=env)
    assert int(out.split()[3]) == 16 * 512     # 12 tiles, rounded up to a multiple of the 8 XCDs
    check(lockstep_gemm, str(tmp_path), 1, 256, 264, 128, ta, tb, "bf16", "f32", False, 40, env=env)


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4, 5])
def test_register_staged_engine_every_tile_values(lockstep_gemm, tmp_path, tile):
    env = {"TT_GEMM_ENGINE": "1", "TT_GEMM_TILE": str(tile)}
    check(lockstep_gemm, str(tmp_path), 1, 264, 392, 104, 0, 0, "bf16", "bf16", False, 50 + tile, env=env)
    check(lockstep_gemm, str(tmp_path), 1, 264, 392, 96, 1, 1, "bf16", "f32", True, 60 + tile, env=env)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_k_split_inside_a_launch_values(lockstep_gemm, tmp_path, ta, tb):
    # the partial products of the chunks add up to the product (chunks of 128, 128 and 64 of K = 320; on the smallest tile
    # chunks of 64, 64 and 22 of K = 150 would leave ... K must keep 16-byte rows: 152)
    check(lockstep_gemm, str(tmp_path), 2, 264, 264, 320, ta, tb, "bf16", "f32", False, 70, ksplit=3)
    check(lockstep_gemm, str(tmp_path), 1, 40, 72, 152, ta, tb, "bf16", "f32", False, 71, ksplit=3)


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_generic_kernel_values(lockstep_gemm, tmp_path, ta, tb):
    check(lockstep_gemm, str(tmp_path), 2, 70, 130, 65, ta, tb, "f32", "f32", True, 38)
    check(lockstep_gemm, str(tmp_path), 2, 37, 125, 50, ta, tb, "bf16", "bf16", True, 35)       # rows without 16-byte vectors
    check(lockstep_gemm, str(tmp_path), 1, 33, 10, 17, ta, tb, "bf16", "f32", False, 36, ksplit=1)


def test_random_products_values(lockstep_gemm, tmp_path):
    # seeded random shapes, layouts, types and tuning switches (sizes mostly multiples of eight, some odd): whatever
    # engine the launch code picks or falls back to has to give the product
    rng = np.random.default_rng(2024)
    switches = [{}, {}, {"TT_GEMM_ENGINE": "4"}, {"TT_GEMM_ENGINE": "6"}, {"TT_GEMM_ENGINE": "3", "TT_GEMM_TILE": "5", "EMU_CUS": "8"},
                {"TT_GEMM_ENGINE": "1", "TT_GEMM_TILE": "8"}] + [{"TT_GEMM_ENGINE": "1", "TT_GEMM_TILE": str(t)} for t in range(6)]

    def dim(hi):
        v = int(rng.integers(8, hi))
        return v if rng.random() < 0.15 else max(8, v // 8 * 8)

    for case in range(14):
        M, N, K = dim(560), dim(560), dim(330)
        ta, tb = (int(v) for v in rng.integers(0, 2, 2))
        in_dt = "bf16" if rng.random() < 0.85 else "f32"
        out_dt = "bf16" if rng.integers(0, 2) else "f32"
        ksplit = int(rng.choice([1, 1, 1, 2]))
        if ksplit > 1 and ((K + 1) // 2 + 63) // 64 * 64 >= K:
            ksplit = 1                                       # the second chunk would be empty: the launch refuses that
        relu = bool(rng.integers(0, 2)) and ksplit == 1
        if ksplit > 1:
            out_dt = "f32"                                   # partial products are kept in fp32, as the execute calls ask
        env = switches[int(rng.integers(0, len(switches)))]
        try:
            check(lockstep_gemm, str(tmp_path), int(rng.integers(1, 3)), M, N, K, ta, tb, in_dt, out_dt, relu, 300 + case, ksplit=ksplit, env=env)
        except AssertionError as e:
            raise AssertionError((case, M, N, K, ta, tb, in_dt, out_dt, relu, ksplit, env, str(e)[:500]))


@pytest.mark.parametrize("env", [{"EMU_CUS": "16", "TT_GEMM_ENGINE": "3", "TT_GEMM_TILE": "5"}, {"TT_GEMM_ENGINE": "1", "TT_GEMM_TILE": "8"}, {}])
def test_the_model_of_late_loads_bites(lockstep_gemm, tmp_path, env):
    # global -> LDS loads land only when a wait count lets them (see emu_lockstep.h); if every wait let two more loads
    # stay in flight than the kernel asks for, the engines that load straight into LDS must not get away with it
    shape = (2, 520, 776, 192, 0, 1, "bf16", "f32", False, 42) if env else (1, 264, 392, 96, 0, 1, "bf16", "f32", False, 45)
    check(lockstep_gemm, str(tmp_path), *shape, env=env)
    with pytest.raises(AssertionError):
        check(lockstep_gemm, str(tmp_path), *shape, env=dict(env, EMU_VMCNT_SLACK="2"))


@pytest.mark.parametrize("env", [{"EMU_CUS": "16", "TT_GEMM_ENGINE": "3", "TT_GEMM_TILE": "5"}, {"TT_GEMM_ENGINE": "1", "TT_GEMM_TILE": "8"}, {}])
def test_results_do_not_depend_on_which_wave_runs_ahead(lockstep_gemm, tmp_path, env):
    # the emulation runs the threads of a workgroup in index order between synchronisation points; with the order
    # reversed the last wave reaches every barrier first, issues its loads first and writes its results first
    shape = (2, 520, 776, 192, 1, 0, "bf16", "bf16", True, 42) if env else (1, 264, 392, 96, 1, 0, "bf16", "bf16", True, 45)
    check(lockstep_gemm, str(tmp_path), *shape, env=dict(env, EMU_ORDER="reverse"))
