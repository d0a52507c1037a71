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
def emu(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("emu") / "emu_gemm3")
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=address", "-I" + os.path.join(ROOT, "tests", "emu"),
           "-I" + os.path.join(ROOT, "paper_1805_04170_amd", "csrc"), "-I" + os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "emu", "emu_gemm3.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return exe


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
    (3, 8, 3136, 4096, 256, 0, 0, 1, 0, 1),     # the weight gradient of the VGG-16 first classifier layer (benchmark shape)
    (3, 8, 256, 4096, 3136, 1, 0, 0, 0, 2),     # its forward product with the in-shard K split, fp32 partial sums
    (3, 16, 512, 2048, 2048, 1, 1, 1, 0, 1),    # wide MLP shard product
    (3, 2, 520, 776, 64, 0, 0, 1, 0, 1),
    (3, 1, 264, 1000, 192, 1, 0, 1, 0, 1),      # 1000 columns: ragged last tile, 16-byte rows
    (3, 1, 264, 1004, 128, 1, 1, 0, 0, 1),      # fp32 rows of 1004
    (2, 8, 256, 3136, 4096, 1, 1, 0, 0, 2),     # direct-to-LDS engine: data gradient of the VGG-16 first classifier layer
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
def test_register_staged_engine_stays_inside_its_buffers(tmp_path, cfg, case):
    names = ["E1_BM", "E1_BN", "E1_WM", "E1_WN", "E1_DEPTH", "E1_KMASK", "E1_AKC", "E1_BKC", "E1_BF16", "E1_VEC"]
    exe = str(tmp_path / "emu_gemm1")
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=address"] + ["-D%s=%d" % (n, v) for n, v in zip(names, cfg)] + [
        "-I" + os.path.join(ROOT, "tests", "emu"), "-I" + os.path.join(ROOT, "paper_1805_04170_amd", "csrc"),
        "-I" + os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "emu", "emu_gemm1.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    r = run(exe, case)
    assert r.returncode == 0, r.stdout[-400:] + r.stderr[-1200:]
