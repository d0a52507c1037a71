"""Builds the host emulation programs of tests/emu (helper of the emulation tests, no test itself).  All builds are
started together on a small thread pool when the first test asks for one, so their compile times overlap with each other
and with the tests that are already running."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = shutil.which("clang++", path="/opt/rocm/llvm/bin") or shutil.which("clang++")
EMU = os.path.join(ROOT, "tests", "emu")
CSRC = os.path.join(ROOT, "paper_1805_04170_amd", "csrc")
INCLUDES = ["-I" + EMU, "-I" + CSRC, "-I" + os.path.join(ROOT, "include")]
# -DTT_TUNING: the environment overrides of the launch heuristics (absent from the product build) let a test force an engine
BASE = ["-std=c++17", "-x", "c++", "-DTT_TUNING"]
ASAN = ["-fsanitize=address", "-fno-omit-frame-pointer"]
# -O1 where the checked launches are long (unoptimised code runs them several times slower), -O0 where the optimiser
# would need minutes (all four engines' instantiations in one unit)
PROGRAMS = {
    "gemm3": ("emu_gemm3.cpp", ["-O0"] + ASAN),
    "conv": ("emu_conv.cpp", ["-O1"] + ASAN),
    "convert": ("emu_convert.cpp", ["-O1"] + ASAN),
    "shard_gemm": ("emu_shard_gemm.cpp", ["-O0"] + ASAN),
    "shard_gemm_lockstep": ("emu_shard_gemm.cpp", ["-O0", "-DTT_EMU_LOCKSTEP"]),
}
GEMM1_NAMES = ["E1_BM", "E1_BN", "E1_WM", "E1_WN", "E1_DEPTH", "E1_KMASK", "E1_AKC", "E1_BKC", "E1_BF16", "E1_VEC"]
LIBRARY_UNITS = [os.path.join(EMU, f) for f in ("emu_lib_gemm.cpp", "emu_lib_conv.cpp", "emu_lib_convert.cpp", "emu_lib_flatten.cpp", "emu_lib_static.cpp")] + \
                [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".cpp")]
LIBRARY_FLAGS = ["-O0", "-fPIC", "-DTT_EMU_LOCKSTEP", "-DTT_HOST_EMULATION"]
# the same units in address mode under the sanitizer, linked with the driver of a whole training step
STEP_FLAGS = {"emu_lib_conv.cpp": ["-O1"], "emu_lib_convert.cpp": ["-O1"]}      # the rest -O0


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("emulation build failed: %s\n%s" % (" ".join(cmd), r.stderr[-4000:]))


class Emulators:
    def __init__(self, outdir):
        self.out = str(outdir)
        self.pool = ThreadPoolExecutor(6)
        self.jobs = {}
        for name in PROGRAMS:
            self._submit(name)
        self._submit("library")
        self._submit("step")

    def _submit(self, name):
        if name in self.jobs:
            return
        if name == "library":
            objs = [os.path.join(self.out, "lib_" + os.path.basename(u) + ".o") for u in LIBRARY_UNITS]
            parts = [self.pool.submit(_run, [CLANG] + BASE + LIBRARY_FLAGS + INCLUDES + ["-c", u, "-o", o])
                     for u, o in zip(LIBRARY_UNITS, objs)]
            so = os.path.join(self.out, "libtensor_tiling_emulated.so")

            def link():
                for p in parts:
                    p.result()
                _run([CLANG, "-shared", "-o", so] + objs)
                return so
            self.jobs[name] = link            # linked by whoever asks first (a pool worker waiting on the pool could starve it)
            return
        if name == "step":
            units = LIBRARY_UNITS + [os.path.join(EMU, "emu_step.cpp")]
            objs = [os.path.join(self.out, "step_" + os.path.basename(u) + ".o") for u in units]
            parts = [self.pool.submit(_run, [CLANG] + BASE + STEP_FLAGS.get(os.path.basename(u), ["-O0"]) + ASAN +
                                      ["-DTT_HOST_EMULATION"] + INCLUDES + ["-c", u, "-o", o]) for u, o in zip(units, objs)]
            exe = os.path.join(self.out, "emu_step")

            def link_step():
                for p in parts:
                    p.result()
                _run([CLANG] + ASAN + ["-o", exe] + objs)
                return exe
            self.jobs[name] = link_step
            return
        if isinstance(name, tuple):           # ("gemm1", configuration): the register-staged engine, one instantiation
            src, flags = "emu_gemm1.cpp", ["-O1"] + ASAN + ["-D%s=%d" % (n, v) for n, v in zip(GEMM1_NAMES, name[1])]
            exe = os.path.join(self.out, "emu_gemm1_" + "_".join(str(v) for v in name[1]))
        else:
            src, flags = PROGRAMS[name]
            exe = os.path.join(self.out, "emu_" + name)
        fut = self.pool.submit(_run, [CLANG] + BASE + flags + INCLUDES + [os.path.join(EMU, src), "-o", exe])
        self.jobs[name] = lambda: (fut.result(), exe)[1]

    def prefetch(self, names):
        for n in names:
            self._submit(n)

    def get(self, name):
        self._submit(name)
        path = self.jobs[name]()
        self.jobs[name] = lambda: path
        return path
