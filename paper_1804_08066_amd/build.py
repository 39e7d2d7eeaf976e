"""Build libmqgrad.so (gfx950 kernels + C ABI + host MDP) in-tree with hipcc, and libmqgrad_bench.so
(the streaming kernels that bench.py uses as its measured ceilings; not part of the library)."""
import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmqgrad.so")
BENCH_LIB = os.path.join(HERE, "libmqgrad_bench.so")
SOURCES = ["api.hip", "quantize_pack.hip", "quantize_wave.hip", "aggregate_update.hip", "minmax.hip", "mdp.cpp"]
BENCH_SOURCES = ["bench_stream.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off: the kernels' only fused operations are their explicit fma calls, so that the
# fp32 results are reproducible to the bit.  Packed-fp32 instruction selection is switched off.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off", "-fno-fast-math", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def needs_build():
    """True when a library is missing or older than any of its sources or headers."""
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".hip", ".cpp"))] + \
        [os.path.join(ROOT, "include", "mqgrad.h")]
    for lib in (LIB, BENCH_LIB):
        if not os.path.exists(lib):
            return True
        t = os.path.getmtime(lib)
        if any(os.path.getmtime(d) > t for d in deps):
            return True
    return False


def _link(names, out, tmpdir, verbose, extra_flags):
    def compile_one(name):
        obj = os.path.join(tmpdir, name + ".o")
        cmd = [HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, name), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=min(6, len(names))) as pool:
        objs = list(pool.map(compile_one, names))
    tmp = out + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,--no-undefined", *objs, "-o", tmp])
    os.replace(tmp, out)


def build(verbose=False, extra_flags=()):
    """Compile every source (one hipcc process per file, in parallel) and link both libraries."""
    tmpdir = tempfile.mkdtemp(prefix="mqgrad_build_")
    try:
        _link(SOURCES, LIB, tmpdir, verbose, extra_flags)
        _link(BENCH_SOURCES, BENCH_LIB, tmpdir, verbose, extra_flags)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
