"""Compile libsignvote.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_1810_05291_amd.build

The objects go to paper_1810_05291_amd/_build/, the library to paper_1810_05291_amd/libsignvote.so.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsignvote.so")
SOURCES = ["api.hip", "step_kernels.hip", "multi_kernels.hip", "vote_kernels.hip", "qsgd_kernels.hip", "bench_copy.hip"]
HEADERS = ["common.h", "device_utils.h", "step_tiles.h", "vote_tiles.h", os.path.join("..", "..", "include", "signvote.h"),
           os.path.join("..", "..", "include", "signvote_bench.h"), os.path.join("..", "..", "include", "signvote_qsgd.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-std=c++17", "-O3", "-fPIC",
    "-ffp-contract=off",                 # the momentum / update formulas fix where the fused multiply-adds are
    "-fno-fast-math",
    "-fno-gpu-flush-denormals-to-zero",  # the sign of a denormal is data
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def _stale(out, deps):
    if not os.path.exists(out):
        return True
    t = os.path.getmtime(out)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, extra_flags=(), lib_path: str = LIB, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hdrs = [os.path.join(CSRC, h) for h in HEADERS] + [os.path.abspath(__file__)]
    tag = "" if lib_path == LIB else "." + os.path.basename(lib_path)
    jobs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src + tag + ".o")
        if force or _stale(o, [s] + hdrs):
            jobs.append([HIPCC, *FLAGS, *extra_flags, "-c", s, "-o", o])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stdout + r.stderr)
        return r.stderr

    with ThreadPoolExecutor(max_workers=min(4, max(1, len(jobs)))) as ex:
        for err in ex.map(run, jobs):
            if verbose and err.strip():
                print(err, file=sys.stderr)
    objs = [os.path.join(OBJ, src + tag + ".o") for src in SOURCES]
    if jobs or not os.path.exists(lib_path):
        run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path, *objs])
    return lib_path


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
