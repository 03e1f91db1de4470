"""Build libsta.so (the C-ABI HIP library) and libsta_mfma_probe.so (a matrix-instruction-only kernel that the
benchmark alone loads) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libsta.so")
BUILD_DIR = os.path.join(HERE, "_build")
SOURCES = ["sta_api.hip", "sta_permute.hip", "sta_attention.hip", "sta_reduce.hip", "sta_backward.hip"]
PROBE_SOURCE = "bench_mfma_probe.hip"
PROBE_OUT = os.path.join(HERE, "libsta_mfma_probe.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept out of every kernel
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    # no NaN is ever produced inside the kernels (the only infinities are the initial running maxima, which meet
    # finite values only); saying so lets max chains compile to v_max3_f32 without per-operand canonicalisation
    "-fno-honor-nans",
]


def _compile(src: str) -> str:
    obj = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    noise = "is not a recognized feature for this target"
    warn = "\n".join(l for l in r.stderr.splitlines() if l.strip() and noise not in l)
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES) + 1) as ex:
        objs = list(ex.map(_compile, SOURCES + [PROBE_SOURCE]))
    for out, members in ((OUT, objs[:-1]), (PROBE_OUT, objs[-1:])):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + members
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
        if verbose:
            print(out)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
