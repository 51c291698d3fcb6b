"""Compile the HIP sources under csrc/ into paper_2006_06762_amd/libanr.so for gfx950.

Run as ``python -m paper_2006_06762_amd.build`` (hipcc cross-compiles without a GPU).
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libanr.so")

SOURCES = ["api.cpp", "gemm.hip", "tbg.hip", "conv_direct.hip", "conv_igemm.hip", "conv_gather.hip", "conv_pointwise.hip", "dwconv.hip", "nrm.hip", "static_scratch.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
    # packed fp32 instructions are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# Per-file flags.  The convolution and GEMM kernels keep their MFMA accumulators in ordinary vector
# registers instead of the accumulation registers: prologues and epilogues then need no copies
# between the two register files.  Measured: 0.25-0.35 us per launch on the three benchmark
# convolutions, 1-2 % on the general convolution kernels, 6-10 % on GEMMs of 512^3 x 16 and
# 2048^3; no gain on the attention kernels, which are left alone.
FILE_FLAGS = {
    "conv_igemm.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "conv_gather.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "gemm.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
}


def _compile(src, verbose, extra):
    out = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc"] + FLAGS + FILE_FLAGS.get(src, []) + list(extra) + ["-c", os.path.join(CSRC, src), "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr))
    if verbose and err.strip():
        print(err, flush=True)
    return out


def build(verbose: bool = False, extra=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, verbose, extra), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def _stale() -> bool:
    """True when the library is missing or older than any source it is built from."""
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    srcs = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    inc = os.path.join(ROOT, "include")
    srcs += [os.path.join(inc, f) for f in os.listdir(inc)]
    return any(os.path.getmtime(f) > built for f in srcs if os.path.isfile(f))


def ensure_built(verbose: bool = False) -> str:
    """Build the library unless a built one is there that is newer than every file under
    csrc/ and include/ (tests, the smoke run and the benchmark load what is built)."""
    if not _stale():
        return LIB
    if not shutil.which("hipcc"):
        if os.path.exists(LIB):
            return LIB      # a box without the compiler runs what was shipped
        raise RuntimeError("libanr.so is missing and hipcc is not on PATH")
    return build(verbose=verbose)


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
