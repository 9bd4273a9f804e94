"""Build liblasp2.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2502_07563_amd.build [--out FILE] [extra hipcc flags]

The flag that switches packed-fp32 instruction selection off is required on
the test machines.

A checking variant in which every hand-counted vector-memory wait of the matrix-core kernels
waits for everything (`s_waitcnt vmcnt(0)`) is built beside the product library with

    python -m paper_2502_07563_amd.build --out paper_2502_07563_amd/liblasp2_fullwaits.so -DLASP2_FULL_WAITS

and loaded instead of it by setting LASP2_LIB_PATH to that file (the binding reads it), e.g. to
run the GPU parity tests once on it when a miscounted wait is suspected.
"""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "liblasp2.so")
SOURCES = ["lasp2_api.hip", "kernels_generic.hip", "kernels_mfma.hip", "kernels_softmax.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose: bool = False, extra=(), out: str = LIB) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + ["-o", out] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    argv = sys.argv[1:]
    out = LIB
    if "--out" in argv:
        i = argv.index("--out")
        out = os.path.abspath(argv[i + 1])
        del argv[i:i + 2]
    print(build(verbose=True, extra=argv, out=out))
