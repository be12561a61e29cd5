"""Build libcmn.so (HIP kernels + C-ABI) for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcmn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # one rounding per float op, like the definition
    "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",
    "-fhip-fp32-correctly-rounded-divide-sqrt",  # Adam's sqrt and division round like the host's
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the two-phase step kernel parks averaged gradients in a register array indexed by a fully
    # unrolled loop; without full unrolling the array would fall into scratch memory
    "-mllvm", "-pragma-unroll-threshold=1000000",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_lib(verbose: bool = False, extra_flags=()) -> str:
    """Compile every csrc/*.hip to an object (in parallel) and link libcmn.so."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    flags = [f for f in HIPCC_FLAGS if f != "-shared"] + list(extra_flags)
    with tempfile.TemporaryDirectory(prefix="cmn_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            cmd = ["hipcc", *flags, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        with ThreadPoolExecutor(max_workers=8) as ex:
            objs = list(ex.map(compile_one, sources()))
        link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
