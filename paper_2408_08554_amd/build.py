"""Compile the HIP sources under csrc/ for gfx950 into paper_2408_08554_amd/libabq.so.

Run here on the CPU container (hipcc cross-compiles); the built library travels with the
tree.  `python -m paper_2408_08554_amd.build` rebuilds everything.
"""
import concurrent.futures
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libabq.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    # packed-FP32 instructions are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    subprocess.run([HIPCC, *FLAGS, "-c", src, "-o", obj], check=True, stderr=subprocess.PIPE, text=True)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        futs = {ex.submit(_compile, s): s for s in srcs}
        objs = []
        for f, s in futs.items():
            try:
                objs.append(f.result())
            except subprocess.CalledProcessError as e:
                raise RuntimeError(f"hipcc failed on {s}:\n{e.stderr}") from None
            if verbose:
                print("compiled", os.path.basename(s), flush=True)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *sorted(objs), "-o", LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
