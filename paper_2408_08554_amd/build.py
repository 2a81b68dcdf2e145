"""Compile the HIP sources under csrc/ for gfx950 into paper_2408_08554_amd/libabq.so.

Run here on the CPU container (hipcc cross-compiles); the built library travels with the
tree.  `python -m paper_2408_08554_amd.build` rebuilds everything
(`--incremental`: only what changed).
"""
import concurrent.futures
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libabq.so")
PROBE_LIB = os.path.join(HERE, "libabq_probe.so")   # measurement aids of the benchmark, not part of libabq.so

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    # packed-FP32 instructions are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]
if os.environ.get("ABQ_BUILD_TUNING") == "1":   # the tuner's A/B builds only: lets ABQ_* environment variables override launch plans
    FLAGS.append("-DABQ_TUNING_ENV")


def _compile(src: str, newest_header: float = 0.0) -> str:
    obj = os.path.join(OBJ, os.path.relpath(src, CSRC).replace(os.sep, "_") + ".o")
    if newest_header and os.path.exists(obj) and os.path.getmtime(obj) >= max(newest_header, os.path.getmtime(src)):
        return obj   # --incremental: neither the source nor any header is newer than the object
    extra = ["-Rpass-analysis=kernel-resource-usage"] if os.path.basename(src) in NO_SCRATCH else []
    done = subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], check=True, stderr=subprocess.PIPE, text=True)
    if extra:
        _check_no_scratch(src, done.stderr, NO_SCRATCH[os.path.basename(src)])
    return obj


# Kernels that load registers with hand-written load instructions and wait for them by hand: the compiler does not know
# that such a register fills later, so it must not spill it in between.  The build fails if one of them uses scratch memory.
NO_SCRATCH = {"abq_f4.hip": "f4_gemm_kernel"}


def _check_no_scratch(src: str, remarks: str, kernel: str) -> None:
    name, seen = None, 0
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].strip()
        elif "ScratchSize [bytes/lane]:" in line and name and kernel in name:
            seen += 1
            if int(line.split(":")[-1].split()[0]) != 0:
                os.remove(os.path.join(OBJ, os.path.relpath(src, CSRC).replace(os.sep, "_") + ".o"))
                raise RuntimeError(f"{src}: kernel {name} uses scratch memory; its hand-written loads would be spilled before they land")
    if not seen:
        raise RuntimeError(f"{src}: no resource-usage remark for {kernel}; the scratch check did not run")


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compiles every source (always, unless `incremental`: then only what is older than its source or a header)."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    probe_srcs = sorted(glob.glob(os.path.join(CSRC, "probe", "*.hip")))
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h")) + [__file__]
    newest = max(os.path.getmtime(h) for h in headers) if incremental else 0.0
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        futs = {ex.submit(_compile, s, newest): s for s in srcs + probe_srcs}
        objs, probe_objs = [], []
        for f, s in futs.items():
            try:
                (probe_objs if s in probe_srcs else objs).append(f.result())
            except subprocess.CalledProcessError as e:
                raise RuntimeError(f"hipcc failed on {s}:\n{e.stderr}") from None
            if verbose:
                print("compiled", os.path.basename(s), flush=True)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *sorted(objs), "-o", LIB], check=True)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *sorted(probe_objs), "-o", PROBE_LIB], check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv))
