"""Compile the HIP library for gfx950 into paper_2310_03675_amd/libhdqt.so.

    python -m paper_2310_03675_amd.build
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhdqt.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "quantize.hip", "quantize_fast.hip", "quantize_dual.hip", "gemm.hip", "gemm_fast.hip", "im2col.hip", "profile.hip", "probe.hip"]

# -ffp-contract=off: every binary32 operation of the quantizer rounds on its own,
# as in the definition the results are checked against.
# packed-fp32-ops off: keep the compiler from pairing float operations into the
# packed forms.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, extra=()) -> str:
    """One object per source, compiled side by side (the two large files take a minute
    each), then one link."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    os.makedirs(OBJ_DIR, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *flags, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        return obj

    jobs = min(len(SOURCES), int(os.environ.get("MAX_JOBS", "0")) or os.cpu_count() or 1, 8)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
