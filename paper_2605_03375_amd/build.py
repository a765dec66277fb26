"""Compile libtutti (HIP, gfx950) in-tree: paper_2605_03375_amd/libtutti.so.

hipcc cross-compiles without a GPU.  `python -m paper_2605_03375_amd.build` or `build_lib()`.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtutti.so")
BENCH_LIB = os.path.join(HERE, "libtutti_bench.so")  # the same sources with the measurement aids compiled in
SOURCES = [os.path.join(CSRC, "tutti_api.hip"), os.path.join(CSRC, "tutti_host.cpp")]
DEPS = SOURCES + [os.path.join(CSRC, "tutti_kernels.hip.h"), os.path.join(ROOT, "include", "tutti.h"),
                  os.path.join(ROOT, "include", "tutti_bench.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
    # no packed-fp32 instructions in any HIP code of this repository
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _build(out: str, defines, force: bool, verbose: bool) -> str:
    if not force and os.path.exists(out):
        if os.path.getmtime(out) >= max(os.path.getmtime(p) for p in DEPS):
            return out
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *defines, f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}", *SOURCES, "-o", out]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True, cwd=ROOT)
    return out


def build_lib(force: bool = True, verbose: bool = False) -> str:
    """The product library: paper_2605_03375_amd/libtutti.so."""
    return _build(LIB, [], force, verbose)


def build_bench_lib(force: bool = True, verbose: bool = False) -> str:
    """The measurement library: the same entry points plus baselines, tuning knobs and all launch shapes."""
    return _build(BENCH_LIB, ["-DTUTTI_BENCH_BUILD"], force, verbose)


if __name__ == "__main__":
    print(build_lib(force=True, verbose=True))
    print(build_bench_lib(force=True, verbose=True))
