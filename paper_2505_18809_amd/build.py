"""Build libvorta.so (the product) and libvorta_probe.so (a measurement aid only bench.py loads)
in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvorta.so")
PROBE_LIB = os.path.join(HERE, "libvorta_probe.so")
SOURCES = ["vorta_host.cpp", "vorta_passes.hip", "vorta_attn_f32.hip", "vorta_attn_bf16.hip", "vorta_api.hip"]
PROBE_SOURCES = ["mfma_probe.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix instructions write their results to ordinary vector registers, which the softmax
    # reads directly, also in the kernel that runs one wavefront per SIMD
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]
# the host pass does not know the packed-fp32 target feature and says so: harmless, not a warning of ours
NOISE = ("packed-fp32-ops", "is not a recognized feature")


def _compile(sources, lib, verbose):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in sources:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".cpp") else [path])
    cmd += ["-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in NOISE))
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    return err


def build(verbose: bool = False, allow_warnings: bool = False) -> str:
    """Compiles both libraries.  Compiler warnings are errors of the build (they are printed
    and the build raises) unless allow_warnings is set."""
    err = _compile(SOURCES, LIB, verbose) + _compile(PROBE_SOURCES, PROBE_LIB, verbose)
    if "warning:" in err:
        print(err, file=sys.stderr)
        if not allow_warnings:
            raise RuntimeError(f"hipcc reported {err.count('warning:')} warning(s); the build is kept warning-free")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, allow_warnings="--allow-warnings" in sys.argv))
