"""Builds libplora.so (host C++ + gfx950 kernels) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libplora.so")
SOURCES = ["plora_pool.cpp", "plora_manager.cpp", "plora_predictor.cpp", "plora_kernels.hip", "plora_probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build(verbose=False):
    """Always compiles; returns the path of the shared library."""
    objs = []
    common = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-result"]
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [HIPCC, "--offload-arch=gfx950"] + common
        if src.endswith(".cpp"):
            cmd += ["-fopenmp-simd"]  # honours the simd pragmas of the host code; no OpenMP runtime involved
        if src == "plora_manager.cpp":
            cmd += ["-ffp-contract=off"]  # its scores decide an order: one rounding per operation
        if src.endswith(".hip"):
            # no packed-fp32 instructions from the auto-vectoriser (device pass only)
            cmd += ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
        cmd += ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines() if "not a recognized feature for this target" not in l)
        if r.returncode:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
        objs.append(obj)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
