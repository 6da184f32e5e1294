"""Builds libpf.so (host C++ + ahead-of-time gfx950 kernels) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpf.so")
SOURCES = ["api.cpp", "ir.cpp", "rewrite.cpp", "plan.cpp", "codegen.cpp", "runtime.cpp", "metric.cpp", "score.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build(verbose=False):
    cmd = [HIPCC, "-shared", "-fPIC", "-O2", "-std=c++17", "--offload-arch=gfx950",
           # packed fp32 instructions are kept out of device code on purpose
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-ffp-contract=off",
           "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        if s.endswith(".cpp"):
            cmd += ["-x", "hip", path]      # host-only C++ goes through the same driver
        else:
            cmd += ["-x", "hip", path]
    cmd += ["-o", LIB, "-L/opt/rocm/lib", "-lhiprtc", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed building libpf.so")
    if verbose and (r.stdout or r.stderr):
        sys.stderr.write(r.stdout + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
