"""Builds liboxy.so (HIP kernels for gfx950 + host pool) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liboxy.so")
SOURCES = ["oxy_kernels.hip", "oxy_pool.cpp", "oxy_sched.cpp"]
# packed fp32 VALU forms are switched off for device code on purpose
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


PROBE_SRC = os.path.join(HERE, "benchaid", "probe_kernels.hip")
PROBE_LIB = os.path.join(HERE, "benchaid", "libprobe.so")


def _hipcc(sources, target, verbose):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-result"]
    cmd += DEVICE_FLAGS
    cmd += list(sources) + ["-o", target]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return target


def build_library(verbose=False):
    """liboxy.so (the method) and benchaid/libprobe.so (the benchmark's measurement aids)."""
    _hipcc([os.path.join(CSRC, s) for s in SOURCES], LIB, verbose)
    _hipcc([PROBE_SRC], PROBE_LIB, verbose)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
