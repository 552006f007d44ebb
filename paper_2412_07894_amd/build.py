"""Builds the C-ABI library (libhyd_attn.so) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhyd_attn.so")
SOURCES = [os.path.join(CSRC, "hyd_api.hip"), os.path.join(CSRC, "hyd_plan.cpp")]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # no NaN is ever produced on a live lane (masks use -inf only as an exp2 argument), so max/min
    # need no sNaN-quieting copies
    "-fno-honor-nans",
    "-Wall", "-Wno-unused-function",
]


def sources_newer_than_lib():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "hyd_attn.h"))
    deps.append(os.path.join(os.path.dirname(HERE), "include", "hyd_plan.h"))
    return any(os.path.getmtime(f) > t for f in deps)


def build(verbose=False, extra_flags=()):
    cmd = ["hipcc", *HIPCC_FLAGS, *extra_flags, *SOURCES, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass does not know the device-only target feature; that notice is harmless
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra_flags=sys.argv[1:])
    print("built", LIB)
