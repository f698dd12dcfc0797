"""Builds liba2cid.so (host planner/scheduler + gfx950 kernels) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liba2cid.so")
SOURCES = ["a2cid_host.cpp", "a2cid_engine.hip"]
HEADERS = ["a2cid_internal.h", "a2cid_kernels.hip.h"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(ROOT, "include", "a2cid.h")]
    return any(os.path.getmtime(p) > os.path.getmtime(LIB) for p in deps)


def build(force: bool = True) -> str:
    if not force and not stale():
        return LIB
    cmd = [HIPCC] + FLAGS + ["-x", "hip"] + [os.path.join(CSRC, f) for f in SOURCES] + ["-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
