"""Builds libsconv.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libsconv.so")
MICRO_SRC = os.path.join(CSRC, "micro", "sconv_micro.hip")
MICRO_LIB = os.path.join(HERE, "libsconv_micro.so")   # issue-rate microbenchmarks (bench.py --micro)

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         # packed fp32 instructions stay off: the compiler must not form them on its own
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", INCLUDE, "-I", CSRC]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    if not os.path.exists(MICRO_LIB):
        return True
    deps = sources() + [MICRO_SRC] + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(INCLUDE, "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, jobs: int = 8) -> str:
    """Compile every .hip file to an object (in parallel) and link the shared library."""
    if not force and not stale():
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        procs.append((src, subprocess.Popen([HIPCC, *FLAGS, "-c", src, "-o", obj],
                                            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    build_micro()
    return LIB


def build_micro() -> str:
    """The microbenchmark library: one source file, its own shared object."""
    pr = subprocess.run([HIPCC, *FLAGS, "-shared", MICRO_SRC, "-o", MICRO_LIB],
                        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    msgs = [l for l in pr.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    if pr.returncode != 0:
        raise RuntimeError("hipcc failed for the microbenchmarks:\n" + "\n".join(msgs))
    return MICRO_LIB


def _drain(procs):
    for src, pr in procs:
        out, _ = pr.communicate()
        # the host pass does not know the GPU feature flag and says so: harmless
        msgs = [l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip()]
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n" + "\n".join(msgs))
        if msgs:
            print("\n".join(msgs))
    procs.clear()


if __name__ == "__main__":
    print(build())
