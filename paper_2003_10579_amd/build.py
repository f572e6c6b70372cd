"""Builds libssgd.so (hipcc, gfx950) in-tree next to the sources."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libssgd.so")
SOURCES = ["api.hip", "schedule.hip", "linear.hip", "linear_tile.hip", "linear_defer.hip", "full_loss.hip", "full_grad.hip", "mlp.hip", "mc.hip"]
HEADERS = ["common.hpp", "rng.hpp", "mlp.hpp", os.path.join("..", "..", "include", "ssgd.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# event-process arithmetic (clock sums, AdaSync rule) must round like plain IEEE operations
NO_CONTRACT = {"schedule.hip": ["-ffp-contract=off"], "mc.hip": ["-ffp-contract=off"], "api.hip": ["-ffp-contract=off"]}


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) is False or os.path.exists(cand)):
            return cand
    return "hipcc"


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    return any(os.path.getmtime(f) > t for f in deps)


def build(force: bool = True, jobs: int = 5) -> str:
    """Compile every translation unit and link the shared library."""
    if not force and not stale():
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        extra = NO_CONTRACT.get(src, [])
        procs.append((src, subprocess.Popen([hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj])))
        if len(procs) >= jobs:
            name, p = procs.pop(0)
            if p.wait() != 0:
                raise RuntimeError(f"hipcc failed on {name}")
    for name, p in procs:
        if p.wait() != 0:
            raise RuntimeError(f"hipcc failed on {name}")
    subprocess.check_call([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB])
    return LIB


if __name__ == "__main__":
    print(build())
