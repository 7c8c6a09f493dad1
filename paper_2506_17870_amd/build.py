"""Builds libnq.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2506_17870_amd.build [--force]

Objects go to _build/ next to this file, the library to paper_2506_17870_amd/libnq.so.
Four translation units per nesting (h, l) hold the GEMM/convolution kernels, so the
units compile in parallel; the GEMM over the paper's word pages is one unit for all nestings.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libnq.so")
YARDSTICKS = os.path.join(HERE, "nq_yardsticks")   # standalone hardware yardsticks (csrc/nq_yardsticks.hip)

# (h, l): INT(8|h) for l = 1..6 and INT(6|h) for l = 1..4
NESTINGS = [(7, 1), (6, 2), (5, 3), (4, 4), (3, 5), (2, 6), (5, 1), (4, 2), (3, 3), (2, 4)]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _units():
    units = [(os.path.join(CSRC, f + ".hip"), os.path.join(OBJ, f + ".o"), [])
             for f in ("nq_pack", "nq_page", "nq_glue", "nq_gemm", "nq_gemm_words")]   # nq_yardsticks.hip is a program of its own
    for h, l in NESTINGS:
        for part in (1, 0, 2, 3):
            units.append((os.path.join(CSRC, "nq_gemm_inst.hip"), os.path.join(OBJ, f"nq_gemm_inst_{h}{l}_{part}.o"),
                          [f"-DNQ_INST_H={h}", f"-DNQ_INST_L={l}", f"-DNQ_INST_PART={part}"]))
    return units


def _stale(unit) -> bool:
    """A unit is rebuilt when its object is missing or older than any file it was compiled from (the compiler
    writes the list next to the object, -MMD)."""
    src, obj, _ = unit
    dep = obj[:-2] + ".d"
    if not os.path.exists(obj) or not os.path.exists(dep):
        return True
    with open(dep) as f:
        text = f.read().replace("\\\n", " ")
    files = text.split(":", 1)[1].split() if ":" in text else [src]
    t = os.path.getmtime(obj)
    return any((not os.path.exists(x)) or os.path.getmtime(x) > t for x in files)


def _compile(unit):
    src, obj, defs = unit
    cmd = ["hipcc", *FLAGS, *defs, "-MMD", "-MF", obj[:-2] + ".d", "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {os.path.basename(obj)}:\n{r.stderr[-4000:]}")
    return obj


def build(force: bool = False, jobs: int | None = None) -> str:
    os.makedirs(OBJ, exist_ok=True)
    units = _units()
    todo = [u for u in units if force or _stale(u)]
    jobs = jobs or min(8, os.cpu_count() or 1)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(_compile, todo))
    if todo or not os.path.exists(LIB):
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *[u[1] for u in units]]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr[-4000:])
    # a kernel template that the host pass fails to instantiate shows up only as an undefined symbol at load time
    import ctypes
    ctypes.CDLL(LIB, mode=os.RTLD_NOW)
    ysrc = os.path.join(CSRC, "nq_yardsticks.hip")
    if force or not os.path.exists(YARDSTICKS) or os.path.getmtime(YARDSTICKS) < os.path.getmtime(ysrc):
        r = subprocess.run(["hipcc", *[f for f in FLAGS if f != "-fPIC"], ysrc, "-o", YARDSTICKS],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for nq_yardsticks:\n" + r.stderr[-4000:])
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
