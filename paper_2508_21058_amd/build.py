"""Builds libmoc.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2508_21058_amd.build [-j N]

Each translation unit is compiled to an object file under csrc/_build/ (only
when its sources changed, unless force=True) and linked into
paper_2508_21058_amd/libmoc.so.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libmoc.so")
UNITS = ["moc_api", "moc_pool", "moc_route", "moc_lists", "moc_attn_fwd", "moc_attn_bwd", "moc_probe", "moc_perturb", "moc_outer"]
# -Wno-inline-asm: the tile-copy asm lists m0 (which it sets) as clobbered; clang warns that m0 is reserved
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _deps():
    hdrs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hdrs.append(os.path.join(HERE, "..", "include", "moc.h"))
    return max(os.path.getmtime(h) for h in hdrs)


def _compile(unit: str, force: bool, hdr_time: float) -> str:
    src = os.path.join(CSRC, unit + ".hip")
    obj = os.path.join(OBJ, unit + ".o")
    if (not force and os.path.exists(obj) and os.path.getmtime(obj) >= os.path.getmtime(src)
            and os.path.getmtime(obj) >= hdr_time):
        return obj
    cmd = ["hipcc", *FLAGS, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {unit}:\n{r.stdout}\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines()
                     if "warning" in l and "packed-fp32-ops" not in l and "hip-link" not in l)
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(force: bool = False, jobs: int = 6) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hdr_time = _deps()
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda u: _compile(u, force, hdr_time), UNITS))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        tmp = LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    j = 6
    if "-j" in sys.argv:
        j = int(sys.argv[sys.argv.index("-j") + 1])
    print(build(force="--force" in sys.argv, jobs=j))
