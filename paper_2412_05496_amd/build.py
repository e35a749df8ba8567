"""Builds libflexattn.so for gfx950 with hipcc (in-tree, no JIT cache).

    python -m paper_2412_05496_amd.build [--jobs N] [--incremental]

FLEXATTN_EXTRA_FLAGS (environment) is appended to the hipcc command line of every unit.

Every (mask_mod, score_mod) variant of the forward and backward kernels is its own translation
unit, so the compile runs in parallel.
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libflexattn.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
NUM_VARIANTS = 13         # must equal kNumVariants in csrc/variants.h

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"),
         "-I" + CSRC, "-Wno-unused-result", "-Wno-pass-failed",
         # packed-fp32 VALU forms are not to be generated on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         *os.environ.get("FLEXATTN_EXTRA_FLAGS", "").split()]


def _units():
    units = [("blockmask", "blockmask.hip", []), ("fwd", "fwd.hip", []), ("bwd", "bwd.hip", []),
             ("decode", "decode.hip", []), ("probe", "probe.hip", [])]
    for i in range(NUM_VARIANTS):
        units.append((f"fwd_inst_{i}", "fwd_inst.hip", [f"-DFLEXATTN_VARIANT={i}"]))
        units.append((f"bwd_inst_{i}", "bwd_inst.hip", [f"-DFLEXATTN_VARIANT={i}"]))
        units.append((f"fwd_paged_inst_{i}", "fwd_paged_inst.hip", [f"-DFLEXATTN_VARIANT={i}"]))
    return [u for u in units if os.path.exists(os.path.join(CSRC, u[1]))]


def _newest_header() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(ROOT, "include", "flexattn.h"))
    return max(os.path.getmtime(h) for h in hs)


def _compile(unit, force: bool) -> str:
    name, src, defs = unit
    src_path, obj = os.path.join(CSRC, src), os.path.join(OBJ, name + ".o")
    if (not force and os.path.exists(obj)
            and os.path.getmtime(obj) > max(os.path.getmtime(src_path), _newest_header())):
        return obj
    cmd = [HIPCC, *FLAGS, *defs, "-c", src_path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {name}:\n{' '.join(cmd)}\n{err}")
    if err.strip():
        sys.stderr.write(f"[{name}] {err}\n")
    return obj


def build(jobs: int = 0, force: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    units = _units()
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda u: _compile(u, force), units))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--jobs", type=int, default=0)
    ap.add_argument("--incremental", action="store_true", help="skip objects newer than their sources")
    args = ap.parse_args()
    print(build(args.jobs, force=not args.incremental))
