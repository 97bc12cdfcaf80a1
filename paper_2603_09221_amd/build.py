"""Build of the HIP library for gfx950: every kernel family is its own translation unit (and, where the
kernels are templates over the state size, one object per state size), compiled in parallel and linked
into paper_2603_09221_amd/lib/libttc_lqr.so.

    python -m paper_2603_09221_amd.build [--force] [-j N]

Without --force only objects older than a source file are rebuilt.
"""
from __future__ import annotations

import argparse
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG), "include")
OBJDIR = os.path.join(PKG, "lib", "_build")
OUT = os.path.join(PKG, "lib", "libttc_lqr.so")

HIPCC_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

# (source, state sizes it is compiled for; None = once)
UNITS = [("ttc_api.hip", None),
         ("k_solve.hip", (32, 64, 128)),
         ("k_doubling.hip", (16, 32, 64, 128)),
         ("k_rollout.hip", (16, 32, 64, 128)),
         ("k_tv.hip", (16, 32, 64, 128)),
         ("k_scan.hip", (16, 32, 64, 128)),
         ("k_backward.hip", (16, 32, 64, 128)),
         ("k_small.hip", None),
         ("k_tv_small.hip", None),
         ("k_cxt.hip", None),
         ("k_cxt_bwd.hip", None),
         ("k_block.hip", None)]

# Per (source, state size) compile flags: wavefronts of one 16-row block each (twice as many per problem) instead of
# two row blocks, where measured faster.  The dense solve inside these kernels is a third or more of their time and
# all but one wavefront share its tiles; the default forward kernel is faster with fewer, fatter wavefronts (its
# constant operands stay in registers; at d = 64 four problems fit a compute unit).  Measured, problems/s:
# backward d = 64, T = 8: 1.99M against 1.79M; time-heterogeneous d = 128, T = 16: 179k against 170k; squaring path
# d = 128, T = 16: 501k against 488k (T = 32, bf16 inputs: 421k against 404k).
_ONE_ROW_BLOCK = "-DTTC_ROW_BLOCKS(D)=((D)==%d?1:((D)>=32?2:1))"
UNIT_FLAGS = {("k_backward.hip", 64): [_ONE_ROW_BLOCK % 64],
              ("k_tv.hip", 128): [_ONE_ROW_BLOCK % 128],
              ("k_doubling.hip", 128): [_ONE_ROW_BLOCK % 128]}

_NOISE = "is not a recognized feature for this target"


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if _NOISE not in l and "warning generated" not in l)
    if res.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), err))
    if err.strip():
        print(err, file=sys.stderr)


def _newest_source():
    t = 0.0
    for folder in (CSRC, INCLUDE):
        for name in os.listdir(folder):
            t = max(t, os.path.getmtime(os.path.join(folder, name)))
    return max(t, os.path.getmtime(os.path.abspath(__file__)))


def build(force: bool = True, jobs: int | None = None, extra_flags=()) -> str:
    """Compile and link; returns the path of the shared library."""
    os.makedirs(OBJDIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(16, os.cpu_count() or 1)
    newest = _newest_source()
    work, objs = [], []
    for src, sizes in UNITS:
        for d in (sizes or (None,)):
            stem = os.path.splitext(src)[0] + ("" if d is None else "_%d" % d)
            obj = os.path.join(OBJDIR, stem + ".o")
            objs.append(obj)
            if force or not os.path.exists(obj) or os.path.getmtime(obj) < newest:
                cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + UNIT_FLAGS.get((src, d), []) + \
                      (["-DTTC_D=%d" % d] if d else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
                work.append(cmd)
    # the largest state sizes take longest: start them first
    work.sort(key=lambda c: -max([int(a[8:]) for a in c if a.startswith("-DTTC_D=")] or [0]))
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(_run, work))
    if work or not os.path.exists(OUT):
        _run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", OUT] + objs)
    return OUT


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--force", action="store_true")
    ap.add_argument("-j", type=int, default=None)
    ap.add_argument("--flag", action="append", default=[], help="extra hipcc flag (repeatable), e.g. --flag=-DTTC_PHASE_TIMERS")
    a = ap.parse_args()
    print(build(force=a.force, jobs=a.j, extra_flags=a.flag))
