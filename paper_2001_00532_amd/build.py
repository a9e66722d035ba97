"""Builds libpsk.so (the C-ABI library) from csrc/*.hip with hipcc for gfx950.

Run as ``python -m paper_2001_00532_amd.build``.  Objects go to ``_build/`` (ignored by git), the
library lands next to this file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libpsk.so")
OBJDIR = os.path.join(HERE, "_build")
# the instrumented build (-DPSK_CU_TRACE: per-workgroup start/end/CU records, see psk_cu_trace_set)
OUT_TRACE = os.path.join(HERE, "libpsk_trace.so")
OBJDIR_TRACE = os.path.join(HERE, "_build_trace")

SOURCES = ["api.hip", "partition.hip", "spmv_csr.hip", "spmm.hip", "spmv_bcsr.hip", "mttkrp.hip", "spmv_csr_f64.hip", "spmv_csr_divide.hip", "spmv_bcsr_g.hip", "spmm_narrow.hip", "slab.hip", "api_slab.hip", "calibrate.hip"]
HEADERS = ["psk_dev.h", "psk_internal.h", os.path.join("..", "..", "include", "psk.h")]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # keep the compiler from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str, objdir: str = OBJDIR, extra=()) -> str:
    obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    noise = "'-packed-fp32-ops' is not a recognized feature"
    warn = "\n".join(l for l in r.stderr.splitlines() if noise not in l).strip()
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def stale() -> bool:
    if not os.path.exists(OUT):
        return True
    t = os.path.getmtime(OUT)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def _link(objs, out: str) -> None:
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out + ".tmp", *objs]
    subprocess.check_call(cmd)
    os.replace(out + ".tmp", out)


def build(force: bool = True) -> str:
    """Compile every kernel file and link libpsk.so and the instrumented libpsk_trace.so.  With force=False only
    when sources are newer."""
    if not force and not stale() and os.path.exists(OUT_TRACE) and os.path.getmtime(OUT_TRACE) >= os.path.getmtime(OUT):
        return OUT
    os.makedirs(OBJDIR, exist_ok=True)
    os.makedirs(OBJDIR_TRACE, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        plain = [ex.submit(_compile, s) for s in SOURCES]
        traced = [ex.submit(_compile, s, OBJDIR_TRACE, ("-DPSK_CU_TRACE",)) for s in SOURCES]
        objs = [f.result() for f in plain]
        objs_t = [f.result() for f in traced]
    _link(objs, OUT)
    _link(objs_t, OUT_TRACE)
    return OUT


if __name__ == "__main__":
    print(build(force=True))
