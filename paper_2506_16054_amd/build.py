"""Compiles the HIP sources under csrc/ for gfx950, in-tree (no JIT cache):

    lib/libparo.so        the product library (everything include/paro.h declares)
    lib/libparo_probe.so  measurement aids of bench.py (csrc/probe/): matrix-rate and instruction-issue probes

    python -m paper_2506_16054_amd.build
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIBDIR = os.path.join(PKG, "lib")
LIBPATH = os.path.join(LIBDIR, "libparo.so")
PROBE_LIBPATH = os.path.join(LIBDIR, "libparo_probe.so")
SOURCES = ("host_api.cpp", "permute.hip", "quantize.hip", "blocklist.hip", "calibrate.hip", "sparse_attn.hip")
PROBE_SOURCES = ("probe/issue_probe.hip",)

# -packed-fp32-ops is switched off on purpose: all float math here is scalar per lane.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def spilling_kernels(remarks: str):
    """(kernel, bytes per lane) of every kernel whose resource report shows scratch memory."""
    out, name = [], None
    for line in remarks.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"remark:\s+ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and int(m.group(1)) > 0:
            out.append((name, int(m.group(1))))
    return out


def _compile(src: str, extra, objdir: str = LIBDIR) -> str:
    obj = os.path.join(objdir, os.path.splitext(os.path.basename(src))[0] + ".o")
    device = src.endswith(".hip")
    report = ["-Rpass-analysis=kernel-resource-usage"] if device else []
    cmd = [hipcc(), *HIPCC_FLAGS, *report, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    # Every kernel here is written to live in registers: a spill to scratch memory in a hot loop
    # costs a multiple of the run time, so it fails the build instead of shipping.
    spills = spilling_kernels(r.stderr) if device else []
    if spills and not os.environ.get("PARO_ALLOW_SPILLS"):
        raise RuntimeError("%s: kernels spill registers to scratch memory: %s" % (src, spills))
    return obj


def _link(out: str, objs) -> None:
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))


def build_library(extra_flags=(), verbose: bool = True, out: str = LIBPATH, probe_out: str | None = PROBE_LIBPATH) -> str:
    """Compile every source and link ``out`` (default: the in-tree library the binding loads) and, unless
    ``probe_out`` is None, the measurement-aid library next to it."""
    objdir = os.path.dirname(out)
    os.makedirs(objdir, exist_ok=True)
    srcs = SOURCES + (PROBE_SOURCES if probe_out else ())
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags), objdir), srcs))
    _link(out, objs[: len(SOURCES)])
    if probe_out:
        os.makedirs(os.path.dirname(probe_out), exist_ok=True)
        _link(probe_out, objs[len(SOURCES):])
    if verbose:
        print("built", out, probe_out or "")
    return out


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
