"""Compiles the HIP sources under csrc/ for gfx950, in-tree (no JIT cache):

    lib/libparo.so        the product library (everything include/paro.h declares)
    lib/libparo_probe.so  measurement aids of bench.py (csrc/probe/): matrix-rate and instruction-issue probes
    lib/libparo_timeline.so  the product library with sparse_attn.hip compiled under -DPARO_TIMELINE=1 (every wavefront of
                          the attention kernels records its start and end clock; read by `probe --timeline`)

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
TIMELINE_LIBNAME = "libparo_timeline.so"
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


def _compile(src: str, extra, objdir: str = LIBDIR, tag: str = "") -> str:
    obj = os.path.join(objdir, os.path.splitext(os.path.basename(src))[0] + tag + ".o")
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


# ---- static instruction counts of the attention kernels' block loops (read by bench.py) --------------------
_RARE = 12  # a loop block with this many v_cndmask or v_mul is a rarely taken branch (ragged-tail masking, re-referencing)


def instruction_class(op: str) -> str:
    """Issue class of a vector instruction mnemonic, as priced by the instruction-issue probe."""
    op = re.sub(r"_(e32|e64|dpp|sdwa)$", "", op)
    if "mfma" in op:
        return "mfma_16x16" if "_16x16x" in op else "mfma"
    if op in ("v_exp_f32", "v_rcp_f32", "v_log_f32", "v_rsq_f32", "v_sqrt_f32", "v_exp_f16"):
        return "transcendental"
    if op.startswith("v_permlane"):
        return "permlane_swap"
    if op in ("v_fma_f32", "v_fmac_f32", "v_fmamk_f32", "v_fmaak_f32"):
        return "fma"
    if op in ("v_add_f32", "v_sub_f32", "v_subrev_f32", "v_mul_f32"):
        return "add_mul"
    if op in ("v_add_u32", "v_sub_u32", "v_subrev_u32", "v_and_b32", "v_or_b32", "v_xor_b32", "v_mov_b32", "v_lshlrev_b32", "v_lshrrev_b32"):
        return "int_simple"
    return "half_rate"  # max/min, conversions, byte permute, cross-lane moves, 64-bit address arithmetic, ...


def loop_instruction_counts(asm: str) -> dict:
    """{kernel symbol: [ {class: count per loop iteration}, ... one entry per innermost loop that holds matrix
    instructions ]} from the compiler's assembly listing.  Loop blocks that are rarely taken branches are left out."""
    out = {}
    for m in re.finditer(r"^(_ZN4paro\w*attn\w+):[^\n]*\n(.*?)\n\s*s_endpgm", asm, re.S | re.M):
        name, body = m.group(1), m.group(2)
        loops, label, header = {}, None, None
        for line in body.split("\n"):
            t = line.strip()
            lm = re.match(r"^(\.LBB\d+_\d+):\s*(;.*)?$", t)
            if lm:
                label, note = lm.group(1), lm.group(2) or ""
                hm = re.search(r"Header=(BB\d+_\d+)", note)
                header = "." + "L" + hm.group(1) if hm else (label if "Loop Header" in note else None)
                if header:
                    loops.setdefault(header, []).append([])
                continue
            if header and t and not t.startswith(";") and not t.startswith("."):
                op = t.split()[0]
                if op.startswith("v_"):
                    loops[header][-1].append(op)
                elif op.startswith("s_cbranch") or op == "s_branch":
                    loops[header].append([])  # what follows a branch is another basic block
        entries = []
        for blocks in loops.values():
            counts = {}
            for ops in blocks:
                if sum(o.startswith("v_cndmask") for o in ops) >= _RARE or sum(o.startswith("v_mul_f32") for o in ops) >= _RARE:
                    continue
                for o in ops:
                    c = instruction_class(o)
                    counts[c] = counts.get(c, 0) + 1
            if counts.get("mfma") or counts.get("mfma_16x16"):
                entries.append(counts)
        if entries:
            out[name] = entries
    return out


def write_loop_counts(extra, objdir: str) -> str:
    import json

    asm_path = os.path.join(objdir, "sparse_attn.s")
    cmd = [hipcc(), *HIPCC_FLAGS, *extra, "-S", "--cuda-device-only", os.path.join(CSRC, "sparse_attn.hip"), "-o", asm_path]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc -S failed on sparse_attn.hip:\n%s" % r.stderr)
    counts = loop_instruction_counts(open(asm_path).read())
    os.remove(asm_path)
    path = os.path.join(objdir, "attn_loop_counts.json")
    with open(path, "w") as f:
        json.dump(counts, f, indent=1, sort_keys=True)
    return path


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
        counts = ex.submit(write_loop_counts, list(extra_flags), objdir)
        timeline = ex.submit(_compile, "sparse_attn.hip", [*extra_flags, "-DPARO_TIMELINE=1"], objdir, "_timeline") if probe_out else None
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags), objdir), srcs))
        counts.result()
        timeline_obj = timeline.result() if timeline else None
    _link(out, objs[: len(SOURCES)])
    if probe_out:
        os.makedirs(os.path.dirname(probe_out), exist_ok=True)
        _link(probe_out, objs[len(SOURCES):])
        others = [o for o, src in zip(objs, SOURCES) if src != "sparse_attn.hip"]
        _link(os.path.join(os.path.dirname(probe_out), TIMELINE_LIBNAME), others + [timeline_obj])
    if verbose:
        print("built", out, probe_out or "")
    return out


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
