"""The build refuses kernels that spill registers to scratch memory: the parser of the compiler's
resource report is checked here on a canned report (no compiler run)."""
from paper_2506_16054_amd.build import spilling_kernels

REPORT = """a.hip:13:1: remark: Function Name: _ZN4paro6kern_aEv [-Rpass-analysis=kernel-resource-usage]
a.hip:13:1: remark:     TotalSGPRs: 27 [-Rpass-analysis=kernel-resource-usage]
a.hip:13:1: remark:     VGPRs: 150 [-Rpass-analysis=kernel-resource-usage]
a.hip:13:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:13:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:40:1: remark: Function Name: _ZN4paro6kern_bEv [-Rpass-analysis=kernel-resource-usage]
a.hip:40:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]
a.hip:40:1: remark:     ScratchSize [bytes/lane]: 216 [-Rpass-analysis=kernel-resource-usage]
a.hip:40:1: remark:     VGPRs Spill: 54 [-Rpass-analysis=kernel-resource-usage]
'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)
"""


def test_spill_report_names_only_kernels_with_scratch():
    assert spilling_kernels(REPORT) == [("_ZN4paro6kern_bEv", 216)]
    assert spilling_kernels("") == []
    assert spilling_kernels(REPORT.replace("216", "0")) == []


def test_kernels_contain_no_inline_assembly_instructions():
    """An instruction written as inline assembly is invisible to the compiler's hazard handling (a
    conversion placed directly behind the exponential it consumes needs a wait state that only
    compiler-visible instructions get), so the kernels use builtins; the one `asm` left is the empty
    optimization barrier.  (csrc/probe/ is not part of the product library: its instruction-issue probes
    time single named instructions and are written in assembly on purpose.)"""
    import glob
    import os
    import re

    from paper_2506_16054_amd.build import CSRC

    found = []
    for path in sorted(p for p in glob.glob(os.path.join(CSRC, "*")) if os.path.isfile(p)):
        text = open(path).read()
        for m in re.finditer(r"\basm\s*(?:volatile)?\s*\(\s*\"([^\"]*)\"", text):
            if m.group(1).strip():
                found.append((os.path.basename(path), m.group(1)))
    assert found == [], found


LISTING = """\t.text
_ZN4paro11attn_i8_demoEv:                ; @_ZN4paro11attn_i8_demoEv
; %bb.0:
\tv_mov_b32_e32 v1, 0
\ts_cbranch_scc1 .LBB0_3
.LBB0_1:                                ; =>This Inner Loop Header: Depth=1
\tv_mfma_i32_32x32x32_i8 v[0:15], v[16:19], v[20:23], v[0:15]
\tv_fma_f32 v1, v2, v3, v4
\tv_fmac_f32_e32 v1, v2, v3
\tv_add_f32_e32 v1, v2, v3
\tv_exp_f32_e32 v1, v1
\tv_max3_i32 v1, v2, v3, v4
\tv_permlane32_swap_b32_e32 v1, v2
\tv_add_u32_e32 v1, v2, v3
\ts_nop 1
\tds_read_b128 v[4:7], v8
\ts_cbranch_vccz .LBB0_1
.LBB0_2:                                ; =>This Inner Loop Header: Depth=1
\tv_add_f32_e32 v1, v2, v3
\ts_cbranch_vccz .LBB0_2
.LBB0_3:
\ts_endpgm
"""


def test_loop_instruction_counts_reads_the_loops_that_hold_matrix_instructions():
    """bench.py's issue-cost roofline multiplies these counts by measured per-class costs: the parser must count
    vector instructions of loop blocks only, class them as the probe prices them, and skip loops without
    matrix instructions."""
    from paper_2506_16054_amd.build import instruction_class, loop_instruction_counts

    got = loop_instruction_counts(LISTING)
    assert got == {"_ZN4paro11attn_i8_demoEv": [{"mfma": 1, "fma": 2, "add_mul": 1, "transcendental": 1, "half_rate": 1,
                                                 "permlane_swap": 1, "int_simple": 1}]}
    assert instruction_class("v_cvt_pknorm_u16_f32") == "half_rate"
    assert instruction_class("v_mul_f32_e32") == "add_mul"


def test_probe_library_exports_what_bench_calls():
    """lib/libparo_probe.so is a measurement aid next to the product library; bench.py fails if it is missing."""
    import ctypes
    import os

    import torch  # noqa: F401  (before the library, as probe.lib() does: both must bind to the same HIP runtime)

    from paper_2506_16054_amd.probe import LIBPATH

    assert os.path.exists(LIBPATH), "build with python -m paper_2506_16054_amd.build"
    lib = ctypes.CDLL(LIBPATH)
    for name in ("paro_probe_mfma", "paro_probe_last_error", "paro_probe_issue_kinds", "paro_probe_issue_name", "paro_probe_issue",
                 "paro_probe_block", "paro_probe_pair", "paro_probe_copy"):
        assert hasattr(lib, name), name
    assert lib.paro_probe_issue_kinds() >= 22


def test_timeline_library_is_the_product_plus_the_record_reader_and_the_product_has_no_recorder():
    """lib/libparo_timeline.so (read by `probe --timeline`) exports everything the product library does plus
    paro_timeline_read; the product library itself carries no timeline code."""
    import ctypes
    import os

    import torch  # noqa: F401

    from paper_2506_16054_amd import binding as pb

    timeline = os.path.join(os.path.dirname(pb.LIBPATH), "libparo_timeline.so")
    assert os.path.exists(timeline), "build with python -m paper_2506_16054_amd.build"
    tl = ctypes.CDLL(timeline)
    for name in pb.EXPORTS:
        assert hasattr(tl, name), name
    assert hasattr(tl, "paro_timeline_read")
    assert not hasattr(ctypes.CDLL(pb.LIBPATH), "paro_timeline_read")


def test_bench_refuses_more_than_one_gpu():
    """The whole build runs on one GPU; the bench says so instead of timing anything (no GPU is touched)."""
    import os
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr + r.stdout
    assert not r.stdout.strip().startswith("{")
