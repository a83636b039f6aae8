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
