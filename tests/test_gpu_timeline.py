"""The measurement build of the attention kernels works on the box (it is not part of the product path)."""
import pytest


@pytest.mark.gpu
def test_timeline_build_records_every_wavefront_of_a_launch():
    """The measurement build of the attention kernels (lib/libparo_timeline.so, `probe --timeline`) on a small d = 64 /
    block 64 layer, in a process of its own because it takes the product library's place: one record per row block,
    each with a start before its end and the row's number of live blocks."""
    import os
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import numpy as np\n"
        "from paper_2506_16054_amd import probe, workloads as wl\n"
        "w = wl.Workload('t64', 1, 16, 64, 4, 12, 16, 0, 64, 0.4, 8, 8, 'bf16', 31)\n"
        "wl.WORKLOADS['t64'] = w\n"
        "text = probe.timeline('t64', records_path='/tmp/paro_t64_timeline.npy')\n"
        "rec = np.load('/tmp/paro_t64_timeline.npy')\n"
        "assert rec.shape == (16 * w.k, 8) and (rec[:, 1] > rec[:, 0]).all()\n"
        "assert rec[:, 2].sum() == round(0.4 * w.k * w.k) * 16, (rec[:, 2].sum(), w.k)\n"
        "print(text.splitlines()[0])\n"
    )
    r = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "192 wavefronts (1 per row block)" in r.stdout
