"""The oracle reproduces its committed digest on the tiny workload (drift guard, CPU only)."""
import json
import os

import numpy as np

from tests.golden import make_golden


def test_tiny_digest_is_reproduced():
    path = os.path.join(os.path.dirname(make_golden.__file__), "tiny_oracle.json")
    stored = json.load(open(path))
    now = make_golden.build()
    assert now["perm_ids"] == stored["perm_ids"]
    assert now["bitmask"] == stored["bitmask"] and now["col_idx"] == stored["col_idx"]
    for a, b in zip(now["heads"], stored["heads"]):
        for key in ("idx_sha", "qc_sha", "kc_sha", "vc_sha", "sq", "sk", "sv"):
            assert a[key] == b[key], key
        assert np.allclose(a["o_samples"]["values"], b["o_samples"]["values"], rtol=1e-12, atol=0)
        assert abs(a["o_abs_sum"] - b["o_abs_sum"]) <= 1e-9 * b["o_abs_sum"]
