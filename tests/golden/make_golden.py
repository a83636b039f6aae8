"""Writes tests/golden/tiny_oracle.json: a digest of what the CPU oracle computes on the
"tiny" workload.  Calls only the oracle and the input generators; never the HIP library.
It guards the oracle against silent drift (a regression record, not a pin).

    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import paro_oracle as po  # noqa: E402
from paper_2506_16054_amd import workloads as wl  # noqa: E402
from tests.helpers import blocklist_for, gather_fn, oracle_head  # noqa: E402


def digest(a) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:16]


def build():
    w = wl.WORKLOADS["tiny"]
    perm_ids = wl.make_perm_ids(w)
    masks = wl.make_block_masks(w, gather_fn(w), perm_ids)
    bits, row_ptr, col_idx = blocklist_for(w, masks)
    rec = {"workload": w.name, "seed": w.seed, "perm_ids": perm_ids.tolist(),
           "bitmask": bits.tolist(), "row_ptr": row_ptr.tolist(), "col_idx": col_idx.tolist(), "heads": []}
    for h in range(w.nh):
        q, k, v = wl.make_head_qkv(w, 0, h)
        r = oracle_head(w, q, k, v, perm_ids[h], row_ptr[h], col_idx)
        o = po.cast_output(r["o"], w.dtype)
        rec["heads"].append({
            "idx_sha": digest(r["idx"].astype(np.int32)),
            "qc_sha": digest(r["qc"].astype(np.int8)), "kc_sha": digest(r["kc"].astype(np.int8)),
            "vc_sha": digest(r["vc"].astype(np.int8)),
            "sq": [float(x) for x in r["sq"]], "sk": [float(x) for x in r["sk"]], "sv": [float(x) for x in r["sv"]],
            "o_samples": {"rows": [0, 31, 77, 127], "cols": [0, 63],
                          "values": [[float(o[n, c]) for c in (0, 63)] for n in (0, 31, 77, 127)]},
            "o_abs_sum": float(np.abs(o).sum()),
        })
    return rec


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=1)
    print("wrote", path)
