"""The parallel whole-head driver of the oracle (used by the full-size GPU parity tests) returns
exactly what a plain serial call returns."""
import numpy as np

from paper_2506_16054_amd import workloads as wl
from tests.helpers import blocklist_for, gather_fn, oracle_head, oracle_whole_heads


def test_whole_heads_in_worker_processes_equal_the_serial_oracle():
    w = wl.Workload("par", 1, 2, 64, 3, 6, 7, 0, 32, 0.5, 8, 8, "f32", 21, perm_choice=(4, 1))
    perm_ids = wl.make_perm_ids(w)
    masks = wl.make_block_masks(w, gather_fn(w), perm_ids)
    _, row_ptr, col_idx = blocklist_for(w, masks)
    q, k, v = wl.make_qkv(w)
    got = oracle_whole_heads(w, (0, 1), lambda h: (q[0, h], k[0, h], v[0, h]), perm_ids, row_ptr, col_idx, workers=3)
    for h in (0, 1):
        ref = oracle_head(w, q[0, h], k[0, h], v[0, h], perm_ids[h], row_ptr[h], col_idx)
        assert np.array_equal(got[h][0], ref["op"])
        assert np.array_equal(got[h][1], ref["flip_risk"])
