"""GPU parity on a seeded sweep of small random shapes: grids with extents of 1, sequences shorter
than one block, exact multiples of the block, ragged tails, text tokens, both block sizes and head
dimensions, all bit widths.  Every case is checked against the oracle end to end, and the fused
entry points against the separate steps bit for bit."""
import numpy as np
import pytest

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl
from tests.helpers import (assert_equal_up_to_output_rounding, blocklist_for, check_attention, gather_fn, oracle_head,
                           same_attention_kernel_for_raw_q)
from tests.test_gpu_parity import MAX_ABS, REL_L2, REL_L2_BF16, host, tdtype, to_dev

pytestmark = pytest.mark.gpu


def random_case(i):
    rng = np.random.default_rng([2024, i])
    block = int(rng.choice([32, 64]))
    d = int(rng.choice([64, 128]))
    F, H, W = (int(rng.integers(1, 10 if i % 3 == 0 else 7)) for _ in range(3))
    if i % 5 == 0:
        F, H, W = 1, 1, int(rng.integers(1, block))  # shorter than one block
    if i % 7 == 0:
        F, H, W = 2, block // 2, int(rng.integers(1, 4))  # exact multiple of the block
    n_img = F * H * W
    T_text = int(rng.choice([0, 0, block, 2 * block])) if n_img % block == 0 else 0
    bits = [(8, 8), (8, 4), (4, 4), (4, 8), (16, 16)][i % 5]
    dtype = "bf16" if rng.random() < 0.5 else "f32"
    nh = int(rng.integers(1, 4))
    B = int(rng.integers(1, 3))
    density = float(rng.choice([0.15, 0.4, 0.8, 1.0]))
    return wl.Workload("rand%d" % i, B, nh, d, F, H, W, T_text, block, density, bits[0], bits[1], dtype, 9000 + i)


@pytest.mark.parametrize("i", range(64))
def test_random_shape(i):
    import torch

    from paper_2506_16054_amd import binding as pb
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = random_case(i)
    s = pb.shape_of(w)
    perm_ids = wl.make_perm_ids(w)
    masks = wl.make_block_masks(w, gather_fn(w), perm_ids)
    bm, row_ptr, col_idx = blocklist_for(w, masks)
    q, k, v = wl.make_qkv(w)
    dq, dk, dv = (to_dev(x, w.dtype) for x in (q, k, v))
    pa = ParoAttention(s, perm_ids, bm, w.bits_qk, w.bits_pv, tdtype(w.dtype))
    assert np.array_equal(pa.h_row_ptr, row_ptr) and np.array_equal(pa.h_col_idx, col_idx)
    o_sep = pa.run(dq, dk, dv).clone()
    o_fused = pa.run_fused(dq, dk, dv).clone()
    torch.cuda.synchronize()
    assert torch.equal(o_sep, o_fused), "fused entry points differ from the separate steps"
    if pa.can_fuse_q:
        if same_attention_kernel_for_raw_q(w):
            assert torch.equal(pa.run_rawq(dq, dk, dv), o_fused), "in-kernel Q quantization differs"
        else:
            assert_equal_up_to_output_rounding(pa.run_rawq(dq, dk, dv), o_fused, "in-kernel Q quantization")
    pa.prepare_fused_qkv(dq, dk, dv)
    assert torch.equal(pa.attend_fused(), o_fused), "the one-launch quantizer differs from the three calls"
    saved = pa.row_order
    pa.row_order = None
    assert torch.equal(pa.run_fused(dq, dk, dv), o_fused), "the launch order changed the result"
    pa.row_order = saved
    got = host(o_fused)
    rel = REL_L2_BF16 if w.bits_qk == 16 else REL_L2
    for b in range(w.B):
        for h in range(w.nh):
            r = oracle_head(w, q[b, h], k[b, h], v[b, h], perm_ids[h], row_ptr[h], col_idx)
            check_attention(got[b, h], r["o"], po.unpermute(r["flip_risk"], r["idx"]), MAX_ABS, rel, "%s b%d h%d" % (w.name, b, h))


# Rows with more than 64 and more than 128 live blocks: the kernels fetch the column indices of a
# row 64 at a time, one chunk ahead, so these lengths cross one and two chunk changes.  Block 32
# keeps the sequences short enough for the oracle to check every element.
LONG_ROWS = {
    "k130_dense_i8": wl.Workload("k130_dense_i8", 1, 1, 64, 2, 8, 259, 0, 32, 1.0, 8, 8, "bf16", 9101),   # N = 4144, ragged
    "k66_int4pv_d128": wl.Workload("k66_int4pv_d128", 1, 1, 128, 1, 11, 190, 0, 32, 0.9, 8, 4, "f32", 9102),  # N = 2090
    "k129_bf16": wl.Workload("k129_bf16", 1, 1, 64, 3, 4, 343, 0, 32, 1.0, 16, 16, "f32", 9103),          # N = 4116
    "k140_i4i4_b64": wl.Workload("k140_i4i4_b64", 1, 1, 64, 2, 7, 638, 0, 64, 0.6, 4, 4, "bf16", 9104),     # N = 8932
}


@pytest.mark.parametrize("name", list(LONG_ROWS))
def test_long_live_lists(name):
    import torch

    from paper_2506_16054_amd import binding as pb
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = LONG_ROWS[name]
    s = pb.shape_of(w)
    perm_ids = wl.make_perm_ids(w)
    masks = wl.make_block_masks(w, gather_fn(w), perm_ids)
    bm, row_ptr, col_idx = blocklist_for(w, masks)
    longest = int(np.max(np.diff(row_ptr[0])))
    assert longest > (128 if w.k > 128 else 64)
    q, k, v = wl.make_qkv(w)
    dq, dk, dv = (to_dev(x, w.dtype) for x in (q, k, v))
    pa = ParoAttention(s, perm_ids, bm, w.bits_qk, w.bits_pv, tdtype(w.dtype))
    o_fused = pa.run_fused(dq, dk, dv).clone()
    assert torch.equal(pa.run(dq, dk, dv), o_fused)
    got = host(o_fused)
    r = oracle_head(w, q[0, 0], k[0, 0], v[0, 0], perm_ids[0], row_ptr[0], col_idx)
    rel = REL_L2_BF16 if w.bits_qk == 16 else REL_L2
    st = check_attention(got[0, 0], r["o"], po.unpermute(r["flip_risk"], r["idx"]), MAX_ABS, rel, name)
    print("%s: N %d, longest row %d blocks, max_abs %.2e rel_l2 %.2e" % (name, w.N, longest, st["max_abs"], st["rel_l2"]))
