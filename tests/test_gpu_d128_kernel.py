"""GPU parity of the attention kernel that d = 128 / block 64 / 8-bit codes launch (four wavefronts of 16 queries per
row block), on the shapes where its bookkeeping can go wrong: a ragged last block with several blocks before it
(keys past N masked, padded query rows in wavefronts that hold no real row at all), text tokens with a ragged
tail, rows of 1, 2 and 3 live blocks (the request pipeline's start-up cases), an empty row, rows of more than 64
live blocks (a second chunk of the column list), logits that climb by hundreds of octaves.  Every case through the
separate steps AND the fused entry points (which must agree bit for bit), against the oracle at the stated bar."""
import numpy as np
import pytest

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl
from tests.helpers import blocklist_for, check_attention, gather_fn, oracle_head
from tests.test_gpu_parity import MAX_ABS, REL_L2, host, tdtype, to_dev

pytestmark = pytest.mark.gpu

CASES = {
    # 189 = 2 * 64 + 61 tokens, batch 2
    "ragged": wl.Workload("q16_ragged", 2, 2, 128, 3, 7, 9, 0, 64, 0.6, 8, 8, "bf16", 41, perm_choice=(2, 5)),
    # 128 image tokens (two whole blocks) + 37 text tokens: the text block is the ragged one
    "text_ragged": wl.Workload("q16_text", 1, 2, 128, 1, 8, 16, 37, 64, 0.5, 8, 8, "f32", 42, perm_choice=(1, 4)),
    # 578 = 9 * 64 + 2 tokens: two real rows in the last row block, three of its four wavefronts hold padded rows only
    "few_real_rows": wl.Workload("q16_few", 1, 1, 128, 2, 17, 17, 0, 64, 0.3, 8, 8, "bf16", 43, perm_choice=(3,)),
    # 4350 = 67 * 64 + 62 tokens, every block live: rows of 68 blocks, two chunks of the column list
    "long_dense": wl.Workload("q16_long", 1, 1, 128, 5, 29, 30, 0, 64, 1.0, 8, 8, "bf16", 44, perm_choice=(5,)),
}


def _run_and_check(w, masks, q, k, v, what):
    import torch

    from paper_2506_16054_amd import binding as pb
    from paper_2506_16054_amd.pipeline import ParoAttention

    perm_ids = wl.make_perm_ids(w)
    bm, row_ptr, col_idx = blocklist_for(w, masks)
    pa = ParoAttention(pb.shape_of(w), perm_ids, bm, 8, 8, tdtype(w.dtype))
    dq, dk, dv = (to_dev(x, w.dtype) for x in (q, k, v))
    pa.op.fill_(float("nan"))
    pa.o.fill_(float("nan"))
    o_sep = pa.run(dq, dk, dv).clone()
    pa.o.fill_(float("nan"))
    o_fused = pa.run_fused(dq, dk, dv)
    torch.cuda.synchronize()
    assert torch.equal(o_sep, o_fused)
    assert not torch.isnan(o_fused).any() and bool((pa.op[:, :, w.N:] == 0).all())
    got = host(o_fused)
    stats = []
    for b in range(w.B):
        for h in range(w.nh):
            r = oracle_head(w, q[b, h], k[b, h], v[b, h], perm_ids[h], row_ptr[h], col_idx)
            stats.append(check_attention(got[b, h], r["o"], po.unpermute(r["flip_risk"], r["idx"]), MAX_ABS, REL_L2, "%s b%d h%d" % (what, b, h)))
    return row_ptr, stats


@pytest.mark.parametrize("name", sorted(CASES))
def test_edge_shapes(name):
    w = CASES[name]
    assert w.N % w.block != 0
    masks = wl.make_block_masks(w, gather_fn(w), wl.make_perm_ids(w))
    q, k, v = wl.make_qkv(w)
    row_ptr, _ = _run_and_check(w, masks, q, k, v, name)
    if name == "long_dense":
        assert int(np.diff(row_ptr[0]).max()) == w.k > 64


def test_rows_of_one_two_three_and_no_live_blocks():
    w = CASES["ragged"].replace(B=1, nh=1, perm_choice=(0,), F=5, Hg=8, Wg=9, seed=45)  # 360 tokens, 6 blocks, ragged
    assert w.k == 6 and w.N % 64 != 0
    masks = np.zeros((1, 6, 6), bool)
    masks[0, 0, [5]] = True            # one live block, and it is the ragged one
    masks[0, 1, [0, 5]] = True         # two
    masks[0, 2, [1, 2, 4]] = True      # three
    masks[0, 4, :] = True              # all
    masks[0, 5, [0, 1, 2, 3]] = True   # the ragged row block (40 real rows), no diagonal; row block 3 attends nothing
    q, k, v = wl.make_qkv(w)
    row_ptr, _ = _run_and_check(w, masks, q, k, v, "short rows")
    assert np.diff(row_ptr[0]).tolist() == [1, 2, 3, 0, 6, 4]


def test_row_maximum_climbing_hundreds_of_octaves():
    w = CASES["ragged"].replace(B=1, nh=2, perm_choice=(0, 0), density=1.0, dtype="f32", seed=46)
    masks = wl.make_block_masks(w, gather_fn(w))
    rng = np.random.default_rng(47)
    ramp = np.linspace(0.05, 9.0, w.N)[:, None]
    q = np.abs(rng.standard_normal((1, 2, w.N, w.d))).astype(np.float32) * 3
    k = np.abs(rng.standard_normal((1, 2, w.N, w.d))).astype(np.float32)
    k[0, 0] *= ramp
    k[0, 1] *= ramp[::-1]
    v = rng.standard_normal((1, 2, w.N, w.d)).astype(np.float32)
    _, stats = _run_and_check(w, masks, q, k, v, "steep")
    logit = (q[0, 0, :1].astype(np.float64) @ k[0, 0].astype(np.float64).T) / np.sqrt(w.d) * np.log2(np.e)
    assert logit.max() - logit.min() > 200
    assert max(s["rel_l2"] for s in stats) < 3e-3
