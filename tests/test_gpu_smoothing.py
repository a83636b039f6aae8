"""GPU parity of the optional K pre-conditioning (paro_k_channel_mean, paro_permute_quantize_smoothed) through the
C ABI: the channel means and the codes and scales of the smoothed keys bit for bit against the oracle, the attention
output of the smoothed path at the stated bar."""
import numpy as np
import pytest

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl
from tests.helpers import blocklist_for, check_attention, gather_fn, oracle_head
from tests.test_gpu_parity import MAX_ABS, REL_L2, SMALL, host, tdtype, to_dev, unpack_rows_int4

pytestmark = pytest.mark.gpu


def _offset_keys(w, k):
    """Keys with a per-channel offset of several standard deviations, the case smoothing is for."""
    rng = np.random.default_rng(w.seed + 5)
    off = rng.uniform(-6.0, 6.0, size=(1, w.nh, 1, w.d)).astype(np.float32)
    k = (k + off).astype(np.float32)
    return po.round_to_bf16(k).astype(np.float32) if w.dtype == "bf16" else k


@pytest.mark.parametrize("name", ["video64", "video32_f32", "flux128", "video64_i4i4", "video64_int4"])
def test_smoothed_keys_and_attention_match_the_oracle(name):
    import torch

    from paper_2506_16054_amd import binding as pb
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = SMALL[name]
    s = pb.shape_of(w)
    perm_ids = wl.make_perm_ids(w)
    masks = wl.make_block_masks(w, gather_fn(w), perm_ids)
    bm, row_ptr, col_idx = blocklist_for(w, masks)
    q, k, v = wl.make_qkv(w)
    k = _offset_keys(w, k)
    dq, dk, dv = (to_dev(x, w.dtype) for x in (q, k, v))
    pa = ParoAttention(s, perm_ids, bm, w.bits_qk, w.bits_pv, tdtype(w.dtype))
    pa.o.fill_(float("nan"))
    got = host(pa.run_fused_smooth_k(dq, dk, dv))
    torch.cuda.synchronize()
    assert not np.isnan(got).any()
    mean = pa.k_mean.cpu().numpy()
    _, fk = pa._fused_buffers()
    for b in range(w.B):
        for h in range(w.nh):
            assert np.array_equal(mean[b, h], po.k_channel_mean(k[b, h])), "channel means of head %d" % h
            ks = po.smooth_k(k[b, h])
            r = oracle_head(w, q[b, h], ks, v[b, h], perm_ids[h], row_ptr[h], col_idx)
            g_k = fk[b, h].cpu().numpy()
            g_k = unpack_rows_int4(g_k) if w.bits_qk == 4 else g_k
            assert np.array_equal(g_k.astype(np.int32), r["kc"]), "codes of the smoothed keys, head %d" % h
            assert np.array_equal(pa.sk[b, h].cpu().numpy(), r["sk"])
            check_attention(got[b, h], r["o"], po.unpermute(r["flip_risk"], r["idx"]), MAX_ABS, REL_L2, "%s smoothed b%d h%d" % (name, b, h))
    # the offset dominated the scales of the plain path: smoothing must have shrunk them
    plain = ParoAttention(s, perm_ids, bm, w.bits_qk, w.bits_pv, tdtype(w.dtype))
    plain.run_fused(dq, dk, dv)
    torch.cuda.synchronize()
    assert float((pa.sk / plain.sk).max()) < 0.9


def test_channel_mean_of_a_long_head_is_bit_exact():
    """N = 17550 tokens, the length of the video workloads: 137 passes of the workgroup, a ragged last pass."""
    import torch

    from paper_2506_16054_amd import binding as pb

    for d, dtype in ((64, "bf16"), (128, "f32")):
        w = wl.Workload("mean", 1, 2, d, 13, 30, 45, 0, 64, 0.3, 8, 8, dtype, 31)
        s = pb.shape_of(w)
        rng = np.random.default_rng(d)
        k = (rng.standard_normal((1, 2, w.N, d)) * 2.0 + rng.uniform(-5, 5, size=(1, 2, 1, d))).astype(np.float32)
        if dtype == "bf16":
            k = po.round_to_bf16(k).astype(np.float32)
        mean = torch.empty((1, 2, d), dtype=torch.float32, device="cuda:0")
        pb.paro_k_channel_mean(s, to_dev(k, dtype), mean)
        torch.cuda.synchronize()
        for h in range(2):
            assert np.array_equal(mean[0, h].cpu().numpy(), po.k_channel_mean(k[0, h]))
