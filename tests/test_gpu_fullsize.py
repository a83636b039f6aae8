"""GPU parity at the full benchmark shapes, in the launch configuration bench.py times.

The whole workload runs on the GPU through the C ABI.  For the listed heads the oracle recomputes
EVERY row block (worker processes, tests/helpers.oracle_whole_heads): codes and scales of the whole
head bit for bit, the attention output of the whole head element by element at the stated bar.
The forms of the path that bench.py times (one quantizer launch + attention with the inverse reorder in
its stores, scheduled launch order) must reproduce the oracle-checked five-step result bit for bit on
the WHOLE tensor, which ties every row of every head of the timed path to the checked one; so must the
entry point that quantizes Q inside the attention kernel wherever it runs the same attention kernel
(elsewhere: equal up to the rounding of the output).  Properties that hold at any size are checked on the full
tensors: the reorder round trip is the identity, padded rows are zero, nothing is NaN."""
import numpy as np
import pytest

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl
from tests.helpers import assert_equal_up_to_output_rounding, check_attention, oracle_whole_heads, same_attention_kernel_for_raw_q
from tests.test_gpu_parity import MAX_ABS, REL_L2, REL_L2_BF16, host, tdtype, unpack_rows_int4, unpack_vt_int4, vt_to_rows

pytestmark = pytest.mark.gpu


def run_full(w):
    import torch

    from paper_2506_16054_amd import binding as pb
    from paper_2506_16054_amd.pipeline import ParoAttention

    s = pb.shape_of(w)
    perm_ids = wl.make_perm_ids(w)
    masks = wl.make_block_masks(w, lambda pid: pb.paro_perm_index(s, pid), perm_ids)
    bitmask = wl.pack_bitmask(masks)
    dev = torch.device("cuda:0")
    q = torch.empty((w.B, w.nh, w.N, w.d), dtype=tdtype(w.dtype), device=dev)
    k, v = torch.empty_like(q), torch.empty_like(q)
    for h in range(w.nh):
        hq, hk, hv = wl.make_head_qkv(w, 0, h)
        q[0, h], k[0, h], v[0, h] = (torch.from_numpy(x).to(dev) for x in (hq, hk, hv))
    pa = ParoAttention(s, perm_ids, bitmask, w.bits_qk, w.bits_pv, tdtype(w.dtype), dev)
    pa.op.fill_(float("nan"))
    pa.o.fill_(float("nan"))
    o = pa.run(q, k, v).clone()
    torch.cuda.synchronize()
    return pa, perm_ids, masks, (q, k, v), o


def check_timed_forms(w, pa, q, k, v, o):
    """Every form of the path that bench.py times, against the five-step result, whole tensor."""
    import torch

    pa.o.fill_(float("nan"))
    pa.prepare_fused_qkv(q, k, v)
    assert torch.equal(pa.attend_fused(), o), "%s: one-launch quantizer + attention with inverse reorder differs" % w.name
    if pa.can_fuse_q:
        pa.o.fill_(float("nan"))
        if same_attention_kernel_for_raw_q(w):
            assert torch.equal(pa.run_rawq(q, k, v), o), "%s: attention that quantizes its own Q differs" % w.name
        else:
            assert_equal_up_to_output_rounding(pa.run_rawq(q, k, v), o, "%s: attention that quantizes its own Q" % w.name)
    # the launch order is a schedule, not arithmetic: with and without it the result is the same
    order = pa.row_order
    pa.use_blocklist(pa.row_ptr, pa.col_idx, None)
    pa.o.fill_(float("nan"))
    pa.prepare_fused_qkv(q, k, v)
    assert torch.equal(pa.attend_fused(), o), "%s: unscheduled launch order differs" % w.name
    pa.use_blocklist(pa.row_ptr, pa.col_idx, order)
    torch.cuda.synchronize()


def check_whole_heads(w, heads):
    import torch

    from paper_2506_16054_amd import binding as pb

    pa, perm_ids, masks, (q, k, v), o = run_full(w)
    assert pa.live_blocks == int(masks.sum()) * w.B
    # --- properties on the full tensors
    assert not torch.isnan(pa.op).any() and not torch.isnan(o).any()
    assert bool((pa.op[:, :, w.N:] == 0).all())
    back = torch.empty_like(q)
    pb.paro_unpermute(pa.s, perm_ids, pa.xp[0], back)
    torch.cuda.synchronize()
    assert torch.equal(back, q)  # reorder followed by its inverse is the identity, bit for bit
    # --- the timed forms of the path reproduce this result on every row of every head
    check_timed_forms(w, pa, q, k, v, o)
    # --- whole heads against the oracle
    rel = REL_L2_BF16 if w.bits_qk == 16 else REL_L2
    refs = oracle_whole_heads(w, heads, lambda h: tuple(host(t[0, h]) for t in (q, k, v)), perm_ids, pa.h_row_ptr, pa.h_col_idx)
    for h in heads:
        hq, hk, hv = (host(t[0, h]) for t in (q, k, v))
        idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, int(perm_ids[h]))
        assert np.array_equal(pb.paro_perm_index(pa.s, int(perm_ids[h])), idx)
        if w.bits_qk != 16:
            qc, sq = po.prepare_operand(hq, idx, w.npad, w.block, w.bits_qk)
            kc, sk = po.prepare_operand(hk, idx, w.npad, w.block, w.bits_qk)
            vc, sv = po.prepare_operand(hv, idx, w.npad, w.block, w.bits_pv)
            g_q, g_k = pa.qc[0, h].cpu().numpy(), pa.kc[0, h].cpu().numpy()
            if w.bits_qk == 4:
                g_q, g_k = unpack_rows_int4(g_q), unpack_rows_int4(g_k)
            assert np.array_equal(g_q.astype(np.int32), qc)
            assert np.array_equal(g_k.astype(np.int32), kc)
            g_vc = pa.vc[0, h].cpu().numpy()
            g_vc = unpack_vt_int4(g_vc) if w.bits_pv == 4 else g_vc.astype(np.int32)
            assert np.array_equal(vt_to_rows(g_vc, w.block), vc)
            for g_s, o_s in ((pa.sq, sq), (pa.sk, sk), (pa.sv, sv)):
                assert np.array_equal(g_s[0, h].cpu().numpy(), o_s)
        ref_p, risk_p = refs[h]
        got_p = host(pa.op[0, h])
        check_attention(got_p[: w.N], ref_p[: w.N], risk_p[: w.N], MAX_ABS, rel, "%s head %d, all %d row blocks" % (w.name, h, w.k))
        # the inverse reorder of the whole head
        assert np.array_equal(host(o[0, h])[idx], got_p[: w.N])


def test_headline_cogvideox5b_int8():
    check_whole_heads(wl.WORKLOADS["cogvideox5b"], heads=(0, 17, 47))


def test_cogvideox5b_int4_pv():
    check_whole_heads(wl.WORKLOADS["cogvideox5b_int4pv"], heads=(5, 30))


def test_cogvideox2b_density_half():
    check_whole_heads(wl.WORKLOADS["cogvideox2b"], heads=(3, 29))


def test_flux_text_blocks_d128():
    check_whole_heads(wl.WORKLOADS["flux"], heads=(0, 11, 23))


def test_headline_shape_bf16_mode():
    check_whole_heads(wl.WORKLOADS["cogvideox5b"].replace(name="cogvideox5b_bf16", bits_qk=16, bits_pv=16, nh=8), heads=(2, 7))


def test_headline_shape_all_int4():
    check_whole_heads(wl.WORKLOADS["cogvideox5b"].replace(name="cogvideox5b_i4i4", bits_qk=4, bits_pv=4, density=0.5, nh=8), heads=(1, 6))


def test_headline_shape_calibration_sampled():
    """Offline calibration (Sec. 4.1 metric, Sec. 4.2 (3) masks) at N = 17550 on 8 heads: properties that
    hold at any size on every head; one head's metrics of one axis order against the oracle over the
    whole map (row block by row block); sampled row blocks of the chosen orders' block sums."""
    import time

    import torch

    from oracle import paro_calibration as pc
    from paper_2506_16054_amd import binding as pb
    from paper_2506_16054_amd import pipeline
    from tests.test_gpu_calibration import EPS, REL, SIGMA, TIE, stats_on_gpu

    w = wl.WORKLOADS["cogvideox5b"].replace(name="cogvideox5b_calib", nh=8)
    s = pb.shape_of(w)
    q = np.empty((1, w.nh, w.N, w.d), np.float32)
    k = np.empty_like(q)
    for h in range(w.nh):
        q[0, h], k[0, h], _ = wl.make_head_qkv(w, 0, h)
    dq, dk = (torch.from_numpy(x).to("cuda:0").to(torch.bfloat16) for x in (q, k))
    pipeline.calibrate(s, dq, dk, EPS, SIGMA, 0.5, w.density)  # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    res = pipeline.calibrate(s, dq, dk, EPS, SIGMA, 0.5, w.density)
    torch.cuda.synchronize()
    print("calibration of %d heads at N=%d: %.1f ms" % (w.nh, w.N, (time.perf_counter() - t0) * 1e3))
    bsum = res["block_sum"].cpu().numpy()
    perm = res["h_perm_ids"]
    bits = res["bitmask"].cpu().numpy()
    ext = np.minimum(w.block, w.N - w.block * np.arange(w.k))
    n_live = int(np.rint(float(np.float32(w.density)) * w.k * w.k))
    for h in range(w.nh):
        assert np.allclose(bsum[0, h].sum(axis=1), ext, rtol=REL)
        got = np.unpackbits(bits[h], bitorder="little")[: w.k * w.k].reshape(w.k, w.k).astype(bool)
        assert int(got.sum()) == n_live
        assert np.array_equal(got, pc.mask_from_block_sums(bsum[0, h].astype(np.float64), float(np.float32(w.density)), w.k))
    for h in (1, 6):
        idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, int(perm[h]))
        for i in (0, 137, w.k - 1):
            ref = pc.row_block_stats(q[0, h], k[0, h], idx, i, w.block, EPS)
            assert np.allclose(bsum[0, h, i], ref["sum"][0], rtol=REL, atol=1e-30), (h, i)
    # one head, one order, the whole map
    h, t = 3, 4
    g_sum, g_max, g_cnt, g_ms, g_mq = stats_on_gpu(w, q, k, t)
    idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, t)
    entries = pc.block_entries(w.N, w.block)
    lo = np.zeros((w.k, w.k), np.int64)
    hi = np.zeros_like(lo)
    r_sum = np.zeros((w.k, w.k))
    r_max = np.zeros((w.k, w.k))
    for i in range(w.k):
        st = pc.row_block_stats(q[0, h], k[0, h], idx, i, w.block, EPS, TIE)
        lo[i], hi[i], r_sum[i], r_max[i] = st["cnt_lo"][0], st["cnt_hi"][0], st["sum"][0], st["max"][0]
    assert np.all(g_cnt[0, h] >= lo) and np.all(g_cnt[0, h] <= hi)
    assert np.allclose(g_sum[0, h], r_sum, rtol=REL, atol=1e-30) and np.allclose(g_max[0, h], r_max, rtol=REL, atol=1e-30)
    assert pc.m_sparse(lo, entries, SIGMA) - 1e-7 <= g_ms[h] <= pc.m_sparse(hi, entries, SIGMA) + 1e-7
    assert g_mq[h] == pytest.approx(pc.m_quant(r_max, r_sum, entries), rel=2 * REL)
    print("head %d order %d: M_sparse %.4f M_quant %.2f" % (h, t, g_ms[h], g_mq[h]))
