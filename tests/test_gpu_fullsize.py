"""GPU parity at the full benchmark shapes, in the launch configuration bench.py times.

The whole workload runs on the GPU through the C ABI; the oracle recomputes sampled heads
(codes and scales of the whole head, bit for bit) and sampled row blocks of those heads
(attention output rows), including the first, the heaviest, the lightest and the ragged last row
block.  Properties that hold at any size are checked on the full tensors: the reorder round trip
is the identity, padded rows are zero, nothing is NaN."""
import numpy as np
import pytest

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl
from tests.helpers import KERNEL_TIE_TOL, check_attention
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
    o = pa.run(q, k, v)
    torch.cuda.synchronize()
    return pa, perm_ids, masks, (q, k, v), o


def check_sampled(w, heads):
    import torch

    pa, perm_ids, masks, (q, k, v), o = run_full(w)
    assert pa.live_blocks == int(masks.sum()) * w.B
    # --- properties on the full tensors
    assert not torch.isnan(pa.op).any() and not torch.isnan(o).any()
    assert bool((pa.op[:, :, w.N:] == 0).all())
    from paper_2506_16054_amd import binding as pb

    back = torch.empty_like(q)
    pb.paro_unpermute(pa.s, perm_ids, pa.xp[0], back)
    torch.cuda.synchronize()
    assert torch.equal(back, q)  # reorder followed by its inverse is the identity, bit for bit
    # --- sampled heads against the oracle
    rel = REL_L2_BF16 if w.bits_qk == 16 else REL_L2
    for h in heads:
        hq, hk, hv = (host(t[0, h]) for t in (q, k, v))
        idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, int(perm_ids[h]))
        assert np.array_equal(pb.paro_perm_index(pa.s, int(perm_ids[h])), idx)
        qc, sq = po.prepare_operand(hq, idx, w.npad, w.block, w.bits_qk)
        kc, sk = po.prepare_operand(hk, idx, w.npad, w.block, w.bits_qk)
        vc, sv = po.prepare_operand(hv, idx, w.npad, w.block, w.bits_pv)
        if w.bits_qk != 16:
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
        row_ptr = pa.h_row_ptr[h]
        live = np.diff(row_ptr)
        rows = sorted({0, w.k - 1, int(np.argmax(live)), int(np.argmin(live)), w.k // 3})
        diag = {}
        qmax_p = None if w.bits_pv in (0, 16) else po.qmax_of(w.bits_pv)
        ref = po.sparse_attention_head(qc, sq, kc, sk, vc, sv, w.N, w.block, row_ptr, pa.h_col_idx, qmax_p, rows,
                                       tie_tol=KERNEL_TIE_TOL, diag=diag)
        got = host(pa.op[0, h])
        for i in rows:
            sl = slice(i * w.block, min((i + 1) * w.block, w.N))
            st = check_attention(got[sl], ref[sl], diag["flip_risk"][sl], MAX_ABS, rel, "%s h%d row block %d" % (w.name, h, i))
            print("%s h%d row block %d (%d live): max_abs %.2e rel_l2 %.2e" % (w.name, h, i, live[i], st["max_abs"], st["rel_l2"]))
        # and the inverse reorder of those rows
        g_o = host(o[0, h])
        for i in rows:
            for n_new in range(i * w.block, min((i + 1) * w.block, w.N)):
                assert np.array_equal(g_o[idx[n_new]], got[n_new])


def test_headline_cogvideox5b_int8():
    check_sampled(wl.WORKLOADS["cogvideox5b"], heads=(0, 17, 47))


def test_cogvideox5b_int4_pv():
    check_sampled(wl.WORKLOADS["cogvideox5b_int4pv"], heads=(5, 30))


def test_cogvideox2b_density_half():
    check_sampled(wl.WORKLOADS["cogvideox2b"], heads=(3, 29))


def test_flux_text_blocks_d128():
    check_sampled(wl.WORKLOADS["flux"], heads=(0, 11, 23))


def test_headline_shape_bf16_mode():
    check_sampled(wl.WORKLOADS["cogvideox5b"].replace(name="cogvideox5b_bf16", bits_qk=16, bits_pv=16, nh=8), heads=(2, 7))


def test_headline_shape_all_int4():
    check_sampled(wl.WORKLOADS["cogvideox5b"].replace(name="cogvideox5b_i4i4", bits_qk=4, bits_pv=4, density=0.5, nh=8), heads=(1, 6))
