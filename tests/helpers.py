"""Shared test helpers: run the CPU oracle over a synthetic workload (or a few heads of it)."""
import numpy as np

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl


def gather_fn(w):
    return lambda pid: po.perm_index(w.F, w.Hg, w.Wg, w.T_text, pid)


def blocklist_for(w, masks):
    bits = wl.pack_bitmask(masks)
    row_ptr, col_idx = po.mask_to_blocklist(bits, w.nh, w.k)
    return bits, row_ptr, col_idx


def oracle_head(w, q, k, v, perm_id, row_ptr_h, col_idx, row_blocks=None):
    """All intermediate results of the oracle for one head.  q, k, v: [N, d] float32."""
    idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, int(perm_id))
    out = {"idx": idx}
    qc, sq = po.prepare_operand(q, idx, w.npad, w.block, w.bits_qk)
    kc, sk = po.prepare_operand(k, idx, w.npad, w.block, w.bits_qk)
    vc, sv = po.prepare_operand(v, idx, w.npad, w.block, w.bits_pv)
    out.update(qc=qc, sq=sq, kc=kc, sk=sk, vc=vc, sv=sv)
    qmax_p = None if w.bits_pv == 16 else po.qmax_of(w.bits_pv)
    op = po.sparse_attention_head(qc, sq, kc, sk, vc, sv, w.N, w.block, row_ptr_h, col_idx, qmax_p, row_blocks)
    out["op"] = op
    out["o"] = po.unpermute(op, idx)
    return out


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))
