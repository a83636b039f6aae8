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


# Relative error bound of the HIP kernel's evaluation of Pt / sP (fp32 fma of the logit, the
# hardware exp2 and fp32 running maxima); P codes whose exact value lies this close to a
# rounding tie may legitimately come out as either neighbour.
KERNEL_TIE_TOL = 2e-5


def oracle_head(w, q, k, v, perm_id, row_ptr_h, col_idx, row_blocks=None):
    """All intermediate results of the oracle for one head.  q, k, v: [N, d] float32."""
    idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, int(perm_id))
    out = {"idx": idx}
    qc, sq = po.prepare_operand(q, idx, w.npad, w.block, w.bits_qk)
    kc, sk = po.prepare_operand(k, idx, w.npad, w.block, w.bits_qk)
    vc, sv = po.prepare_operand(v, idx, w.npad, w.block, w.bits_pv)
    out.update(qc=qc, sq=sq, kc=kc, sk=sk, vc=vc, sv=sv)
    qmax_p = None if w.bits_pv in (0, 16) else po.qmax_of(w.bits_pv)
    diag = {}
    op = po.sparse_attention_head(qc, sq, kc, sk, vc, sv, w.N, w.block, row_ptr_h, col_idx, qmax_p, row_blocks,
                                  tie_tol=KERNEL_TIE_TOL, diag=diag)
    out["op"] = op
    out["flip_risk"] = diag["flip_risk"]
    out["o"] = po.unpermute(op, idx)
    return out


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def check_attention(got, ref, risk, max_abs, rel, what=""):
    """Element-wise and relative-L2 bar, widened only by what flips of near-tie P codes can cause."""
    got, ref, risk = (np.asarray(a, np.float64) for a in (got, ref, risk))
    diff = np.abs(got - ref)
    worst = float(np.max(diff - risk))
    assert worst <= max_abs, "%s: max-abs %.3e beyond tie allowance exceeds %.1e" % (what, worst, max_abs)
    lhs = float(np.linalg.norm(got - ref))
    rhs = rel * float(np.linalg.norm(ref)) + float(np.linalg.norm(risk))
    assert lhs <= rhs, "%s: L2 error %.3e exceeds %.3e" % (what, lhs, rhs)
    risky_rows = float(np.mean(risk.max(axis=-1) > 0))
    return {"max_abs": float(diff.max()), "rel_l2": lhs / max(float(np.linalg.norm(ref)), 1e-300), "risky_rows": risky_rows}
