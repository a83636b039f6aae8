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


# Rounding ties of the P codes.  A P code is an integer decision taken on floating-point values
# (E = Pt / sP): an implementation whose E carries a relative error may round an entry that lies
# within that error of a half-integer to the other neighbour, and one such flip moves an output
# element by sP * sv * |Vc| / l of its key - far more than the evaluation error itself.
# kernel_tie_tolerance() is the error of the HIP kernel's E, derived from its arithmetic, entry by entry.
LOG2E = 1.4426950408889634
LN2 = 0.6931471805599453
ACC_BIAS = 1.5 * 2.0**23  # start value of the kernel's integer accumulators, read as a float


def kernel_tie_tolerance(x_nat, m_new_nat, c_log2, folded):
    """Relative error bound of the kernel's E = qmaxP * 2^(c*S - m' - e) for one tile.
    x_nat [rows, cols], m_new_nat [rows]: logits and running maxima in natural-log units (as the
    oracle holds them); c_log2: the tile's logit scale in log2 units per integer step.

    The exponent is ONE fp32 fma of exact integers plus an offset: its rounding is half an ulp of
    the result, |y| * 2^-24 with |y| <= |x - m'| + 8 (log2 of qmaxP and e <= 0 shift the tile by a
    few octaves); the offset itself (m', e and constants, |m'| + 40 at most) comes from a handful of
    fp32 operations, 4 half-ulps; v_exp_f32 is good to about 1 ulp, 2^-23.  With the accumulator
    bias folded into the offset (8-bit P codes) the offset has the magnitude c * 1.5 * 2^23 and is
    rounded once more, half an ulp of that; its exact residue is applied to the block's weight, so
    it perturbs the codes only.  Errors of an exponent turn into relative errors of E times ln 2."""
    x2 = np.abs(x_nat - m_new_nat[:, None]) * LOG2E
    m2 = np.abs(m_new_nat)[:, None] * LOG2E
    err_exponent = 2.0**-24 * (x2 + 8.0) + 4 * 2.0**-24 * (m2 + 40.0)
    if folded:
        err_exponent = err_exponent + 2.0**-23 * (c_log2 * ACC_BIAS + m2 + 40.0)
    return LN2 * err_exponent + 2.0**-23


class TieRisk:
    """Observer of ``po.sparse_attention_head``: per output element, the first-order bound on what
    flipping every P code within the kernel's evaluation error of a rounding tie can change.  Every
    near-tie entry contributes sP * sv * |Vc| of its key; the contributions are carried through the
    same rescaling recurrence as the accumulator and divided by the same denominator.
    ``tol`` fixes one relative tolerance for all entries (used by the hand-worked test); otherwise
    the tolerance is kernel_tie_tolerance() of each tile (``sq``, ``sk``, ``d`` give its logit scale;
    ``folded`` [k] says for which row blocks the kernel folds the accumulator bias into the exponent)."""

    def __init__(self, vc, sv, block, n_valid, tol=None, sq=None, sk=None, d=None, folded=None, code_gain=1.0):
        self.absv = np.abs(np.asarray(vc, np.float64))
        self.sv = np.asarray(sv, np.float64)
        self.block, self.n_valid, self.tol = block, n_valid, tol
        self.sq, self.sk, self.d, self.folded = sq, sk, d, folded
        self.code_gain = code_gain  # factor by which the kernel's integer products exceed the plain code products
        self.out = np.zeros(self.absv.shape, np.float64)
        self._risk = None
        self._row = None

    def visit(self, i, j, x, m_new, p, codes, s_p, alpha):
        if self._row != i:
            self._row, self._risk = i, np.zeros((p.shape[0], self.absv.shape[1]))
        self._risk = alpha[:, None] * self._risk
        if s_p is None or s_p <= 0:
            return
        c0 = j * self.block
        e = p / s_p
        if self.tol is not None:
            tol = self.tol
        else:
            c_log2 = float(self.sq[i]) * float(self.sk[j]) * LOG2E / np.sqrt(self.d) / self.code_gain
            tol = kernel_tie_tolerance(x, m_new, c_log2, self.folded is not None and bool(self.folded[i]))
        near = np.abs(np.abs(e - np.rint(e)) - 0.5) <= tol * e + 1e-12
        self._risk += (near.astype(np.float64) @ self.absv[c0 : c0 + p.shape[1]]) * (s_p * self.sv[j])

    def row_block_done(self, i, l):
        if self._row != i:
            return
        r0 = i * self.block
        nz = l > 0
        self.out[r0 : r0 + l.shape[0]][nz] = self._risk[nz] / l[nz, None]
        self._row = None


def tie_risk_for(vc, sv, sq, sk, block, n_valid, d, bits_qk, bits_pv, row_ptr_h, col_idx):
    """The kernel folds the accumulator bias into the exponent only where P has 8-bit codes (with 4-bit
    codes one flipped code moves an element by up to a seventh of its largest term) and only for row
    blocks whose largest tile scale keeps the offset below 2^13; 4-bit Q and K codes enter its integer
    product times 16 each, so one integer step is 1/256 of a plain code step."""
    k = len(sq)
    gain = 256.0 if bits_qk == 4 else 1.0
    folded = np.zeros(k, bool)
    if bits_pv == 8:
        for i in range(k):
            cols = col_idx[int(row_ptr_h[i]) : int(row_ptr_h[i + 1])]
            if len(cols):
                c_max = float(sq[i]) * float(np.max(np.asarray(sk)[cols])) * LOG2E / np.sqrt(d) / gain
                folded[i] = c_max * ACC_BIAS < 8192.0
    return TieRisk(vc, sv, block, n_valid, sq=sq, sk=sk, d=d, folded=folded, code_gain=gain)


def oracle_head(w, q, k, v, perm_id, row_ptr_h, col_idx, row_blocks=None):
    """All intermediate results of the oracle for one head.  q, k, v: [N, d] float32."""
    idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, int(perm_id))
    out = {"idx": idx}
    qc, sq = po.prepare_operand(q, idx, w.npad, w.block, w.bits_qk)
    kc, sk = po.prepare_operand(k, idx, w.npad, w.block, w.bits_qk)
    vc, sv = po.prepare_operand(v, idx, w.npad, w.block, w.bits_pv)
    out.update(qc=qc, sq=sq, kc=kc, sk=sk, vc=vc, sv=sv)
    qmax_p = None if w.bits_pv in (0, 16) else po.qmax_of(w.bits_pv)
    risk = tie_risk_for(vc, sv, sq, sk, w.block, w.N, w.d, w.bits_qk, w.bits_pv, row_ptr_h, col_idx)
    op = po.sparse_attention_head(qc, sq, kc, sk, vc, sv, w.N, w.block, row_ptr_h, col_idx, qmax_p, row_blocks, observer=risk)
    out["op"] = op
    out["flip_risk"] = risk.out
    out["o"] = po.unpermute(op, idx)
    return out


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


# Share of the elements that may exceed the plain element-wise bar through a flipped near-tie P code
# (seen: none with 8-bit P codes, 4 of 1.1 million on a whole head with 4-bit P codes, where one flip moves
# an element by up to a seventh of its largest term).
MAX_TIE_EXCESS = 2e-5


def same_attention_kernel_for_raw_q(w) -> bool:
    """paro_sparse_attn_unpermuted_rawq runs on the kernel with one wavefront per 32 queries.  At d = 128, block 64
    with 8-bit codes throughout, the other entry points run the kernel with four wavefronts of 16 queries, whose
    floating-point sums associate differently: there the two agree to the rounding of the output, not bit for bit."""
    return not (w.d == 128 and w.block == 64 and w.bits_qk == 8 and w.bits_pv == 8)


def assert_equal_up_to_output_rounding(got, want, what=""):
    """Two evaluations of the same fp32 formula whose sums associate differently (torch tensors): equal up to one
    unit in the last place of the output type, plus 1e-6 of the largest magnitude for elements that cancel to near 0."""
    g, r = got.float(), want.float()
    bf16 = str(got.dtype).endswith("bfloat16")
    ulp = 2.0 ** -7 if bf16 else 2.0 ** -22
    tol = ulp * r.abs() + 1e-6 * float(r.abs().max())
    bad = int(((g - r).abs() > tol).sum())
    assert bad == 0, "%s: %d elements differ by more than the output rounding" % (what, bad)
    if bf16:  # fp32 differences of 1e-7 relative survive the rounding to bf16 only now and then
        assert float((g != r).float().mean()) < 0.05, "%s: more than 5 %% of the elements differ in the last place" % what


def check_attention(got, ref, risk, max_abs, rel, what=""):
    """The stated bar: relative L2 <= rel on everything, plainly; |got - ref| <= max_abs on every
    element that no near-tie P code can reach (risk == 0).  The remaining elements may exceed max_abs
    by at most their tie allowance, and those that do are counted, reported and bounded."""
    got, ref, risk = (np.asarray(a, np.float64) for a in (got, ref, risk))
    diff = np.abs(got - ref)
    ref_norm = max(float(np.linalg.norm(ref)), 1e-300)
    rel_err = float(np.linalg.norm(got - ref)) / ref_norm
    assert rel_err <= rel, "%s: relative L2 %.3e exceeds %.1e" % (what, rel_err, rel)
    safe = risk == 0
    worst_safe = float(diff[safe].max()) if safe.any() else 0.0
    assert worst_safe <= max_abs, "%s: max-abs %.3e exceeds %.1e where no P code is near a tie" % (what, worst_safe, max_abs)
    over = diff > max_abs
    n_over = int(over.sum())
    assert not (over & (diff - risk > max_abs)).any(), "%s: max-abs %.3e beyond the tie allowance" % (what, float((diff - risk).max()))
    assert n_over <= int(np.ceil(MAX_TIE_EXCESS * diff.size)), "%s: %d of %d elements beyond %.1e" % (what, n_over, diff.size, max_abs)
    st = {"max_abs": float(diff.max()), "rel_l2": rel_err, "n_over": n_over, "risky_share": float(np.mean(~safe))}
    print("%s: max_abs %.2e rel_l2 %.2e, %d elements over %.0e (tie allowance), %.2f%% of elements reachable by a tie"
          % (what or "attention", st["max_abs"], rel_err, n_over, max_abs, 100 * st["risky_share"]))
    return st


# ---------------------------------------------------------------------------------------------
# Whole heads of a full-size workload: the oracle over every row block, spread over worker
# processes.  The workers are started with the "spawn" method (fresh interpreters that import only
# numpy and the oracle), so they are safe to start from a process that has already initialised the GPU.
# ---------------------------------------------------------------------------------------------
def _oracle_rows_job(job):
    (dims, q, k, v, perm_id, row_ptr_h, col_idx, row_blocks) = job
    F, Hg, Wg, T_text, n, npad, block, bits_qk, bits_pv = dims
    idx = po.perm_index(F, Hg, Wg, T_text, int(perm_id))
    qc, sq = po.prepare_operand(q, idx, npad, block, bits_qk)
    kc, sk = po.prepare_operand(k, idx, npad, block, bits_qk)
    vc, sv = po.prepare_operand(v, idx, npad, block, bits_pv)
    qmax_p = None if bits_pv in (0, 16) else po.qmax_of(bits_pv)
    risk = tie_risk_for(vc, sv, sq, sk, block, n, q.shape[1], bits_qk, bits_pv, row_ptr_h, col_idx)
    op = po.sparse_attention_head(qc, sq, kc, sk, vc, sv, n, block, row_ptr_h, col_idx, qmax_p, row_blocks, observer=risk)
    rows = np.concatenate([np.arange(i * block, min((i + 1) * block, n)) for i in row_blocks])
    return rows, op[rows], risk.out[rows]


def oracle_whole_heads(w, heads, qkv_of_head, perm_ids, row_ptr, col_idx, workers=None):
    """{h: (op [npad, d], flip_risk [npad, d])} for every row block of the listed heads.
    ``qkv_of_head(h)`` returns the head's (q, k, v) as float32 [N, d] arrays; ``row_ptr`` is [nh, k+1]."""
    import multiprocessing as mp
    import os
    from concurrent.futures import ProcessPoolExecutor

    if workers is None:
        workers = max(1, min(16, len(os.sched_getaffinity(0))))
    dims = (w.F, w.Hg, w.Wg, w.T_text, w.N, w.npad, w.block, w.bits_qk, w.bits_pv)
    jobs, owner = [], []
    for h in heads:
        q, k, v = qkv_of_head(h)
        live = np.diff(row_ptr[h])
        # deal the row blocks to the workers heaviest first, so the chunks carry equal work
        order = np.argsort(-live, kind="stable")
        per = max(1, workers // max(1, len(heads))) if len(heads) < workers else 1
        chunks = [sorted(int(i) for i in order[c::per]) for c in range(per)]
        for rows in chunks:
            if rows:
                jobs.append((dims, q, k, v, int(perm_ids[h]), row_ptr[h], col_idx, rows))
                owner.append(h)
    out = {h: (np.zeros((w.npad, w.d)), np.zeros((w.npad, w.d))) for h in heads}
    with ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn")) as ex:
        for h, (rows, op_rows, risk_rows) in zip(owner, ex.map(_oracle_rows_job, jobs)):
            out[h][0][rows] = op_rows
            out[h][1][rows] = risk_rows
    return out
