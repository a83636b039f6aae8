"""CPU oracle for the PAROAttention hot path (arXiv 2506.16054).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, float64 statement of what the path
computes.  It is imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py`` and by nothing else; it shares no code with the HIP
library and never calls it.

The path (Sec. 4 of the paper; Fig. 3):

    reorder tokens of each head into one of the six orders of (F, H, W)      (Sec. 4.1)
 -> quantize Q, K, V with one symmetric scale per block of ``b`` tokens       (Sec. 4.3 (1))
 -> FlashAttention-style loop over the live blocks of a static per-head
    block mask (Sec. 4.2 (2)), with the running P tile quantized as one
    b x b group before the PV product                                         (Sec. 4.3 (1),(2))
 -> put the output rows back into the default token order                     (Sec. 4.1)

Sparsity and quantization change the answer, and because P is quantized tile by tile while
the running row maximum evolves, the answer depends on the visiting order.  The oracle is
therefore the algorithm, step by step; the textbook softmax(QK^T/sqrt(d))V is only its limit
(density 1, quantization off) and is used as a pin in the tests, not here.

Readings taken where the paper is silent (each is listed in the design notes of the build):
  * order numbering: lexicographic over the letters "FHW" (0 FHW ... 5 WHF), slowest axis
    first; the same order is used for Q, K and V of a head; text tokens keep their place;
  * N need not be a multiple of b: the last block is padded, padded keys never receive
    probability mass, padded query rows are ignored;
  * Q, K, V group = b tokens x d channels of one head; scale = absmax / qmax; round half to
    even; the code step is evaluated in IEEE binary32 so an fp32 device kernel can match it
    bit for bit;
  * 1/sqrt(d) is applied in floating point after the integer product;
  * P group = the b x b tile of exp(X - m) with m the running row maximum *at visit time*;
    scale = tile max / qmax_P; live blocks are visited in ascending column-block order;
  * the softmax denominator accumulates the unquantized tile.

Pins (see tests/test_oracle_*.py): numpy reshape/transpose for the index; brute-force dense
and masked softmax; permutation equivariance; closed forms for constant-logit tiles and for
b = 1; the scale/2 quantizer bound; 1/qmax convergence.  No value printed by the paper pins
the *quantized* attention output (the paper prints none): for that function the status is
"parity unpinned by any published number"; it is pinned by the closed forms and limits above.
"""
from __future__ import annotations

import itertools
import math
from typing import Optional, Sequence, Tuple

import numpy as np

AXES = "FHW"
# Sec. 4.1: the search space is the 3! = 6 orderings of the axes [F, H, W]; numbering is this build's reading.
AXIS_ORDERS: Tuple[Tuple[int, int, int], ...] = tuple(itertools.permutations(range(3)))


def order_name(perm_id: int) -> str:
    return "".join(AXES[a] for a in AXIS_ORDERS[perm_id])


# ---------------------------------------------------------------------------------------------
# O1 / O5: token reorder  (Sec. 1, Fig. 2(c); Sec. 4.1)
# ---------------------------------------------------------------------------------------------
def perm_index(F: int, Hg: int, Wg: int, T_text: int, perm_id: int) -> np.ndarray:
    """Gather index ``idx`` with Xp[n'] = X[idx[n']].

    The default sequence order is [F, H, W]: token (f, h, w) sits at n = (f*Hg + h)*Wg + w, so
    neighbours along F are Hg*Wg apart (Sec. 1).  In order (a0, a1, a2), slowest first, the same
    token sits at n' = (c[a0]*D[a1] + c[a1])*D[a2] + c[a2].  Text tokens, appended after the
    image tokens, are not reordered (Sec. 4.2 (1)).
    """
    if not 0 <= perm_id < 6:
        raise ValueError("perm_id must be in 0..5")
    dims = (F, Hg, Wg)
    a0, a1, a2 = AXIS_ORDERS[perm_id]
    n_img = F * Hg * Wg
    idx = np.empty(n_img + T_text, np.int64)
    for f in range(F):
        for h in range(Hg):
            for w in range(Wg):
                c = (f, h, w)
                n = (f * Hg + h) * Wg + w
                n_new = (c[a0] * dims[a1] + c[a1]) * dims[a2] + c[a2]
                idx[n_new] = n
    for t in range(T_text):
        idx[n_img + t] = n_img + t
    return idx


def permute(x: np.ndarray, idx: np.ndarray, npad: int) -> np.ndarray:
    """x [N, d] -> xp [npad, d]: reordered rows, zero rows after N."""
    xp = np.zeros((npad, x.shape[1]), x.dtype)
    for n_new in range(idx.shape[0]):
        xp[n_new] = x[idx[n_new]]
    return xp


def unpermute(op: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """op [npad, d] -> o [N, d] with o[idx[n']] = op[n']."""
    o = np.empty((idx.shape[0], op.shape[1]), op.dtype)
    for n_new in range(idx.shape[0]):
        o[idx[n_new]] = op[n_new]
    return o


# ---------------------------------------------------------------------------------------------
# O2: block-aligned symmetric quantizer  (Sec. 4.3 (1))
# ---------------------------------------------------------------------------------------------
def qmax_of(bits: int) -> int:
    if bits == 8:
        return 127
    if bits == 4:
        return 7
    raise ValueError("bits must be 8 or 4")


def quantize_blocks(xp: np.ndarray, n_valid: int, block: int, qmax: int):
    """One scale per block of ``block`` tokens x d channels.

    Returns (codes int32 [npad, d], scales float32 [k]).  absmax is taken over valid rows;
    scale = absmax / qmax in binary32 (1.0 for an all-zero block); code = rint(x / scale) in
    binary32, clamped to [-qmax, qmax]; rows >= n_valid get code 0.
    """
    npad, _ = xp.shape
    k = npad // block
    x32 = xp.astype(np.float32)
    codes = np.zeros(xp.shape, np.int32)
    scales = np.ones(k, np.float32)
    for blk in range(k):
        lo = blk * block
        hi = min(lo + block, n_valid)
        if hi <= lo:
            continue
        tile = x32[lo:hi]
        absmax = np.float32(np.max(np.abs(tile)))
        if absmax > 0:
            scales[blk] = absmax / np.float32(qmax)
        r = np.rint(tile / scales[blk])  # float32 / float32: correctly rounded binary32
        codes[lo:hi] = np.clip(r, -qmax, qmax).astype(np.int32)
    return codes, scales


def dequantize_blocks(codes: np.ndarray, scales: np.ndarray, block: int) -> np.ndarray:
    return codes.astype(np.float64) * np.repeat(scales.astype(np.float64), block)[:, None]


def quantize_p_tile(p: np.ndarray, valid: np.ndarray, qmax_p: int):
    """P tile as one group (Sec. 4.3 (1)): scale = max over valid entries / qmax_p, round half
    to even.  Returns (codes float64 of integers, scale).  An all-zero tile gives codes 0."""
    pmax = float(np.max(np.where(valid, p, 0.0))) if valid.any() else 0.0
    if pmax <= 0.0:
        return np.zeros_like(p), 0.0
    s_p = pmax / qmax_p
    codes = np.where(valid, np.rint(p / s_p), 0.0)
    return codes, s_p


# ---------------------------------------------------------------------------------------------
# O3: bitmask -> compacted block list  (Sec. 4.2 (1),(2))
# ---------------------------------------------------------------------------------------------
def mask_nbytes(k: int) -> int:
    """Bytes of one head's bitmask: one bit per b x b block."""
    return (k * k + 7) // 8


def mask_to_blocklist(bitmask: np.ndarray, nh: int, k: int):
    """bitmask uint8 [nh, ceil(k*k/8)], bit (i*k + j), LSB-first -> (row_ptr [nh, k+1], col_idx).

    ``row_ptr`` holds offsets into one ``col_idx`` array shared by all heads; the columns of a
    row are ascending.
    """
    row_ptr = np.zeros((nh, k + 1), np.int32)
    cols = []
    for h in range(nh):
        for i in range(k):
            row_ptr[h, i] = len(cols)
            for j in range(k):
                bit = i * k + j
                if (int(bitmask[h, bit >> 3]) >> (bit & 7)) & 1:
                    cols.append(j)
        row_ptr[h, k] = len(cols)
    return row_ptr, np.asarray(cols, np.int32)


# ---------------------------------------------------------------------------------------------
# O4: block-sparse attention with block-wise quantized QK^T and PV  (Sec. 4.2 (2), 4.3)
# ---------------------------------------------------------------------------------------------
def sparse_attention_head(
    qc: np.ndarray,
    sq: np.ndarray,
    kc: np.ndarray,
    sk: np.ndarray,
    vc: np.ndarray,
    sv: np.ndarray,
    n_valid: int,
    block: int,
    row_ptr: np.ndarray,
    col_idx: np.ndarray,
    qmax_p: Optional[int],
    row_blocks: Optional[Sequence[int]] = None,
    observer=None,
) -> np.ndarray:
    """One head.  qc/kc/vc [npad, d] hold integer codes (or plain values with scales of 1 for an
    unquantized operand); sq/sk/sv [k] are the per-block scales.  ``qmax_p`` None leaves P
    unquantized.  Returns Op float64 [npad, d]; rows of padded tokens and of row blocks that are
    not listed in ``row_blocks`` stay zero.  A row block with no live block gives zeros.

    The live blocks of a row are visited in the order in which the list holds them (ascending
    column block for a list made by ``mask_to_blocklist``); with P quantized per visit against the
    running row maxima the result depends on that order (Sec. 4.3 (1),(2)).

    ``observer``, if given, is shown the intermediate quantities and changes nothing:
    ``observer.visit(i, j, x, m_new, p, codes, s_p, alpha)`` after every visited block (logits, new
    row maxima, P tile, its integer codes and scale - None when P is not quantized - and the rescale
    factor of the earlier sums) and ``observer.row_block_done(i, l)`` with the final denominators of
    row block i.
    """
    npad, d = qc.shape
    k = npad // block
    qf = qc.astype(np.float64)
    kf = kc.astype(np.float64)
    vf = vc.astype(np.float64)
    inv_sqrt_d = 1.0 / math.sqrt(d)
    out = np.zeros((npad, d), np.float64)
    todo = range(k) if row_blocks is None else row_blocks
    for i in todo:
        r0 = i * block
        n_rows = min(block, n_valid - r0)
        if n_rows <= 0:
            continue
        m = np.full(n_rows, -np.inf)
        l = np.zeros(n_rows)
        acc = np.zeros((n_rows, d))
        q_i = qf[r0 : r0 + n_rows]
        for t in range(int(row_ptr[i]), int(row_ptr[i + 1])):
            j = int(col_idx[t])
            c0 = j * block
            n_cols = min(block, n_valid - c0)
            if n_cols <= 0:
                continue
            s_int = q_i @ kf[c0 : c0 + n_cols].T  # exact: integers well below 2^53
            x = s_int * (float(sq[i]) * float(sk[j]) * inv_sqrt_d)
            m_new = np.maximum(m, x.max(axis=1))
            alpha = np.exp(m - m_new)  # exp(-inf) = 0 on the first visit
            p = np.exp(x - m_new[:, None])
            l = alpha * l + p.sum(axis=1)
            if qmax_p is None:
                codes, s_p = None, None
                pv = p @ (vf[c0 : c0 + n_cols] * float(sv[j]))
            else:
                codes, s_p = quantize_p_tile(p, np.ones_like(p, bool), qmax_p)
                pv = (codes @ vf[c0 : c0 + n_cols]) * (s_p * float(sv[j]))
            acc = alpha[:, None] * acc + pv
            m = m_new
            if observer is not None:
                observer.visit(i, j, x, m_new, p, codes, s_p, alpha)
        nz = l > 0
        out[r0 : r0 + n_rows][nz] = acc[nz] / l[nz, None]
        if observer is not None:
            observer.row_block_done(i, l)
    return out


# ---------------------------------------------------------------------------------------------
# Whole path for one head, and for a problem
# ---------------------------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 (8 significand bits), ties to even, of float32 values; returned as float64."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(np.float64)


def k_channel_mean(k: np.ndarray) -> np.ndarray:
    """Optional pre-conditioning of K (not part of the paper's method; 8-bit attention kernels of the family its
    kernel derives from have it): the constant removed from channel c of every key of a head is the mean of
    k[:, c] over the N tokens, taken in float64 and rounded to bfloat16.  Returned as float32 [d]."""
    mean64 = np.asarray(k, dtype=np.float64).mean(axis=0)
    return round_to_bf16(mean64.astype(np.float32)).astype(np.float32)


def smooth_k(k: np.ndarray) -> np.ndarray:
    """k - k_channel_mean(k), one binary32 subtraction per element (the quantizer that follows evaluates in
    binary32 too).  A constant per channel shifts every logit of a query by the same amount, q . mean, which the
    softmax over any set of keys does not see; only the quantization error of K changes."""
    return (np.asarray(k, dtype=np.float32) - k_channel_mean(k)[None, :]).astype(np.float32)


def prepare_operand(x: np.ndarray, idx: np.ndarray, npad: int, block: int, bits: int):
    """permute + quantize one of Q/K/V of one head.
    bits 8 / 4: integer codes and per-block scales; bits 16: the unquantized mode, operands held
    in bfloat16 (scales of 1); bits 0: no rounding at all (exact reference arithmetic)."""
    xp = permute(x, idx, npad)
    if bits == 0:
        return xp.astype(np.float64), np.ones(npad // block, np.float32)
    if bits == 16:
        return round_to_bf16(xp), np.ones(npad // block, np.float32)
    return quantize_blocks(xp, idx.shape[0], block, qmax_of(bits))


def paro_attention_head(
    q: np.ndarray,
    k: np.ndarray,
    v: np.ndarray,
    grid: Tuple[int, int, int],
    T_text: int,
    perm_id: int,
    block: int,
    row_ptr: np.ndarray,
    col_idx: np.ndarray,
    bits_qk: int,
    bits_pv: int,
    smooth: bool = False,
) -> np.ndarray:
    """permute -> quantize -> block-sparse attention -> inverse permute for one head.
    q, k, v: [N, d] in the default token order.  smooth: K is replaced by smooth_k(K) first.
    Returns O float64 [N, d]."""
    F, Hg, Wg = grid
    if smooth:
        k = smooth_k(k)
    n = q.shape[0]
    kblocks = -(-n // block)
    npad = kblocks * block
    idx = perm_index(F, Hg, Wg, T_text, perm_id)
    qc, sq = prepare_operand(q, idx, npad, block, bits_qk)
    kc, sk = prepare_operand(k, idx, npad, block, bits_qk)
    vc, sv = prepare_operand(v, idx, npad, block, bits_pv)
    qmax_p = None if bits_pv in (0, 16) else qmax_of(bits_pv)
    op = sparse_attention_head(qc, sq, kc, sk, vc, sv, n, block, row_ptr, col_idx, qmax_p)
    return unpermute(op, idx)


def cast_output(o: np.ndarray, dtype: str) -> np.ndarray:
    """Round the float64 result to the storage type of the output (fp32, or bf16 round half to
    even), returned as float64 for comparison."""
    o32 = o.astype(np.float32)
    if dtype == "f32":
        return o32.astype(np.float64)
    if dtype == "bf16":
        return round_to_bf16(o32)
    raise ValueError(dtype)


def incoherence(x: np.ndarray) -> float:
    """Psi of Eq. 2: max |x| over mean |x| of a quantization group (diagnostic only)."""
    a = np.abs(x)
    mean = float(a.mean())
    return float(a.max()) / mean if mean > 0 else float("inf")
