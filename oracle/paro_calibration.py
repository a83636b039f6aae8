"""CPU oracle for the offline calibration of PAROAttention (arXiv 2506.16054, Sec. 4.1 "Metric
for Permutation Order" and Sec. 4.2 (3) "Efficient Offline Mask Generation").

TEST INFRASTRUCTURE ONLY: plain float64 NumPy, imported by ``tests/`` alone; it shares no code
with the HIP library and never calls it.

What is computed, per head, from one calibration sample of Q and K:

    P = softmax(Q K^T / sqrt(d))                         the post-softmax attention map
    for each of the six axis orders Theta:
        P^Theta = P with rows and columns reordered       (Sec. 4.1; text tokens keep their place)
        tile P^Theta into k x k blocks of b x b
        n_ij    = #{ |P_ij(m,n)| < eps }                  Eq. (M_sparse)
        M_sparse = fraction of blocks with n_ij / (b b) >= sigma
        Psi_ij  = max |P_ij| / mean |P_ij|                Eq. (M_quant)
        M_quant = mean over blocks of Psi_ij
    M^Theta = alpha * S^Theta / sum_Theta S + (1 - alpha) * M_quant^Theta / sum_Theta M_quant
    the order with the lowest M^Theta is chosen
    mask: block sums of P^Theta (chosen order), thresholded so that a requested density of blocks
    stays live                                             Sec. 4.2 (3)

Readings taken where the paper is silent or at odds with itself:
  * The text defines M_sparse as the share of SPARSE blocks (more is better) and then picks the
    order with the LOWEST combined metric.  To make "lowest" right for both terms the combined
    metric uses S^Theta = 1 - M_sparse^Theta, the share of blocks that are not sparse;
    M_sparse itself is reported as the equation defines it.
  * N need not be a multiple of b: entries of padded rows and columns do not exist; a ragged
    block's count is compared with sigma times its number of real entries and its mean runs
    over its real entries.
  * The comparison n >= sigma * (entries) is evaluated in IEEE binary32 (an integer decision
    taken on floating-point values: both sides use the kernel's precision).
  * Psi of an all-zero block (possible only through underflow) is 0; a term of the combined
    metric whose normaliser is 0 is 0; equal M^Theta: the lowest order id wins.
  * Q and K enter in the 16-bit precision the model's own attention runs in: they are rounded to
    bfloat16 (round to nearest even) before the map is formed.
  * Density control: the n_live = rint(density * k_img^2) image x image blocks with the largest
    block sums stay live (equal sums: lower i*k + j first); rows and columns of text blocks are
    always live (Sec. 4.2 (1): only image tokens are sparsified); nothing else is forced.  With
    several calibration samples the block sums are added over the samples first.
"""
from __future__ import annotations

import math

import numpy as np


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 (ties to even) of float32 values, returned as float64."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)) << np.uint32(16)
    return r.astype(np.uint32).view(np.float32).astype(np.float64)


def attention_rows(q: np.ndarray, k: np.ndarray, rows: np.ndarray) -> np.ndarray:
    """Rows ``rows`` of P = softmax(Q K^T / sqrt(d)) in float64; q, k: [N, d] (default token order)."""
    qb, kb = round_to_bf16(q), round_to_bf16(k)
    x = (qb[rows] @ kb.T) / math.sqrt(q.shape[1])
    x -= x.max(axis=1, keepdims=True)
    e = np.exp(x)
    return e / e.sum(axis=1, keepdims=True)


def attention_map(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    return attention_rows(q, k, np.arange(q.shape[0]))


def reorder_map(p: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """P^Theta[n', m'] = P[idx[n'], idx[m']]: the map of the reordered sequence."""
    return p[np.ix_(idx, idx)]


def block_entries(n: int, block: int) -> np.ndarray:
    """[k, k] number of real entries of every block of an n x n map tiled by ``block``."""
    kb = -(-n // block)
    ext = np.minimum(block, n - block * np.arange(kb))
    return np.outer(ext, ext).astype(np.int64)


def block_stats(p: np.ndarray, block: int, eps: float, tol: float = 0.0):
    """Per-block statistics of a map p [n, m] whose rows start at a block boundary:
    sums, maxima, counts of |p| < eps.  With ``tol`` > 0 also the counts at eps*(1-tol) and
    eps*(1+tol), which bracket the count of any evaluation of p with relative error <= tol."""
    n, m = p.shape
    kr, kc = -(-n // block), -(-m // block)
    sums = np.zeros((kr, kc))
    maxs = np.zeros((kr, kc))
    cnt = np.zeros((kr, kc), np.int64)
    lo = np.zeros((kr, kc), np.int64)
    hi = np.zeros((kr, kc), np.int64)
    a = np.abs(p)
    for i in range(kr):
        for j in range(kc):
            t = a[i * block:(i + 1) * block, j * block:(j + 1) * block]
            sums[i, j] = t.sum()
            maxs[i, j] = t.max()
            cnt[i, j] = int((t < eps).sum())
            lo[i, j] = int((t < eps * (1.0 - tol)).sum())
            hi[i, j] = int((t < eps * (1.0 + tol)).sum())
    out = {"sum": sums, "max": maxs, "cnt": cnt}
    if tol > 0:
        out["cnt_lo"], out["cnt_hi"] = lo, hi
    return out


def row_block_stats(q: np.ndarray, k: np.ndarray, idx: np.ndarray, i: int, block: int, eps: float, tol: float = 0.0):
    """block_stats of row block ``i`` of the reordered map (all column blocks), without forming
    the other rows: for sequences whose full map does not fit in memory."""
    rows = idx[i * block:(i + 1) * block]
    return block_stats(attention_rows(q, k, rows)[:, idx], block, eps, tol)


def sparse_blocks(cnt: np.ndarray, entries: np.ndarray, sigma: float) -> np.ndarray:
    """Indicator of Eq. (M_sparse): n_ij / entries >= sigma, compared in binary32."""
    return cnt.astype(np.float32) >= np.float32(sigma) * entries.astype(np.float32)


def m_sparse(cnt: np.ndarray, entries: np.ndarray, sigma: float) -> float:
    return float(np.mean(sparse_blocks(cnt, entries, sigma)))


def psi_blocks(maxs: np.ndarray, sums: np.ndarray, entries: np.ndarray) -> np.ndarray:
    """Incoherence of every block, Eq. (M_quant): max |x| over mean |x|."""
    mean = sums / entries
    return np.where(sums > 0, maxs / np.where(mean > 0, mean, 1.0), 0.0)


def m_quant(maxs: np.ndarray, sums: np.ndarray, entries: np.ndarray) -> float:
    return float(np.mean(psi_blocks(maxs, sums, entries)))


def combine(ms, mq, alpha: float):
    """Combined metric of the six orders and the chosen order id (lowest metric, lowest id on ties)."""
    ms = np.asarray(ms, np.float64)
    mq = np.asarray(mq, np.float64)
    dense = 1.0 - ms
    t1 = dense / dense.sum() if dense.sum() > 0 else np.zeros_like(dense)
    t2 = mq / mq.sum() if mq.sum() > 0 else np.zeros_like(mq)
    m = alpha * t1 + (1.0 - alpha) * t2
    return m, int(np.argmin(m))


def mask_from_block_sums(sums: np.ndarray, density: float, k_img: int) -> np.ndarray:
    """bool [k, k]: the rint(density * k_img^2) image x image blocks with the largest sums are
    live (equal sums: lower flat index first); text rows and columns are live."""
    k = sums.shape[0]
    n_live = int(np.rint(density * k_img * k_img))
    n_live = min(max(n_live, 0), k_img * k_img)
    mask = np.zeros((k, k), bool)
    ii, jj = np.meshgrid(np.arange(k_img), np.arange(k_img), indexing="ij")
    flat = (ii * k + jj).ravel()
    order = np.lexsort((flat, -sums[:k_img, :k_img].ravel()))  # by sum descending, then flat index ascending
    chosen = flat[order[:n_live]]
    mask.ravel()[chosen] = True
    mask[k_img:, :] = True
    mask[:, k_img:] = True
    return mask


def calibrate_head(q: np.ndarray, k: np.ndarray, gather_indices, block: int, eps: float, sigma: float, alpha: float,
                   density: float, k_img: int, tol: float = 0.0):
    """Everything for one head from one sample: per-order statistics and metrics, the chosen order,
    its block sums and mask.  ``gather_indices[t]`` is the gather index of order t (six of them)."""
    p = attention_map(q, k)
    n = p.shape[0]
    entries = block_entries(n, block)
    per_order = []
    for idx in gather_indices:
        st = block_stats(reorder_map(p, idx), block, eps, tol)
        st["m_sparse"] = m_sparse(st["cnt"], entries, sigma)
        st["m_quant"] = m_quant(st["max"], st["sum"], entries)
        per_order.append(st)
    m, best = combine([s["m_sparse"] for s in per_order], [s["m_quant"] for s in per_order], alpha)
    mask = mask_from_block_sums(per_order[best]["sum"], density, k_img)
    return {"orders": per_order, "M": m, "perm_id": best, "mask": mask, "entries": entries}
