"""Seeded synthetic workloads shaped like the attention layers the paper evaluates on.

This module only *generates inputs* (Q/K/V tensors, per-head permutation ids, per-head block
masks).  It contains none of the method's arithmetic: no permutation-index formula, no
quantizer, no softmax.  Where a generator needs a head's token order (the block mask is
defined on the permuted sequence, Sec. 4.2), the caller passes the gather index in.

Both the CPU oracle's tests and the GPU path's tests/bench draw their inputs from here so the
two sides see bit-identical arrays.

Stand-in statement: the paper measures CogVideoX (N = 17550 = 13*30*45 latent tokens,
Sec. 1 footnote) and Flux (1024 px, Sec. 5.1) attention layers taken from real sampling runs.
Neither the models nor the prompt sets are available here; these generators only reproduce the
*shapes*, the local-aggregation structure (Sec. 1: attention concentrates on 3-D neighbours)
and the density of the calibrated masks.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Callable, Dict, Optional, Sequence

import numpy as np

AXIS_ORDER_NAMES = ("FHW", "FWH", "HFW", "HWF", "WFH", "WHF")


@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic attention-layer problem."""

    name: str
    B: int
    nh: int
    d: int
    F: int
    Hg: int
    Wg: int
    T_text: int
    block: int
    density: float
    bits_qk: int
    bits_pv: int
    dtype: str  # "f32" or "bf16": storage type of Q, K, V and of the output
    seed: int
    perm_choice: Optional[Sequence[int]] = None  # fixed per-head ids (cycled); None = uniform draw
    sigma: float = 2.0  # RBF width of the local positional component, in grid cells

    @property
    def n_img(self) -> int:
        return self.F * self.Hg * self.Wg

    @property
    def N(self) -> int:
        return self.n_img + self.T_text

    @property
    def k(self) -> int:
        return -(-self.N // self.block)

    @property
    def npad(self) -> int:
        return self.k * self.block

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five configurations the benchmark definition names (index 0 is the small case the oracle
# finishes in well under a second; index 2 is the headline workload).
WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 1, 2, 64, 2, 8, 8, 0, 32, 0.5, 8, 8, "f32", 1001, perm_choice=(0, 5)),
    "cogvideox2b": Workload("cogvideox2b", 1, 30, 64, 13, 30, 45, 0, 64, 0.5, 8, 8, "bf16", 2002),
    "cogvideox5b": Workload("cogvideox5b", 1, 48, 64, 13, 30, 45, 0, 64, 0.3, 8, 8, "bf16", 3003),
    "cogvideox5b_int4pv": Workload("cogvideox5b_int4pv", 1, 48, 64, 13, 30, 45, 0, 64, 0.2, 8, 4, "bf16", 4004),
    "flux": Workload("flux", 1, 24, 128, 1, 64, 64, 512, 64, 0.3, 8, 8, "bf16", 5005),
}
WORKLOAD_ORDER = ("tiny", "cogvideox2b", "cogvideox5b", "cogvideox5b_int4pv", "flux")
# The unquantized 16-bit sparse mode (the sparse-only rows of the paper's Tab. 1) on the headline shape.
WORKLOADS["cogvideox5b_bf16"] = WORKLOADS["cogvideox5b"].replace(name="cogvideox5b_bf16", bits_qk=16, bits_pv=16)
# The all-INT4 setting of the paper's Tab. 1 ("QK (INT4), PV (INT4)") on the shape and density of the INT4-PV config.
WORKLOADS["cogvideox5b_int4"] = WORKLOADS["cogvideox5b_int4pv"].replace(name="cogvideox5b_int4", bits_qk=4)


# --------------------------------------------------------------------------------------------
# bf16 helpers (storage format only)
# --------------------------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16, returned as float32."""
    return bf16_to_f32(bf16_bits(x))


# --------------------------------------------------------------------------------------------
# Q, K, V
# --------------------------------------------------------------------------------------------
def _grid_coords(w: Workload) -> np.ndarray:
    """Grid coordinate (f, h, w) of every image token in the default [F,H,W] sequence order."""
    f, h, x = np.meshgrid(np.arange(w.F), np.arange(w.Hg), np.arange(w.Wg), indexing="ij")
    return np.stack([f.ravel(), h.ravel(), x.ravel()], axis=1).astype(np.float64)


def make_head_qkv(w: Workload, b: int, h: int):
    """Q, K, V of one (batch, head): three float32 arrays [N, d] in the default token order.

    X = G + A * phi_h(pos) with G ~ N(0,1) i.i.d. and phi_h random Fourier features whose inner
    product approximates a Gaussian RBF of the grid distance (width ``sigma`` cells).  The
    positional part is shared by Q, K and V of the head, so q.k/sqrt(d) carries a bump of
    about 8 on top of unit-scale noise for 3-D neighbours: the local-aggregation structure.
    Text tokens get G only.  For ``dtype == "bf16"`` values are rounded to bfloat16.
    """
    rng = np.random.default_rng([w.seed, 7, b, h])
    rng_pos = np.random.default_rng([w.seed, 11, h])  # shared over the batch
    omega = rng_pos.normal(0.0, 1.0 / w.sigma, size=(w.d, 3))
    beta = rng_pos.uniform(0.0, 2.0 * math.pi, size=(w.d,))
    amp = math.sqrt(8.0 * math.sqrt(w.d))
    phi = math.sqrt(2.0 / w.d) * np.cos(_grid_coords(w) @ omega.T + beta)  # [n_img, d]
    out = []
    for _ in range(3):
        g = rng.standard_normal(size=(w.N, w.d))
        g[: w.n_img] += amp * phi
        x = g.astype(np.float32)
        if w.dtype == "bf16":
            x = bf16_round(x)
        out.append(x)
    return out[0], out[1], out[2]


def make_qkv(w: Workload):
    """Q, K, V of the whole problem: float32 arrays [B, nh, N, d]."""
    q = np.empty((w.B, w.nh, w.N, w.d), np.float32)
    k = np.empty_like(q)
    v = np.empty_like(q)
    for b in range(w.B):
        for h in range(w.nh):
            q[b, h], k[b, h], v[b, h] = make_head_qkv(w, b, h)
    return q, k, v


def make_perm_ids(w: Workload) -> np.ndarray:
    """Per-head axis-order id in 0..5 (uint8)."""
    if w.perm_choice is not None:
        return np.array([w.perm_choice[h % len(w.perm_choice)] for h in range(w.nh)], np.uint8)
    rng = np.random.default_rng([w.seed, 13])
    return rng.integers(0, 6, size=w.nh).astype(np.uint8)


# --------------------------------------------------------------------------------------------
# Block masks
# --------------------------------------------------------------------------------------------
def _axis_kernel(n: int, sigma: float) -> np.ndarray:
    i = np.arange(n, dtype=np.float64)
    return np.exp(-((i[:, None] - i[None, :]) ** 2) / (2.0 * sigma * sigma))


def block_locality_scores(w: Workload, gather_index: np.ndarray) -> np.ndarray:
    """score[i, j] = sum over token pairs (p in block i, q in block j of the *reordered* image
    sequence) of exp(-|pos_p - pos_q|^2 / 2 sigma^2).

    ``gather_index[n']`` is the default-order position of the token that sits at position n' of
    the reordered sequence.  The Gaussian separates over the three axes, so the pair sum is
    evaluated by applying three small per-axis kernels to the block-membership tensor.
    """
    n_img, blk = w.n_img, w.block
    idx = np.asarray(gather_index[:n_img], dtype=np.int64)
    k_img = -(-n_img // blk)
    member = np.zeros((n_img, k_img), np.float64)
    member[idx, np.arange(n_img) // blk] = 1.0
    y = member.reshape(w.F, w.Hg, w.Wg, k_img)
    y = np.einsum("ab,bhwk->ahwk", _axis_kernel(w.F, w.sigma), y, optimize=True)
    y = np.einsum("ab,fbwk->fawk", _axis_kernel(w.Hg, w.sigma), y, optimize=True)
    y = np.einsum("ab,fhbk->fhak", _axis_kernel(w.Wg, w.sigma), y, optimize=True)
    y = y.reshape(n_img, k_img)[idx]
    return np.add.reduceat(y, np.arange(0, n_img, blk), axis=0)


def make_block_masks(w: Workload, gather_index_of: Callable[[int], np.ndarray], perm_ids=None,
                     score_cache: Optional[Dict[int, np.ndarray]] = None) -> np.ndarray:
    """Per-head static block mask, bool [nh, k, k], defined on the reordered sequence.

    Stand-in for the paper's offline block-sum thresholding (Sec. 4.2 (3)): per head the
    diagonal is kept, then the image x image blocks with the highest locality score until
    ``rint(density * k_img^2)`` are live (one global threshold per head, so rows differ in
    live count).  Ties go to the lower (i, j).  Text rows and columns are always live
    (Sec. 4.2 (1): sparsification applies to image tokens only).  ``score_cache`` (order id ->
    score map) may be shared between calls that differ only in density or seed.
    """
    if perm_ids is None:
        perm_ids = make_perm_ids(w)
    k, blk = w.k, w.block
    if w.T_text and w.n_img % blk:
        raise ValueError("image tokens must fill whole blocks when text tokens follow")
    k_img = -(-w.n_img // blk)
    n_live = max(k_img, int(np.rint(w.density * k_img * k_img)))
    cache: Dict[int, np.ndarray] = {} if score_cache is None else score_cache
    masks = np.zeros((w.nh, k, k), bool)
    for h in range(w.nh):
        pid = int(perm_ids[h])
        if pid not in cache:
            cache[pid] = block_locality_scores(w, gather_index_of(pid))
        rng = np.random.default_rng([w.seed, 17, h])
        score = cache[pid] * (1.0 + 1e-6 * rng.random(size=(k_img, k_img)))
        live = np.eye(k_img, dtype=bool)
        off = np.where(live.ravel(), -np.inf, score.ravel())
        order = np.argsort(-off, kind="stable")
        live.ravel()[order[: n_live - k_img]] = True
        masks[h, :k_img, :k_img] = live
        masks[h, k_img:, :] = True
        masks[h, :, k_img:] = True
    return masks


def pack_bitmask(masks: np.ndarray) -> np.ndarray:
    """bool [nh, k, k] -> uint8 [nh, ceil(k*k/8)]; bit (i*k + j) of a head, LSB-first per byte."""
    nh = masks.shape[0]
    return np.packbits(masks.reshape(nh, -1), axis=1, bitorder="little")


def live_blocks(masks: np.ndarray) -> int:
    return int(masks.sum())
