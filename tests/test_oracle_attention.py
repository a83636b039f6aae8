"""Pins for the oracle's block-sparse quantized attention (CPU only).

The paper prints no worked numeric example of the quantized kernel, so the attention oracle is
pinned by (i) the library/brute-force dense and masked softmax it must reduce to with
quantization off, (ii) permutation equivariance, (iii) closed forms in which the block-wise
quantization is exact (block-constant logits with integer-valued operands; b = 1), which
exercise the scales, the running-maximum rescaling, the P-tile scale and the ragged tail with
quantization ON, (iv) 1/qmax convergence and an a-priori error bound.
"""
import math

import numpy as np
import pytest
import torch

from oracle import paro_oracle as po


def sdpa_reference(q, k, v, token_mask=None):
    """softmax(q k^T / sqrt(d)) v by the library routine, float64."""
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))[None] for a in (q, k, v))
    am = None if token_mask is None else torch.from_numpy(token_mask)[None]
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=am)[0].numpy()


def brute_force(q, k, v, token_mask=None):
    x = (q.astype(np.float64) @ k.astype(np.float64).T) / math.sqrt(q.shape[1])
    if token_mask is not None:
        x = np.where(token_mask, x, -np.inf)
    p = np.exp(x - x.max(axis=1, keepdims=True))
    return (p @ v.astype(np.float64)) / p.sum(axis=1, keepdims=True)


def full_list(k):
    row_ptr = np.arange(0, k * k + 1, k, dtype=np.int32)
    col_idx = np.tile(np.arange(k, dtype=np.int32), k)
    return row_ptr, col_idx


def list_from_mask(m):
    k = m.shape[0]
    bits = np.packbits(m.reshape(1, -1), axis=1, bitorder="little")
    rp, ci = po.mask_to_blocklist(bits, 1, k)
    return rp[0], ci


def rand_mask(rng, k, p=0.5):
    m = rng.random((k, k)) < p
    m |= np.eye(k, dtype=bool)
    return m


def token_mask_from_blocks(m, block, n):
    return np.kron(m, np.ones((block, block), bool))[:n, :n]


def unquantized_head(q, k, v, n, block, rp, ci, qmax_p=None):
    kb = -(-n // block)
    npad = kb * block
    ones = np.ones(kb, np.float32)

    def pad(a):
        out = np.zeros((npad, a.shape[1]))
        out[:n] = a
        return out

    return po.sparse_attention_head(pad(q), ones, pad(k), ones, pad(v), ones, n, block, rp, ci, qmax_p)[:n]


# ----------------------------------------------------------- (i) dense and masked limits
@pytest.mark.parametrize("n,block", [(64, 16), (70, 16), (37, 8)])
def test_dense_limit_equals_library_softmax(n, block):
    rng = np.random.default_rng(n)
    d = 16
    q, k, v = (rng.standard_normal((n, d)) * 1.5 for _ in range(3))
    rp, ci = full_list(-(-n // block))
    o = unquantized_head(q, k, v, n, block, rp, ci)
    assert np.allclose(o, sdpa_reference(q, k, v), rtol=0, atol=1e-12)
    assert np.allclose(o, brute_force(q, k, v), rtol=0, atol=1e-12)


@pytest.mark.parametrize("n,block", [(64, 16), (75, 16)])
def test_dropping_a_block_equals_minus_inf_logits(n, block):
    rng = np.random.default_rng(n + 1)
    d = 8
    kb = -(-n // block)
    q, k, v = (rng.standard_normal((n, d)) * 2 for _ in range(3))
    m = rand_mask(rng, kb, 0.4)
    rp, ci = list_from_mask(m)
    o = unquantized_head(q, k, v, n, block, rp, ci)
    tm = token_mask_from_blocks(m, block, n)
    assert np.allclose(o, brute_force(q, k, v, tm), rtol=0, atol=1e-12)
    assert np.allclose(o, sdpa_reference(q, k, v, tm), rtol=0, atol=1e-12)


def test_empty_row_block_gives_zeros():
    rng = np.random.default_rng(5)
    n, block, d = 32, 8, 4
    q, k, v = (rng.standard_normal((n, d)) for _ in range(3))
    m = np.eye(4, dtype=bool)
    m[2] = False
    rp, ci = list_from_mask(m)
    o = unquantized_head(q, k, v, n, block, rp, ci)
    assert np.all(o[16:24] == 0) and np.all(np.abs(o[:16]).sum(axis=1) > 0)


# ----------------------------------------------------------- (ii) equivariance of the full path
@pytest.mark.parametrize("perm_id", range(6))
def test_full_path_dense_unquantized_is_order_invariant(perm_id):
    rng = np.random.default_rng(11)
    F, H, W, T, d, block = 2, 3, 4, 3, 8, 8
    n = F * H * W + T
    q, k, v = (rng.standard_normal((n, d)) for _ in range(3))
    rp, ci = full_list(-(-n // block))
    o = po.paro_attention_head(q, k, v, (F, H, W), T, perm_id, block, rp, ci, 0, 0)
    assert o.shape == (n, d)
    assert np.allclose(o, sdpa_reference(q, k, v), rtol=0, atol=1e-12)


def test_full_path_mask_lives_in_reordered_coordinates():
    # The block mask indexes the reordered sequence (Sec. 4.2: masks are made after the reorder):
    # keeping only diagonal blocks under order WHF equals a token mask built from the gather index.
    rng = np.random.default_rng(12)
    F, H, W, d, block = 2, 4, 4, 8, 8
    n = F * H * W
    q, k, v = (rng.standard_normal((n, d)) for _ in range(3))
    m = np.eye(n // block, dtype=bool)
    m[0, 2] = True
    rp, ci = list_from_mask(m)
    o = po.paro_attention_head(q, k, v, (F, H, W), 0, 5, block, rp, ci, 0, 0)
    idx = np.arange(n).reshape(F, H, W).transpose(2, 1, 0).reshape(-1)  # WHF by numpy
    tm_new = token_mask_from_blocks(m, block, n)
    tm = np.zeros((n, n), bool)
    tm[np.ix_(idx, idx)] = tm_new
    assert np.allclose(o, brute_force(q, k, v, tm), rtol=0, atol=1e-12)


# ----------------------------------------------------------- (iii) closed forms, quantization ON
@pytest.mark.parametrize("bits_pv", [8, 4])
@pytest.mark.parametrize("n", [64, 59])
def test_block_constant_logits_closed_form(bits_pv, n):
    """Rows of Q equal within a block, rows of K equal within a block, all operands integer
    multiples of their block scale with the absmax at qmax: every quantizer is exact and every
    P tile is constant (codes all qmax_P).  Then O_i = sum_j e^{x_ij} (sum_{n in j} v_n) /
    sum_j n_j e^{x_ij} with x_ij = a_i . b_j / sqrt(d), written here from the raw inputs."""
    rng = np.random.default_rng(100 + n + bits_pv)
    block, d = 16, 8
    kb = -(-n // block)
    npad = kb * block
    qv = po.qmax_of(bits_pv)
    unit = 2.0**-5
    a = rng.integers(-40, 41, size=(kb, d)).astype(np.float64)
    b = rng.integers(-40, 41, size=(kb, d)).astype(np.float64)
    a[:, 0] = 127
    b[:, 1] = -127
    q = np.repeat(a, block, axis=0)[:n] * unit
    k = np.repeat(b, block, axis=0)[:n] * unit
    v = rng.integers(-qv, qv + 1, size=(n, d)).astype(np.float64)
    for j in range(kb):
        v[j * block, 2] = qv  # absmax of every V block is qmax -> scale 0.25 exactly
    v *= 0.25
    m = rand_mask(rng, kb, 0.6)
    rp, ci = list_from_mask(m)

    def prep(x, bits):
        xp = np.zeros((npad, d), np.float32)
        xp[:n] = x
        return po.quantize_blocks(xp, n, block, po.qmax_of(bits))

    qc, sq = prep(q, 8)
    kc, sk = prep(k, 8)
    vc, sv = prep(v, bits_pv)
    assert np.all(sq == np.float32(unit)) and np.all(sv == np.float32(0.25))
    o = po.sparse_attention_head(qc, sq, kc, sk, vc, sv, n, block, rp, ci, qv)[:n]

    x = (a * unit) @ (b * unit).T / math.sqrt(d)  # [kb, kb] block logits
    expect = np.zeros((n, d))
    for i in range(kb):
        js = np.nonzero(m[i])[0]
        w = np.exp(x[i, js] - x[i, js].max())
        num = sum(wj * v[j * block : min((j + 1) * block, n)].sum(axis=0) for wj, j in zip(w, js))
        den = sum(wj * (min((j + 1) * block, n) - j * block) for wj, j in zip(w, js))
        expect[i * block : min((i + 1) * block, n)] = num / den
    assert np.allclose(o, expect, rtol=1e-12, atol=1e-12)


def test_zero_queries_average_the_live_valid_values():
    # Q = 0 -> all logits 0 -> P tile all ones -> O = mean of dequantized V over live, valid keys
    # (a padded key that leaked in would pull the mean toward 0).
    rng = np.random.default_rng(21)
    n, block, d = 43, 8, 4
    kb = -(-n // block)
    npad = kb * block
    v = np.zeros((npad, d), np.float32)
    v[:n] = rng.integers(-127, 128, size=(n, d))
    v[np.arange(0, n, block), 0] = 127
    vc, sv = po.quantize_blocks(v, n, block, 127)
    assert np.all(sv == 1.0)
    kc, sk = po.quantize_blocks(rng.standard_normal((npad, d)).astype(np.float32), n, block, 127)
    qc, sq = np.zeros((npad, d), np.int32), np.ones(kb, np.float32)
    m = rand_mask(rng, kb, 0.5)
    m[:, kb - 1] = True  # every row sees the ragged last block
    rp, ci = list_from_mask(m)
    o = po.sparse_attention_head(qc, sq, kc, sk, vc, sv, n, block, rp, ci, 127)[:n]
    for i in range(kb):
        keys = np.concatenate([np.arange(j * block, min((j + 1) * block, n)) for j in np.nonzero(m[i])[0]])
        rows = slice(i * block, min((i + 1) * block, n))
        assert np.allclose(o[rows], v[keys].mean(axis=0, dtype=np.float64), rtol=1e-13, atol=1e-13)


def test_block_of_one_token_makes_quantization_exact():
    # b = 1, d = 1: every group holds one number, so codes are +-qmax and dequantize exactly;
    # every P tile is 1x1.  The quantized path must then equal the exact masked softmax.
    rng = np.random.default_rng(31)
    n = 12
    q, k, v = (rng.standard_normal((n, 1)).astype(np.float32) * 2 for _ in range(3))
    m = rand_mask(rng, n, 0.5)
    rp, ci = list_from_mask(m)
    o = po.paro_attention_head(q, k, v, (1, 3, 4), 0, 5, 1, rp, ci, 8, 8)
    idx = np.arange(n).reshape(1, 3, 4).transpose(2, 1, 0).reshape(-1)
    tm = np.zeros((n, n), bool)
    tm[np.ix_(idx, idx)] = m
    assert np.allclose(o, brute_force(q, k, v, tm), rtol=1e-5, atol=1e-6)


# ----------------------------------------------------------- (iv) convergence, monotonicity, bound
def _quantized_vs_exact(seed, qmax_qk, qmax_v, qmax_p, n=96, block=16, d=16):
    rng = np.random.default_rng(seed)
    kb = -(-n // block)
    npad = kb * block
    q, k, v = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    m = rand_mask(rng, kb, 0.5)
    rp, ci = list_from_mask(m)

    def prep(x, qmax):
        xp = np.zeros((npad, d), np.float32)
        xp[:n] = x
        return po.quantize_blocks(xp, n, block, qmax)

    qc, sq = prep(q, qmax_qk)
    kc, sk = prep(k, qmax_qk)
    vc, sv = prep(v, qmax_v)
    o = po.sparse_attention_head(qc, sq, kc, sk, vc, sv, n, block, rp, ci, qmax_p)[:n]
    ref = brute_force(q, k, v, token_mask_from_blocks(m, block, n))
    return np.linalg.norm(o - ref) / np.linalg.norm(ref)


def test_error_vanishes_like_one_over_qmax():
    e8 = _quantized_vs_exact(41, 127, 127, 127)
    e12 = _quantized_vs_exact(41, 2047, 2047, 2047)
    e16 = _quantized_vs_exact(41, 32767, 32767, 32767)
    assert 0 < e16 < e12 < e8 < 0.05
    assert 8 < e8 / e12 < 32 and 8 < e12 / e16 < 32  # 16x finer grid -> about 16x smaller error


def test_error_grows_as_bits_shrink():
    e8 = _quantized_vs_exact(42, 127, 127, 127)
    e4pv = _quantized_vs_exact(42, 127, 7, 7)
    e4 = _quantized_vs_exact(42, 7, 7, 7)
    assert e8 < e4pv < e4 < 1.0


def test_p_quantization_error_within_a_priori_bound():
    # Only P quantized.  Each visited tile adds at most (s_P/2) * sum_keys |v| to a row of the
    # numerator, later shrunk by factors alpha <= 1; s_P <= 1/qmax and the denominator is >= 1.
    rng = np.random.default_rng(43)
    n, block, d, qmax = 80, 16, 8, 127
    kb = n // block
    q, k, v = (rng.standard_normal((n, d)) for _ in range(3))
    m = rand_mask(rng, kb, 0.7)
    rp, ci = list_from_mask(m)
    exact = unquantized_head(q, k, v, n, block, rp, ci, None)
    quant = unquantized_head(q, k, v, n, block, rp, ci, qmax)
    assert not np.array_equal(exact, quant)
    tm = token_mask_from_blocks(m, block, n)
    bound = (tm.astype(float) @ np.abs(v)) / (2 * qmax)
    assert np.all(np.abs(quant - exact) <= bound)
    # and the typical error is far below the worst case but not zero
    assert 1e-6 < np.abs(quant - exact).max() < 0.2 * bound.max()


def test_cast_output_bf16_rounds_to_nearest_even():
    x = np.array([1.0, 1.0 + 2.0**-9, 1.0 + 2.0**-8, 1.0 + 3 * 2.0**-9, -3.14159])
    got = po.cast_output(x, "bf16")
    # bf16 has 8 significand bits: spacing 2^-7 in [1,2); ties go to the even neighbour
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == 1.0 and got[3] == 1.0 + 2.0**-7
    assert abs(got[4] + 3.14159) < 2.0**-7
    assert po.cast_output(x, "f32")[4] == np.float32(-3.14159)


def _order_case():
    """Hand-worked case in which the visiting order decides the result (Sec. 4.3 (1),(2): the P tile
    is quantized as one group against the running row maxima at the time of the visit).

    b = 2, d = 1, one row block with queries A = +1 and B = -1, scales chosen so that a logit is
    (q * k) * ln 2, i.e. P entries are powers of two.  Column block 0 holds keys (2, 0), column
    block 1 keys (-2, 0); V codes are (1, 2 | 3, 4), all scales 1.

    Ascending (block 0, then block 1):
      block 0: A sees logits (2, 0) ln2 -> m = 2, P = (1, 1/4);  B sees (-2, 0) -> m = 0, P = (1/4, 1);
               tile maximum 1, sP = 1/127, codes A (127, 32) [31.75 -> 32], B (32, 127); l = 5/4 each.
      block 1: A sees (-2, 0): m stays 2, P = (1/16, 1/4);  B sees (2, 0): m -> 2, earlier sums x 1/4,
               P = (1, 1/4); tile maximum 1, codes A (8, 32) [7.9375 -> 8], B (127, 32).
      l = 5/4 + 5/16 = 25/16 (A) and 5/16 + 5/4 = 25/16 (B).
      numerator A = (127*1 + 32*2) + (8*3 + 32*4) = 343,  B = (32*1 + 127*2)/4 + (127*3 + 32*4) = 580.5
    Descending (block 1, then block 0) the same steps give
      numerator A = (32*3 + 127*4)/4 + (127*1 + 32*2) = 342,  B = (127*3 + 32*4) + (8*1 + 32*2) = 581.
    Each output is numerator / 127 / (25/16)."""
    ln2 = np.float32(math.log(2.0))
    q = np.array([[1.0], [-1.0], [0.0], [0.0]])
    k = np.array([[2.0], [0.0], [-2.0], [0.0]])
    v = np.array([[1.0], [2.0], [3.0], [4.0]])
    sq = np.array([ln2, 1.0], np.float32)
    ones = np.ones(2, np.float32)
    return q, sq, k, ones, v, ones


def test_live_blocks_are_visited_in_ascending_order_hand_worked():
    q, sq, k, sk, v, sv = _order_case()
    rp = np.array([0, 2, 2], np.int32)
    o = po.sparse_attention_head(q, sq, k, sk, v, sv, 4, 2, rp, np.array([0, 1], np.int32), 127)
    l = 25.0 / 16.0
    assert o[0, 0] == pytest.approx(343.0 / 127.0 / l, rel=1e-6)
    assert o[1, 0] == pytest.approx(580.5 / 127.0 / l, rel=1e-6)
    assert np.all(o[2:] == 0)
    # the descending visit is a different result, by more than the tolerance of the check above
    assert abs(343.0 - 342.0) / 343.0 > 1e-3 and abs(581.0 - 580.5) / 581.0 > 5e-4


def test_block_list_order_is_the_visiting_order_hand_worked():
    # the same case with the list holding the blocks in descending order: the other hand-worked values
    q, sq, k, sk, v, sv = _order_case()
    rp = np.array([0, 2, 2], np.int32)
    o = po.sparse_attention_head(q, sq, k, sk, v, sv, 4, 2, rp, np.array([1, 0], np.int32), 127)
    l = 25.0 / 16.0
    assert o[0, 0] == pytest.approx(342.0 / 127.0 / l, rel=1e-6)
    assert o[1, 0] == pytest.approx(581.0 / 127.0 / l, rel=1e-6)


def test_whole_path_visits_a_mask_rows_ascending_hand_worked():
    # the same case through the bitmask -> block list -> attention path: the list made from a mask is ascending
    q, sq, k, sk, v, sv = _order_case()
    bits = np.array([[0b0011]], np.uint8)  # row block 0 attends column blocks 0 and 1 (k = 2: bits 0 and 1)
    rp, ci = po.mask_to_blocklist(bits, 1, 2)
    assert ci.tolist() == [0, 1]
    o = po.sparse_attention_head(q, sq, k, sk, v, sv, 4, 2, rp[0], ci, 127)
    assert o[0, 0] == pytest.approx(343.0 / 127.0 / (25.0 / 16.0), rel=1e-6)
    assert o[1, 0] == pytest.approx(580.5 / 127.0 / (25.0 / 16.0), rel=1e-6)


def test_tie_risk_bounds_the_effect_of_a_rounding_tie():
    # One 2x2 tile, d = 1, P = [[1, .5], [1, .5]] -> P / sP = [127, 63.5]: a tie.  Rounding the
    # tie the other way moves the output by exactly sP * |v1| / l, which is what the test-side
    # observer reports.
    from tests.helpers import TieRisk

    n, block = 2, 2
    q = np.ones((2, 1))
    k = np.array([[0.0], [-math.log(2.0)]])
    v = np.array([[3.0], [-5.0]])
    ones = np.ones(1, np.float32)
    rp, ci = np.array([0, 1], np.int32), np.array([0], np.int32)
    risk = TieRisk(v, ones, block, n, tol=1e-9)
    o = po.sparse_attention_head(q, ones, k, ones, v, ones, n, block, rp, ci, 127, observer=risk)
    assert np.array_equal(o, po.sparse_attention_head(q, ones, k, ones, v, ones, n, block, rp, ci, 127))  # observing changes nothing
    l = 1.5
    up = (127 * 3.0 + 64 * -5.0) / 127 / l
    down = (127 * 3.0 + 63 * -5.0) / 127 / l
    assert np.allclose(o[:, 0], up, rtol=1e-12) or np.allclose(o[:, 0], down, rtol=1e-12)
    assert np.allclose(risk.out[:, 0], 5.0 / 127 / l, rtol=1e-12)
    assert abs(up - down) <= risk.out[0, 0] * (1 + 1e-12)
    # away from ties nothing is flagged
    risk2 = TieRisk(v, ones, block, n, tol=1e-9)
    k2 = np.array([[0.0], [-0.3]])
    po.sparse_attention_head(q, ones, k2, ones, v, ones, n, block, rp, ci, 127, observer=risk2)
    assert np.all(risk2.out == 0)


def test_bf16_mode_rounds_operands_only():
    # bits 16 = operands held in bfloat16, P and all accumulation exact: equals the exact masked
    # softmax evaluated on bf16-rounded inputs (torch's bfloat16 cast is the independent rounding).
    rng = np.random.default_rng(77)
    F, H, W, d, block = 2, 4, 4, 8, 8
    n = F * H * W
    q, k, v = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    m = rand_mask(rng, n // block, 0.5)
    rp, ci = list_from_mask(m)
    o = po.paro_attention_head(q, k, v, (F, H, W), 0, 0, block, rp, ci, 16, 16)
    qb, kb, vb = (torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy() for a in (q, k, v))
    assert not np.array_equal(qb, q)
    tm = token_mask_from_blocks(m, block, n)
    assert np.allclose(o, brute_force(qb, kb, vb, tm), rtol=0, atol=1e-12)
