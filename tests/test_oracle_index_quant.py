"""Pins for the oracle's token reorder, quantizer and block list (CPU only).

Each check ties the oracle to something other than itself: a numpy library routine, a closed
form, a number printed in the paper, or brute force on a tiny input.
"""
import json
import os

import numpy as np
import pytest

from oracle import paro_oracle as po

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")))


# ------------------------------------------------------------------ reorder (Sec. 1, Sec. 4.1)
def test_six_orders_named_lexicographically():
    assert len(po.AXIS_ORDERS) == GOLD["num_orders"]["value"]
    assert [po.order_name(p) for p in range(6)] == ["FHW", "FWH", "HFW", "HWF", "WFH", "WHF"]


@pytest.mark.parametrize("grid", [(2, 8, 8), (3, 4, 5), (1, 6, 7), (13, 30, 45)])
@pytest.mark.parametrize("perm_id", range(6))
def test_perm_index_equals_numpy_transpose(grid, perm_id):
    F, H, W = grid
    n = F * H * W
    idx = po.perm_index(F, H, W, 0, perm_id)
    ref = np.arange(n).reshape(F, H, W).transpose(po.AXIS_ORDERS[perm_id]).reshape(-1)
    assert np.array_equal(idx, ref)
    assert np.array_equal(np.sort(idx), np.arange(n))  # bijection


def test_default_order_is_identity_and_frame_stride():
    F, H, W = 13, 30, 45
    assert F * H * W == GOLD["token_length"]["value"]
    idx = po.perm_index(F, H, W, 0, 0)
    assert np.array_equal(idx, np.arange(F * H * W))
    # In order [H, W, F] the frame axis is fastest: consecutive reordered tokens are the
    # frame neighbours, which sit H*W apart in the default order (Sec. 1).
    idx_hwf = po.perm_index(F, H, W, 0, 3)
    assert po.order_name(3) == "HWF"
    assert np.all(np.diff(idx_hwf[:F]) == H * W)


@pytest.mark.parametrize("perm_id", range(6))
def test_text_tokens_keep_their_place(perm_id):
    idx = po.perm_index(2, 3, 4, 5, perm_id)
    assert np.array_equal(idx[24:], np.arange(24, 29))
    assert np.array_equal(np.sort(idx), np.arange(29))


@pytest.mark.parametrize("perm_id", range(6))
def test_permute_unpermute_round_trip(perm_id):
    rng = np.random.default_rng(perm_id)
    F, H, W, T, d, blk = 3, 5, 4, 3, 8, 16
    n = F * H * W + T
    npad = -(-n // blk) * blk
    x = rng.standard_normal((n, d))
    idx = po.perm_index(F, H, W, T, perm_id)
    xp = po.permute(x, idx, npad)
    assert xp.shape == (npad, d)
    assert np.all(xp[n:] == 0)
    assert np.array_equal(xp[:n], x[idx])  # library fancy-indexing gather
    assert np.array_equal(po.unpermute(xp, idx), x)


def test_perm_id_range_checked():
    with pytest.raises(ValueError):
        po.perm_index(2, 2, 2, 0, 6)


# ------------------------------------------------------------------ quantizer (Sec. 4.3 (1))
@pytest.mark.parametrize("bits", [8, 4])
def test_quantizer_half_step_bound_and_extremes(bits):
    rng = np.random.default_rng(bits)
    qmax = po.qmax_of(bits)
    blk, d, k = 16, 8, 5
    x = (rng.standard_normal((blk * k, d)) * rng.uniform(0.1, 30, size=(blk * k, 1))).astype(np.float32)
    n_valid = blk * k - 5
    x[n_valid:] = 0
    codes, scales = po.quantize_blocks(x, n_valid, blk, qmax)
    assert codes.dtype == np.int32 and scales.dtype == np.float32
    assert np.abs(codes).max() <= qmax
    deq = po.dequantize_blocks(codes, scales, blk)
    for b in range(k):
        lo, hi = b * blk, min((b + 1) * blk, n_valid)
        tile = x[lo:hi].astype(np.float64)
        s = float(scales[b])
        # scale is absmax / qmax (binary32 divide)
        assert scales[b] == np.float32(np.abs(x[lo:hi]).max()) / np.float32(qmax)
        # |x - s*code| <= s/2 (plus binary32 rounding of the quotient)
        assert np.max(np.abs(tile - deq[lo:hi])) <= 0.5 * s * (1 + 1e-6)
        # the absmax element codes to +-qmax
        r, c = np.unravel_index(np.argmax(np.abs(tile)), tile.shape)
        assert abs(codes[lo + r, c]) == qmax
        assert np.sign(codes[lo + r, c]) == np.sign(tile[r, c])
    assert np.all(codes[n_valid:] == 0)


def test_quantizer_hand_worked_block():
    # One block of 2 tokens x 2 channels, absmax 2.54 -> scale 0.02 for INT8.
    x = np.array([[2.54, -1.27], [0.03, 0.0]], np.float32)
    codes, scales = po.quantize_blocks(x, 2, 2, 127)
    assert abs(float(scales[0]) - 0.02) < 1e-8
    assert codes.tolist() == [[127, -64], [2, 0]] or codes.tolist() == [[127, -63], [2, 0]]
    # -1.27/0.02 = -63.5 is a tie only in exact arithmetic; in binary32 2.54f/127 is slightly
    # off 0.02, so accept either neighbour but require the INT4 case, which has no tie:
    codes4, scales4 = po.quantize_blocks(np.array([[7.0, -3.4], [0.6, 0.4]], np.float32), 2, 2, 7)
    assert float(scales4[0]) == 1.0
    assert codes4.tolist() == [[7, -3], [1, 0]]


def test_quantizer_round_half_to_even():
    # scale exactly 1: ties at .5 must go to the even integer
    x = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5]], np.float32)
    codes, scales = po.quantize_blocks(x, 1, 1, 127)
    assert float(scales[0]) == 1.0
    assert codes[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 4]


def test_quantizer_zero_block_and_scale_per_block():
    x = np.zeros((8, 4), np.float32)
    x[4:] = 3.0
    codes, scales = po.quantize_blocks(x, 8, 4, 127)
    assert float(scales[0]) == 1.0 and np.all(codes[:4] == 0)
    assert np.all(codes[4:] == 127)
    assert scales[1] == np.float32(3.0) / np.float32(127)


def test_quantizer_ignores_padded_rows_in_absmax():
    x = np.ones((4, 2), np.float32)
    x[3] = 100.0  # a padded row holding garbage must not set the scale
    codes, scales = po.quantize_blocks(x, 3, 4, 127)
    assert scales[0] == np.float32(1.0) / np.float32(127)
    assert np.all(codes[:3] == 127) and np.all(codes[3] == 0)


def test_p_tile_quantizer_bound_and_max():
    rng = np.random.default_rng(3)
    p = np.exp(-rng.uniform(0, 12, size=(16, 16)))
    for qmax in (127, 7):
        codes, s_p = po.quantize_p_tile(p, np.ones_like(p, bool), qmax)
        assert s_p == p.max() / qmax
        assert codes.max() == qmax and codes.min() >= 0
        assert np.all(codes == np.round(codes))
        assert np.max(np.abs(codes * s_p - p)) <= 0.5 * s_p * (1 + 1e-12)
    codes, s_p = po.quantize_p_tile(np.zeros((4, 4)), np.ones((4, 4), bool), 127)
    assert s_p == 0.0 and np.all(codes == 0)
    # ties: 0.5 -> 0, 1.5 -> 2 when the scale is exactly 1
    codes, s_p = po.quantize_p_tile(np.array([[127.0, 0.5, 1.5, 2.5]]), np.ones((1, 4), bool), 127)
    assert s_p == 1.0 and codes[0].tolist() == [127, 0, 2, 2]


def test_incoherence_matches_hand_worked_example():
    ex = GOLD["incoherence_example"]
    assert po.incoherence(np.array(ex["x"], float)) == ex["psi"]


# ------------------------------------------------------------------ block list (Sec. 4.2)
def test_mask_geometry_matches_paper_size():
    n = GOLD["token_length"]["value"]
    b = GOLD["block_size"]["value"]
    k = -(-n // b)
    assert k == 275
    # 1 bit per 64x64 block -> 9454 B = 9.2 KiB, the size the paper prints
    assert po.mask_nbytes(k) == 9454
    assert round(po.mask_nbytes(k) / 1024, 1) == GOLD["mask_kib_per_head"]["value"]


@pytest.mark.parametrize("k", [1, 3, 8, 11])
def test_blocklist_equals_brute_force(k):
    rng = np.random.default_rng(k)
    nh = 3
    m = rng.random((nh, k, k)) < 0.4
    m[1] = False  # a head with empty rows
    m[2] = True
    bits = np.packbits(m.reshape(nh, -1), axis=1, bitorder="little")
    assert bits.shape[1] == po.mask_nbytes(k)
    row_ptr, col_idx = po.mask_to_blocklist(bits, nh, k)
    assert row_ptr.shape == (nh, k + 1) and col_idx.dtype == np.int32
    assert row_ptr[-1, -1] == col_idx.size == m.sum()  # nnz = popcount
    for h in range(nh):
        for i in range(k):
            got = col_idx[row_ptr[h, i] : row_ptr[h, i + 1]]
            assert np.array_equal(got, np.nonzero(m[h, i])[0])  # ascending
        if h + 1 < nh:
            assert row_ptr[h, k] == row_ptr[h + 1, 0]


def test_blocklist_bit_order_is_lsb_first():
    # k = 3: bit index i*3+j. Byte 0 = 0b00100001 -> bits 0 and 5 -> (0,0) and (1,2); byte 1 = 1 -> bit 8 -> (2,2)
    bits = np.array([[0b00100001, 0b1]], np.uint8)
    row_ptr, col_idx = po.mask_to_blocklist(bits, 1, 3)
    assert row_ptr.tolist() == [[0, 1, 2, 3]]
    assert col_idx.tolist() == [0, 2, 2]
