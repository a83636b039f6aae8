"""Pins of the oracle's optional K pre-conditioning (k_channel_mean, smooth_k): hand-worked values, the
invariance that defines it (a per-channel constant removed from every key leaves the unquantized softmax, dense or
block-masked, unchanged), and what it is for (smaller quantization groups when K carries a common offset)."""
import numpy as np

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl


def test_channel_mean_hand_worked_and_rounded_to_bfloat16():
    k = np.array([[1.0, 10.0], [3.0, 30.0], [2.0, 50.0]], np.float32)
    assert po.k_channel_mean(k).tolist() == [2.0, 30.0]
    assert po.smooth_k(k).tolist() == [[-1.0, -20.0], [1.0, 0.0], [0.0, 20.0]]
    # (1 + (1 + 2^-7)) / 2 = 1 + 2^-8 lies half-way between the bfloat16 neighbours 1 and 1 + 2^-7: ties go to even
    k = np.array([[1.0, 1.0 + 2.0 ** -6], [1.0 + 2.0 ** -7, 1.0 + 2.0 ** -7]], np.float32)
    assert po.k_channel_mean(k).tolist() == [1.0, 1.0 + 2.0 ** -6]  # second column: 1 + 1.5 * 2^-7 -> even neighbour 1 + 2^-6
    # the mean is taken over the tokens (axis 0), per channel
    k = np.arange(12, dtype=np.float32).reshape(4, 3)
    assert po.k_channel_mean(k).tolist() == [4.5, 5.5, 6.5]


def _case(offset):
    w = wl.Workload("smooth", 1, 1, 64, 2, 4, 12, 9, 32, 0.5, 8, 8, "f32", 77, perm_choice=(4,))
    q, k, v = (x[0, 0] for x in wl.make_qkv(w))
    k = (k + offset).astype(np.float32)
    perm_ids = wl.make_perm_ids(w)
    idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, int(perm_ids[0]))
    masks = wl.make_block_masks(w, lambda pid: po.perm_index(w.F, w.Hg, w.Wg, w.T_text, pid), perm_ids)
    row_ptr, col_idx = po.mask_to_blocklist(wl.pack_bitmask(masks), 1, w.k)
    return w, q, k, v, int(perm_ids[0]), row_ptr[0], col_idx


def _run(w, q, k, v, pid, rp, ci, bits, smooth):
    return po.paro_attention_head(q, k, v, (w.F, w.Hg, w.Wg), w.T_text, pid, w.block, rp, ci, bits, bits, smooth=smooth)


def test_unquantized_block_sparse_attention_does_not_see_the_smoothing():
    """Ragged N (105 = 3 * 32 + 9), text tokens, half of the blocks masked, K with a large common offset."""
    w, q, k, v, pid, rp, ci = _case(np.linspace(-6.0, 9.0, 64, dtype=np.float32)[None, :])
    plain = _run(w, q, k, v, pid, rp, ci, 0, False)
    smoothed = _run(w, q, k, v, pid, rp, ci, 0, True)
    assert np.abs(plain).max() > 0.1
    # the smoothed keys are rounded to binary32 once more: 1e-6 relative on logits of magnitude <= 100
    assert np.abs(plain - smoothed).max() <= 2e-4 * np.abs(plain).max()
    # and it is the column means that are removed
    assert np.abs(po.smooth_k(k).astype(np.float64).mean(axis=0)).max() <= 2.0 ** -8 * np.abs(k.astype(np.float64).mean(axis=0)).max()


def test_smoothing_shrinks_the_quantization_error_of_keys_with_a_common_offset():
    w, q, k, v, pid, rp, ci = _case(np.full((1, 64), 12.0, np.float32))
    exact = _run(w, q, k, v, pid, rp, ci, 0, False)
    err_plain = np.linalg.norm(_run(w, q, k, v, pid, rp, ci, 8, False) - exact)
    err_smooth = np.linalg.norm(_run(w, q, k, v, pid, rp, ci, 8, True) - exact)
    assert err_smooth < 0.7 * err_plain  # the errors of Q, P and V stay
    # the codes of the smoothed keys: padded rows stay zero, scales shrink to those of the offset-free keys
    idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, pid)
    kc, sk = po.prepare_operand(po.smooth_k(k), idx, w.npad, w.block, 8)
    kc0, sk0 = po.prepare_operand(k, idx, w.npad, w.block, 8)
    assert not kc[w.N:].any()
    assert (sk < 0.5 * sk0).all()
