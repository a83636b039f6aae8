"""Pins of the calibration oracle (oracle/paro_calibration.py) against what the paper's equations
and plain mathematics fix: hand-worked maps, brute-force loops over Eq. (M_sparse)/(M_quant),
row-stochastic invariants under reordering, closed forms of the combined metric, and a
constructed head whose best axis order is known."""
import itertools

import numpy as np
import pytest
from scipy.special import softmax

from oracle import paro_calibration as pc
from oracle import paro_oracle as po


def test_incoherence_of_the_worked_example_and_the_papers_example_thresholds():
    import json
    import os

    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")))
    ex = gold["incoherence_example"]
    x = np.abs(np.array(ex["x"], float))
    psi = pc.psi_blocks(np.array([[x.max()]]), np.array([[x.sum()]]), np.array([[x.size]]))
    assert psi[0, 0] == pytest.approx(ex["psi"])
    # the example thresholds of Sec. 4.1: a block with exactly 90 % of its entries below 1e-3 counts as sparse
    eps, sigma = gold["sparse_metric_examples"]["epsilon"], gold["sparse_metric_examples"]["sigma"]
    blk = np.full((10, 10), 2e-3)
    blk.ravel()[:90] = 5e-4
    st = pc.block_stats(blk, 10, eps)
    assert st["cnt"][0, 0] == 90 and pc.m_sparse(st["cnt"], pc.block_entries(10, 10), sigma) == 1.0
    blk.ravel()[89] = 2e-3
    st = pc.block_stats(blk, 10, eps)
    assert st["cnt"][0, 0] == 89 and pc.m_sparse(st["cnt"], pc.block_entries(10, 10), sigma) == 0.0


def test_attention_map_is_the_library_softmax_on_bf16_operands():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((37, 16)).astype(np.float32)
    k = rng.standard_normal((37, 16)).astype(np.float32)
    p = pc.attention_map(q, k)
    qb, kb = po.round_to_bf16(q).astype(np.float64), po.round_to_bf16(k).astype(np.float64)
    ref = softmax(qb @ kb.T / 4.0, axis=1)
    assert np.allclose(p, ref, rtol=1e-13, atol=0)
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14)
    # the rounding matters: the map of unrounded operands differs measurably
    assert np.abs(softmax(q.astype(np.float64) @ k.astype(np.float64).T / 4.0, axis=1) - p).max() > 1e-5


def test_hand_worked_identity_map():
    p = np.eye(4)
    st = pc.block_stats(p, 2, 0.5)
    assert st["sum"].tolist() == [[2, 0], [0, 2]]
    assert st["max"].tolist() == [[1, 0], [0, 1]]
    assert st["cnt"].tolist() == [[2, 4], [4, 2]]
    ent = pc.block_entries(4, 2)
    assert ent.tolist() == [[4, 4], [4, 4]]
    assert pc.m_sparse(st["cnt"], ent, 0.9) == 0.5   # only the two zero blocks reach 90 %
    assert pc.m_sparse(st["cnt"], ent, 0.5) == 1.0   # ">=": exactly half of a diagonal block is below eps
    psi = pc.psi_blocks(st["max"], st["sum"], ent)
    assert psi.tolist() == [[2.0, 0.0], [0.0, 2.0]]  # max 1 over mean 1/2; all-zero block -> 0
    assert pc.m_quant(st["max"], st["sum"], ent) == 1.0


def test_uniform_and_one_hot_blocks_closed_forms():
    n, b = 12, 4
    p = np.full((n, n), 1.0 / n)
    ent = pc.block_entries(n, b)
    st = pc.block_stats(p, b, 1e-3)
    assert np.all(st["cnt"] == 0) and pc.m_sparse(st["cnt"], ent, 0.9) == 0.0
    assert np.allclose(pc.psi_blocks(st["max"], st["sum"], ent), 1.0)
    st = pc.block_stats(p, b, 0.1)  # 1/12 < 0.1: every entry is "small"
    assert np.all(st["cnt"] == b * b) and pc.m_sparse(st["cnt"], ent, 0.9) == 1.0
    quarter = np.full((4, 4), 0.25)
    assert np.all(pc.block_stats(quarter, 2, 0.25)["cnt"] == 0)  # the inequality of Eq. (M_sparse) is strict
    one = np.zeros((n, n))
    one[5, 9] = 0.7  # block (1, 2)
    st = pc.block_stats(one, b, 1e-3)
    psi = pc.psi_blocks(st["max"], st["sum"], ent)
    assert psi[1, 2] == pytest.approx(b * b) and psi.sum() == pytest.approx(b * b)


def test_block_stats_against_brute_force_loops_incl_ragged_tail():
    rng = np.random.default_rng(2)
    n, b, eps, sigma = 11, 4, 0.08, 0.6
    p = rng.random((n, n)) ** 3
    p /= p.sum(axis=1, keepdims=True)
    st = pc.block_stats(p, b, eps)
    ent = pc.block_entries(n, b)
    assert ent.tolist() == [[16, 16, 12], [16, 16, 12], [12, 12, 9]]
    k = 3
    n_sparse, psi_sum = 0, 0.0
    for i, j in itertools.product(range(k), range(k)):
        cnt, tot, mx, entries = 0, 0.0, 0.0, 0
        for m, c in itertools.product(range(b), range(b)):
            r, s = i * b + m, j * b + c
            if r >= n or s >= n:
                continue
            entries += 1
            cnt += abs(p[r, s]) < eps
            tot += abs(p[r, s])
            mx = max(mx, abs(p[r, s]))
        assert entries == ent[i, j] and cnt == st["cnt"][i, j]
        assert tot == pytest.approx(st["sum"][i, j], rel=1e-14) and mx == st["max"][i, j]
        n_sparse += cnt / entries >= sigma
        psi_sum += mx / (tot / entries)
    assert pc.m_sparse(st["cnt"], ent, sigma) == pytest.approx(n_sparse / 9)
    assert pc.m_quant(st["max"], st["sum"], ent) == pytest.approx(psi_sum / 9, rel=1e-13)


def test_tie_brackets_contain_the_count():
    rng = np.random.default_rng(3)
    p = rng.random((16, 16)) * 2e-3
    st = pc.block_stats(p, 8, 1e-3, tol=0.05)
    assert np.all(st["cnt_lo"] <= st["cnt"]) and np.all(st["cnt"] <= st["cnt_hi"])
    assert (st["cnt_hi"] - st["cnt_lo"]).sum() > 0
    perturbed = pc.block_stats(p * (1 + 0.04 * np.sign(rng.standard_normal(p.shape))), 8, 1e-3)
    assert np.all(st["cnt_lo"] <= perturbed["cnt"]) and np.all(perturbed["cnt"] <= st["cnt_hi"])


@pytest.mark.parametrize("grid,T", [((2, 3, 4), 0), ((1, 4, 4), 3)])
def test_invariants_of_a_row_stochastic_map_under_the_six_orders(grid, T):
    F, H, W = grid
    n = F * H * W + T
    rng = np.random.default_rng(4)
    q = rng.standard_normal((n, 8)).astype(np.float32) * 2
    k = rng.standard_normal((n, 8)).astype(np.float32) * 2
    p = pc.attention_map(q, k)
    b, eps = 5, 0.02
    total_small = int((p < eps).sum())
    ext = np.minimum(b, n - b * np.arange(-(-n // b)))
    for pid in range(6):
        idx = po.perm_index(F, H, W, T, pid)
        st = pc.block_stats(pc.reorder_map(p, idx), b, eps)
        assert np.allclose(st["sum"].sum(axis=1), ext, atol=1e-12)  # every row of P sums to 1
        assert int(st["cnt"].sum()) == total_small                   # a reorder moves entries, it does not change them
        assert st["max"].max() == p.max()
    # the reordered map is the map of the reordered operands (rows and columns move together)
    idx = po.perm_index(F, H, W, T, 4)
    assert np.allclose(pc.reorder_map(p, idx), pc.attention_map(q[idx], k[idx]), rtol=1e-12, atol=1e-300)


def test_combined_metric_hand_numbers_and_direction():
    ms = [0.8, 0.6, 0.6, 0.6, 0.6, 0.6]
    mq = [2.0, 4.0, 4.0, 4.0, 4.0, 4.0]
    m, best = pc.combine(ms, mq, 0.5)
    assert m[0] == pytest.approx(0.5 * 0.2 / 2.2 + 0.5 * 2 / 22) and m[1] == pytest.approx(0.5 * 0.4 / 2.2 + 0.5 * 4 / 22)
    assert best == 0 and m.sum() == pytest.approx(1.0)
    # alpha = 1: only sparsity counts, and MORE sparse blocks must win (lowest metric = lowest dense share)
    assert pc.combine([0.1, 0.2, 0.9, 0.3, 0.3, 0.3], [1, 1, 9, 1, 1, 1], 1.0)[1] == 2
    # alpha = 0: only incoherence counts, lower wins
    assert pc.combine([0.1, 0.2, 0.9, 0.3, 0.3, 0.3], [5, 4, 9, 3, 6, 7], 0.0)[1] == 3
    # all equal: every order gets 1/6 and the lowest id is taken; degenerate normalisers give 0, not NaN
    m, best = pc.combine([0.5] * 6, [3.0] * 6, 0.3)
    assert np.allclose(m, 1 / 6) and best == 0
    m, best = pc.combine([1.0] * 6, [0.0] * 6, 0.5)
    assert np.all(m == 0) and best == 0


def test_mask_by_block_sum_threshold_with_density_control():
    rng = np.random.default_rng(5)
    k, k_img = 9, 7
    sums = rng.random((k, k))
    sums[2, 3] = sums[4, 1] = sums[0, 6] = 0.5  # equal sums straddling the threshold
    for density in (0.0, 0.2, 0.5, 1.0):
        mask = pc.mask_from_block_sums(sums, density, k_img)
        img = mask[:k_img, :k_img]
        n_live = int(np.rint(density * k_img * k_img))
        assert int(img.sum()) == n_live
        assert mask[k_img:, :].all() and mask[:, k_img:].all()
        if 0 < n_live < k_img * k_img:
            assert sums[:k_img, :k_img][img].min() >= sums[:k_img, :k_img][~img].max()
    # ties go to the lower i*k + j: make exactly the three equal blocks compete for two places
    s2 = np.zeros((k, k))
    s2[2, 3] = s2[4, 1] = s2[0, 6] = 0.5
    s2[1, 1] = 0.9
    mask = pc.mask_from_block_sums(s2, 3 / 49, k_img)
    assert mask[1, 1] and mask[0, 6] and mask[2, 3] and not mask[4, 1]


def test_constructed_head_prefers_the_order_that_makes_its_partners_contiguous():
    """Tokens attend to the tokens that share their (h, w) cell across frames.  With the frame axis
    fastest (orders HWF = 3 and WHF = 5) the partners are neighbours in the sequence, the map is
    block diagonal and almost every block is sparse; with the frame axis slowest the same mass is
    spread over F times as many blocks.  Both frame-fastest orders are equivalent: the lower id wins."""
    F, H, W, b = 4, 4, 4, 8
    n = F * H * W
    f, h, w = np.meshgrid(np.arange(F), np.arange(H), np.arange(W), indexing="ij")
    cell = (h * W + w).ravel()
    q = np.zeros((n, 16), np.float32)
    q[np.arange(n), cell] = 8.0
    idxs = [po.perm_index(F, H, W, 0, t) for t in range(6)]
    res = pc.calibrate_head(q, q, idxs, b, 1e-3, 0.9, 0.5, 0.25, n // b)
    assert res["perm_id"] == 3
    assert res["M"][3] == pytest.approx(res["M"][5]) and res["M"][3] < res["M"][0] - 0.02
    st3, st0 = res["orders"][3], res["orders"][0]
    k = n // b
    assert st3["m_sparse"] == pytest.approx(1 - 1 / k)      # only the diagonal blocks carry mass
    assert st0["m_sparse"] == pytest.approx(1 - F / k)      # F blocks per block row carry mass
    # each diagonal block: two cells of F tokens, each token gives ~1/F to its F partners
    assert st3["sum"][0, 0] == pytest.approx(b, rel=1e-4)
    assert int(res["mask"].sum()) == int(np.rint(0.25 * k * k)) and res["mask"].diagonal().all()
