"""The seeded input generators: shapes, determinism, mask density and structure (CPU only)."""
import numpy as np
import pytest

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl


def gather_fn(w):
    return lambda pid: po.perm_index(w.F, w.Hg, w.Wg, w.T_text, pid)


def test_named_workloads_have_the_stated_shapes():
    t, c2, c5, c4, fx = (wl.WORKLOADS[n] for n in wl.WORKLOAD_ORDER)
    assert (t.N, t.k, t.block, t.nh, t.d) == (128, 4, 32, 2, 64)
    assert (c2.N, c2.k, c2.nh, c2.density) == (17550, 275, 30, 0.5)
    assert (c5.N, c5.k, c5.npad, c5.nh, c5.density, c5.bits_pv) == (17550, 275, 17600, 48, 0.3, 8)
    assert (c4.density, c4.bits_qk, c4.bits_pv) == (0.2, 8, 4)
    assert (fx.N, fx.k, fx.d, fx.nh, fx.T_text) == (4608, 72, 128, 24, 512)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2.0**-8, 1.0 + 3 * 2.0**-8, -2.5, 3.0e-5], np.float32)
    r = wl.bf16_round(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.0 + 2.0**-6) and r[3] == -2.5
    assert np.array_equal(wl.bf16_to_f32(wl.bf16_bits(r)), r)
    t = __import__("torch")
    ref = t.from_numpy(x).to(t.bfloat16).to(t.float32).numpy()
    assert np.array_equal(r, ref)


def test_qkv_deterministic_local_and_bf16():
    w = wl.WORKLOADS["tiny"].replace(dtype="bf16")
    q1, k1, v1 = wl.make_head_qkv(w, 0, 1)
    q2, k2, v2 = wl.make_head_qkv(w, 0, 1)
    assert np.array_equal(q1, q2) and np.array_equal(v1, v2)
    assert q1.shape == (w.N, w.d) and q1.dtype == np.float32
    assert np.array_equal(wl.bf16_round(q1), q1)
    q0, _, _ = wl.make_head_qkv(w, 0, 0)
    assert not np.array_equal(q0, q1)
    # local aggregation: the logit of a token with its grid neighbour beats that with a far token on average
    logits = (q1.astype(np.float64) @ k1.astype(np.float64).T) / 8.0
    near = np.mean([logits[n, n + 1] for n in range(0, w.N - 1) if (n + 1) % w.Wg])
    far = np.mean(logits[:, ::17])
    assert near > far + 3.0


def test_text_tokens_have_no_positional_part():
    w = wl.WORKLOADS["flux"].replace(nh=1, Hg=8, Wg=8, T_text=64)
    q, k, v = wl.make_head_qkv(w, 0, 0)
    assert q.shape == (128, 128)
    assert np.var(q[64:]) < 1.2 < np.var(q[:64])


def test_perm_ids():
    assert wl.make_perm_ids(wl.WORKLOADS["tiny"]).tolist() == [0, 5]
    p = wl.make_perm_ids(wl.WORKLOADS["cogvideox5b"])
    assert p.dtype == np.uint8 and p.shape == (48,) and set(p.tolist()) == set(range(6))


@pytest.mark.parametrize("perm_id", [0, 3, 5])
def test_block_scores_equal_direct_pair_sum(perm_id):
    w = wl.Workload("t", 1, 1, 8, 3, 4, 5, 0, 8, 0.5, 8, 8, "f32", 1)
    idx = po.perm_index(w.F, w.Hg, w.Wg, 0, perm_id)
    s = wl.block_locality_scores(w, idx)
    f, h, x = np.meshgrid(np.arange(3), np.arange(4), np.arange(5), indexing="ij")
    pos = np.stack([f.ravel(), h.ravel(), x.ravel()], 1).astype(float)[idx]
    kern = np.exp(-((pos[:, None, :] - pos[None, :, :]) ** 2).sum(-1) / (2 * w.sigma**2))
    kb = -(-60 // 8)
    ref = np.array([[kern[i * 8 : (i + 1) * 8, j * 8 : (j + 1) * 8].sum() for j in range(kb)] for i in range(kb)])
    assert np.allclose(s, ref, rtol=1e-12)


def test_masks_density_diagonal_and_determinism():
    w = wl.WORKLOADS["tiny"]
    m = wl.make_block_masks(w, gather_fn(w))
    assert m.shape == (2, 4, 4) and m.dtype == bool
    assert np.all(m[:, np.arange(4), np.arange(4)])
    assert np.all(m.reshape(2, -1).sum(1) == 8)  # density 0.5 of 16 blocks
    assert np.array_equal(m, wl.make_block_masks(w, gather_fn(w)))
    bits = wl.pack_bitmask(m)
    assert bits.shape == (2, 2) and bits.dtype == np.uint8
    rp, ci = po.mask_to_blocklist(bits, 2, 4)
    assert ci.size == 16 == wl.live_blocks(m)


def test_masks_with_text_blocks_are_dense_on_text():
    w = wl.WORKLOADS["flux"].replace(nh=2, Hg=16, Wg=16, T_text=128)
    m = wl.make_block_masks(w, gather_fn(w))
    k_img = 4
    assert m.shape == (2, 6, 6)
    assert np.all(m[:, k_img:, :]) and np.all(m[:, :, k_img:])
    assert np.all(m[:, :k_img, :k_img].reshape(2, -1).sum(1) == max(k_img, round(0.3 * 16)))


def test_headline_mask_has_the_stated_live_count():
    w = wl.WORKLOADS["cogvideox5b"].replace(nh=2)
    m = wl.make_block_masks(w, gather_fn(w), perm_ids=np.array([3, 0], np.uint8))
    assert m.shape == (2, 275, 275)
    assert np.all(m.reshape(2, -1).sum(1) == 22688)  # rint(0.3 * 275^2)
    assert np.all(m[:, np.arange(275), np.arange(275)])
    rows = m[0].sum(1)
    assert rows.min() >= 1 and rows.max() > rows.min()  # one threshold per head -> unequal rows
