"""The C-ABI library loads, exports every declared symbol, and its host-only entry points agree
with the oracle bit for bit (CPU only: nothing here launches a kernel)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import paro_oracle as po
from paper_2506_16054_amd import binding as pb
from paper_2506_16054_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "paro.h")).read()
    declared = set(re.findall(r"\b(paro_[a-z_0-9]+)\s*\(", header))
    assert declared == set(pb.EXPORTS)
    L = pb.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert pb.paro_version() >= 1


def test_shape_arithmetic_and_rejection():
    s = pb.make_shape(1, 48, 64, 13, 30, 45, 0, 64)
    assert (pb.paro_ntokens(s), pb.paro_nblocks(s), pb.paro_npad(s)) == (17550, 275, 17600)
    s = pb.make_shape(1, 24, 128, 1, 64, 64, 512, 64)
    assert (pb.paro_ntokens(s), pb.paro_nblocks(s)) == (4608, 72)
    for bad in (pb.make_shape(1, 2, 48, 2, 2, 2, 0, 64), pb.make_shape(1, 2, 64, 2, 2, 2, 0, 16),
                pb.make_shape(0, 2, 64, 2, 2, 2, 0, 64), pb.make_shape(1, 2, 64, 0, 2, 2, 0, 64),
                pb.make_shape(1, 2, 64, 2, 2, 2, -1, 64), pb.make_shape(1, 300, 64, 2, 2, 2, 0, 64)):
        with pytest.raises(pb.ParoError) as e:
            pb.paro_ntokens(bad)
        assert e.value.status in (pb.PARO_EINVAL, pb.PARO_EUNSUPPORTED)
    assert pb.lib().paro_ntokens(None) == pb.PARO_EINVAL
    assert pb.lib().paro_strerror(pb.PARO_EINVAL) == b"invalid argument"


@pytest.mark.parametrize("grid,T", [((2, 8, 8), 0), ((3, 4, 5), 7), ((1, 6, 7), 0), ((13, 30, 45), 0), ((1, 64, 64), 512)])
def test_perm_index_matches_oracle_bit_exactly(grid, T):
    F, H, W = grid
    s = pb.make_shape(1, 1, 64, F, H, W, T, 64)
    for pid in range(6):
        got = pb.paro_perm_index(s, pid)
        assert got.dtype == np.int32
        assert np.array_equal(got, po.perm_index(F, H, W, T, pid))
    with pytest.raises(pb.ParoError):
        pb.paro_perm_index(s, 6)
    with pytest.raises(pb.ParoError):
        pb.paro_perm_index(s, -1)


@pytest.mark.parametrize("block", [32, 64])
def test_vt_slot_is_the_documented_bijection(block):
    slots = [pb.paro_vt_slot(block, i) for i in range(block)]
    assert sorted(slots) == list(range(block))
    for i in range(block):
        # token i = 32*T + 8*q + 4*g + p  ->  slot 32*T + 16*g + 4*q + p
        T, q, g, p = i // 32, (i % 32) // 8, (i % 8) // 4, i % 4
        assert slots[i] == 32 * T + 16 * g + 4 * q + p
    for bad in (-1, block):
        with pytest.raises(pb.ParoError):
            pb.paro_vt_slot(block, bad)
    with pytest.raises(pb.ParoError):
        pb.paro_vt_slot(48, 0)


@pytest.mark.parametrize("nh,k", [(1, 1), (3, 4), (2, 11), (2, 275)])
def test_blocklist_matches_oracle_bit_exactly(nh, k):
    rng = np.random.default_rng(k)
    m = rng.random((nh, k, k)) < 0.3
    if nh > 1:
        m[1, k // 2] = False  # an empty row
    bits = np.packbits(m.reshape(nh, -1), axis=1, bitorder="little")
    rp, ci = pb.paro_mask_to_blocklist(nh, k, bits)
    rp_o, ci_o = po.mask_to_blocklist(bits, nh, k)
    assert rp.dtype == np.int32 and ci.dtype == np.int32
    assert np.array_equal(rp, rp_o) and np.array_equal(ci, ci_o)


def test_blocklist_capacity_and_null_handling():
    L = pb.lib()
    bits = np.array([[0xFF, 0x01]], np.uint8)  # k = 3, all 9 blocks live
    rp = np.zeros(4, np.int32)
    ci = np.zeros(4, np.int32)
    nnz = ctypes.c_int64(-1)
    st = L.paro_mask_to_blocklist(1, 3, bits.ctypes.data, rp.ctypes.data, ci.ctypes.data, 4, ctypes.byref(nnz))
    assert st == pb.PARO_EINVAL and nnz.value == 9
    assert b"live blocks" in L.paro_last_error()
    assert L.paro_mask_to_blocklist(1, 3, None, rp.ctypes.data, ci.ctypes.data, 4, ctypes.byref(nnz)) == pb.PARO_EINVAL
    assert L.paro_mask_to_blocklist(1, 0, bits.ctypes.data, rp.ctypes.data, ci.ctypes.data, 4, ctypes.byref(nnz)) == pb.PARO_EINVAL
    assert L.paro_mask_to_blocklist(1, 3, bits.ctypes.data, rp.ctypes.data, None, 4, ctypes.byref(nnz)) == pb.PARO_EINVAL


def test_device_entry_points_reject_bad_arguments_before_launch():
    # Host-side validation only: every call below must fail before any HIP call is made.
    L = pb.lib()
    s = pb.make_shape(1, 2, 64, 2, 8, 8, 0, 32)
    perm = np.array([0, 9], np.uint8)
    fake = ctypes.c_void_p(0x1000)
    assert L.paro_permute(ctypes.byref(s), pb.PARO_F32, perm.ctypes.data, fake, ctypes.c_void_p(0x2000), None) == pb.PARO_EINVAL
    assert b"perm_ids[1]" in L.paro_last_error()
    ok = np.array([0, 5], np.uint8)
    assert L.paro_permute(ctypes.byref(s), pb.PARO_F32, ok.ctypes.data, None, fake, None) == pb.PARO_EINVAL
    assert L.paro_permute(ctypes.byref(s), pb.PARO_F32, ok.ctypes.data, fake, fake, None) == pb.PARO_EINVAL
    assert L.paro_permute(ctypes.byref(s), 7, ok.ctypes.data, fake, ctypes.c_void_p(0x2000), None) == pb.PARO_EINVAL
    assert L.paro_unpermute(ctypes.byref(s), pb.PARO_F32, ok.ctypes.data, fake, ctypes.c_void_p(0x2004), None) == pb.PARO_EINVAL
    assert L.paro_quantize(ctypes.byref(s), pb.PARO_F32, 5, pb.PARO_ROWS, fake, ctypes.c_void_p(0x2000), fake, None) == pb.PARO_EINVAL
    assert L.paro_quantize(ctypes.byref(s), pb.PARO_F32, 8, 3, fake, ctypes.c_void_p(0x2000), fake, None) == pb.PARO_EINVAL
    assert L.paro_quantize(ctypes.byref(s), pb.PARO_F32, 8, pb.PARO_VT, fake, None, fake, None) == pb.PARO_EINVAL
    args = [fake, fake, fake, fake, fake, fake, fake, fake]
    assert L.paro_sparse_attn(ctypes.byref(s), 5, 8, *args, 4, None, pb.PARO_F32, fake, None) == pb.PARO_EINVAL
    assert L.paro_sparse_attn(ctypes.byref(s), 8, 16, *args, 4, None, pb.PARO_F32, fake, None) == pb.PARO_EUNSUPPORTED
    assert L.paro_sparse_attn(ctypes.byref(s), 8, 8, *args, -1, None, pb.PARO_F32, fake, None) == pb.PARO_EINVAL
    assert L.paro_sparse_attn(ctypes.byref(s), 8, 8, fake, None, fake, fake, fake, fake, fake, fake, 4, None, pb.PARO_F32, fake, None) == pb.PARO_EINVAL
    assert L.paro_sparse_attn(ctypes.byref(s), 8, 8, *args, 4, None, 5, fake, None) == pb.PARO_EINVAL
    # attention with in-kernel Q quantization: block 64 and 8-bit QK only
    b64 = pb.make_shape(1, 2, 64, 2, 8, 8, 0, 64)
    rq = [fake, fake, fake, fake, fake, fake, fake]
    assert L.paro_sparse_attn_unpermuted_rawq(ctypes.byref(s), pb.PARO_F32, 8, *rq, 4, None, ok.ctypes.data, pb.PARO_F32, fake, None) == pb.PARO_EUNSUPPORTED
    assert L.paro_sparse_attn_unpermuted_rawq(ctypes.byref(b64), pb.PARO_F32, 16, *rq, 4, None, ok.ctypes.data, pb.PARO_F32, fake, None) == pb.PARO_EUNSUPPORTED
    assert L.paro_sparse_attn_unpermuted_rawq(ctypes.byref(b64), 9, 8, *rq, 4, None, ok.ctypes.data, pb.PARO_F32, fake, None) == pb.PARO_EINVAL
    assert L.paro_sparse_attn_unpermuted_rawq(ctypes.byref(b64), pb.PARO_F32, 8, *rq, 4, None, None, pb.PARO_F32, fake, None) == pb.PARO_EINVAL
    assert L.paro_sparse_attn_unpermuted_rawq(ctypes.byref(b64), pb.PARO_F32, 8, fake, fake, None, fake, fake, fake, fake, 4, None, ok.ctypes.data, pb.PARO_F32, fake, None) == pb.PARO_EINVAL
    # device-side mask expansion
    assert L.paro_mask_to_blocklist_device(0, 4, fake, fake, fake, 16, None, None) == pb.PARO_EINVAL
    assert L.paro_mask_to_blocklist_device(2, 0, fake, fake, fake, 16, None, None) == pb.PARO_EINVAL
    assert L.paro_mask_to_blocklist_device(2, 4, None, fake, fake, 16, None, None) == pb.PARO_EINVAL
    assert L.paro_mask_to_blocklist_device(2, 4, fake, fake, None, 16, None, None) == pb.PARO_EINVAL
    assert L.paro_mask_to_blocklist_device(2, 4, fake, fake, fake, -1, None, None) == pb.PARO_EINVAL
    assert L.paro_mask_to_blocklist_device(200, 30000, fake, fake, fake, 16, None, None) == pb.PARO_EINVAL
    assert L.paro_blocklist_cols_device(2, 4, fake, fake, None, 16, None) == pb.PARO_EINVAL
    assert L.paro_blocklist_cols_device(2, 4, fake, None, fake, 16, None) == pb.PARO_EINVAL
    assert L.paro_blocklist_cols_device(2, 4, fake, fake, fake, 0, None) == pb.PARO_EINVAL
    assert L.paro_blocklist_cols_device(0, 4, fake, fake, fake, 16, None) == pb.PARO_EINVAL
    # offline calibration
    f = ctypes.c_float
    assert L.paro_calib_block_stats(ctypes.byref(s), fake, fake, f(0.0), fake, fake, fake, None) == pb.PARO_EINVAL
    assert L.paro_calib_block_stats(ctypes.byref(s), None, fake, f(1e-3), fake, fake, fake, None) == pb.PARO_EINVAL
    assert L.paro_calib_block_stats(ctypes.byref(s), ctypes.c_void_p(0x1008), fake, f(1e-3), fake, fake, fake, None) == pb.PARO_EINVAL
    assert L.paro_calib_metrics(ctypes.byref(s), fake, fake, fake, f(1.5), fake, fake, None) == pb.PARO_EINVAL
    assert L.paro_calib_metrics(ctypes.byref(s), fake, fake, None, f(0.9), fake, fake, None) == pb.PARO_EINVAL
    assert L.paro_calib_choose(0, fake, fake, f(0.5), fake, fake, None) == pb.PARO_EINVAL
    assert L.paro_calib_choose(4, fake, fake, f(-0.1), fake, fake, None) == pb.PARO_EINVAL
    assert L.paro_calib_choose(4, fake, None, f(0.5), fake, fake, None) == pb.PARO_EINVAL
    assert L.paro_calib_mask(ctypes.byref(s), fake, f(1.2), fake, None) == pb.PARO_EINVAL
    assert L.paro_calib_mask(ctypes.byref(s), None, f(0.3), fake, None) == pb.PARO_EINVAL
    ragged_text = pb.make_shape(1, 2, 64, 1, 5, 5, 8, 32)  # 25 image tokens do not fill whole blocks before the text
    assert L.paro_calib_mask(ctypes.byref(ragged_text), fake, f(0.3), fake, None) == pb.PARO_EUNSUPPORTED
    huge = pb.make_shape(1, 1, 64, 40, 32, 32, 0, 64)  # k = 640: k*k exceeds the mask kernel's LDS bit array
    assert L.paro_calib_mask(ctypes.byref(huge), fake, f(0.3), fake, None) == pb.PARO_EUNSUPPORTED


def test_fused_entry_points_validate_on_the_host():
    L = pb.lib()
    s = pb.make_shape(1, 2, 64, 2, 8, 8, 0, 32)
    fake = ctypes.c_void_p(0x1000)
    ok = np.array([0, 5], np.uint8)
    bad = np.array([0, 7], np.uint8)
    assert L.paro_permute_quantize(ctypes.byref(s), pb.PARO_F32, 8, pb.PARO_ROWS, None, fake, ctypes.c_void_p(0x2000), fake, None) == pb.PARO_EINVAL
    assert L.paro_permute_quantize(ctypes.byref(s), pb.PARO_F32, 8, pb.PARO_ROWS, bad.ctypes.data, fake, ctypes.c_void_p(0x2000), fake, None) == pb.PARO_EINVAL
    assert L.paro_permute_quantize(ctypes.byref(s), pb.PARO_F32, 3, pb.PARO_ROWS, ok.ctypes.data, fake, ctypes.c_void_p(0x2000), fake, None) == pb.PARO_EINVAL
    # the one-launch form of the three quantizer calls
    ptr = lambda a: ctypes.c_void_p(a)
    ins = [ptr(0x1000), ptr(0x2000), ptr(0x3000)]
    outs = [ptr(0x4000), fake, ptr(0x5000), fake, ptr(0x6000), fake]  # codes, scales alternating
    qkv = lambda bits_qk, bits_pv, perm, i, o, dt=pb.PARO_F32: L.paro_permute_quantize_qkv(ctypes.byref(s), dt, bits_qk, bits_pv, perm, *i, *o, None)
    assert qkv(8, 8, None, ins, outs) == pb.PARO_EINVAL                       # no perm_ids
    assert qkv(8, 8, bad.ctypes.data, ins, outs) == pb.PARO_EINVAL            # perm id out of range
    assert qkv(8, 16, ok.ctypes.data, ins, outs) == pb.PARO_EINVAL            # unsupported pair of widths
    assert qkv(3, 8, ok.ctypes.data, ins, outs) == pb.PARO_EINVAL
    assert qkv(8, 8, ok.ctypes.data, ins, outs, 7) == pb.PARO_EINVAL          # dtype
    assert qkv(8, 8, ok.ctypes.data, [ptr(0x1000), None, ptr(0x3000)], outs) == pb.PARO_EINVAL
    assert qkv(8, 8, ok.ctypes.data, [ptr(0x1004), ptr(0x2000), ptr(0x3000)], outs) == pb.PARO_EINVAL  # alignment
    assert qkv(8, 8, ok.ctypes.data, ins, [ptr(0x1000), fake, ptr(0x5000), fake, ptr(0x6000), fake]) == pb.PARO_EINVAL  # output aliases an input
    assert qkv(8, 8, ok.ctypes.data, ins, [ptr(0x4000), fake, ptr(0x4000), fake, ptr(0x6000), fake]) == pb.PARO_EINVAL  # two outputs alias
    assert b"alias" in L.paro_last_error()
    args = [fake] * 8
    assert L.paro_sparse_attn_unpermuted(ctypes.byref(s), 8, 8, *args, 4, None, None, pb.PARO_F32, fake, None) == pb.PARO_EINVAL
    assert L.paro_sparse_attn_unpermuted(ctypes.byref(s), 8, 8, *args, 4, None, bad.ctypes.data, pb.PARO_F32, fake, None) == pb.PARO_EINVAL


def test_k_smoothing_entry_points_validate_on_the_host():
    L = pb.lib()
    s = pb.make_shape(1, 2, 64, 2, 8, 8, 0, 32)
    fake, other = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000)
    ok = np.array([0, 5], np.uint8)
    bad = np.array([0, 7], np.uint8)
    assert L.paro_k_channel_mean(ctypes.byref(s), pb.PARO_F32, None, fake, None) == pb.PARO_EINVAL
    assert L.paro_k_channel_mean(ctypes.byref(s), pb.PARO_F32, fake, None, None) == pb.PARO_EINVAL
    assert L.paro_k_channel_mean(ctypes.byref(s), 5, fake, other, None) == pb.PARO_EINVAL
    assert L.paro_k_channel_mean(ctypes.byref(s), pb.PARO_F32, ctypes.c_void_p(0x1008), other, None) == pb.PARO_EINVAL
    sm = lambda dt, bits, perm, k, mean, codes, scales: L.paro_permute_quantize_smoothed(ctypes.byref(s), dt, bits, perm, k, mean, codes, scales, None)
    assert sm(pb.PARO_F32, 8, None, fake, fake, other, fake) == pb.PARO_EINVAL               # no perm_ids
    assert sm(pb.PARO_F32, 8, bad.ctypes.data, fake, fake, other, fake) == pb.PARO_EINVAL    # perm id out of range
    assert sm(pb.PARO_F32, 16, ok.ctypes.data, fake, fake, other, fake) == pb.PARO_EINVAL    # integer codes only
    assert sm(pb.PARO_F32, 8, ok.ctypes.data, fake, None, other, fake) == pb.PARO_EINVAL     # no mean
    assert sm(pb.PARO_F32, 8, ok.ctypes.data, fake, fake, fake, fake) == pb.PARO_EINVAL      # codes alias the input
    assert sm(9, 8, ok.ctypes.data, fake, fake, other, fake) == pb.PARO_EINVAL


def _check_grouped_range(chunk, lv, groups, tail):
    """One XCD's range with several L2 groups: the last `tail` positions hold the lightest row blocks of the whole
    range, heaviest first; in front of them the groups follow each other, each heaviest first."""
    main, back = slice(0, len(chunk) - tail), slice(len(chunk) - tail, None)
    assert lv[back].max() <= lv[main].min()  # nothing lighter was left in the groups
    assert np.all(np.diff(lv[back]) <= 0)
    assert np.all(np.diff(groups[main]) >= 0)
    for gidx in np.unique(groups[main]):
        assert np.all(np.diff(lv[main][groups[main] == gidx]) <= 0)


def test_row_schedule_is_a_permutation_heaviest_first_within_l2_groups_lightest_rows_last():
    rng = np.random.default_rng(5)
    # headline shape: one head's K+V (2.25 MB) fills the L2 budget alone -> groups of one head; the kernel of this
    # shape keeps 256 workgroups on an XCD, so the 128 lightest row blocks of each XCD's range start last
    s = pb.make_shape(1, 48, 64, 13, 30, 45, 0, 64)
    k = 275
    live = rng.integers(1, 120, size=(48, k))
    rp = np.zeros((48, k + 1), np.int32)
    rp[:, 1:] = np.cumsum(live, axis=1)
    rp += np.concatenate([[0], np.cumsum(live.sum(1))[:-1]])[:, None].astype(np.int32)
    order = pb.paro_schedule_rows(s, 8, 8, rp)
    total = 48 * k
    assert order.dtype == np.int32 and np.array_equal(np.sort(order), np.arange(total))
    per_xcd = (total + 7) // 8
    for x in range(8):
        chunk = order[x * per_xcd:(x + 1) * per_xcd]
        assert len(set(chunk // k)) == 6 and np.all(np.bincount(chunk // k)[np.unique(chunk // k)] == k)  # six whole heads
        _check_grouped_range(chunk, live[chunk // k, chunk % k], chunk // k, 128)
    # Flux shape: 1.18 MB per head; an XCD's whole range (three heads, 3.5 MB) fits the L2, so it
    # is sorted as one group and every long row starts first
    s2 = pb.make_shape(1, 24, 128, 1, 64, 64, 512, 64)
    k2 = 72
    live2 = rng.integers(1, 73, size=(24, k2))
    rp2 = np.zeros((24, k2 + 1), np.int32)
    rp2[:, 1:] = np.cumsum(live2, axis=1)
    order2 = pb.paro_schedule_rows(s2, 8, 8, rp2)
    assert np.array_equal(np.sort(order2), np.arange(24 * k2))
    for x in range(8):
        chunk = order2[x * 3 * k2:(x + 1) * 3 * k2]
        assert len(set(chunk // k2)) == 3  # three whole heads (which ones: see the test of unequal heads)
        assert np.all(np.diff(live2[chunk // k2, chunk % k2]) <= 0)
    # 20 heads of the same size: XCD ranges of 2.5 heads touch 3 heads each and are one group
    s3 = pb.make_shape(1, 20, 128, 1, 64, 64, 512, 64)
    live3 = rng.integers(1, 73, size=(20, k2))
    rp3 = np.zeros((20, k2 + 1), np.int32)
    rp3[:, 1:] = np.cumsum(live3, axis=1)
    order3 = pb.paro_schedule_rows(s3, 8, 8, rp3)
    assert np.array_equal(np.sort(order3), np.arange(20 * k2))
    per3 = 20 * k2 // 8
    for x in range(8):
        lo, hi = x * per3, (x + 1) * per3
        chunk = order3[lo:hi]
        assert np.array_equal(np.sort(chunk), np.arange(lo, hi))
        assert np.all(np.diff(live3[chunk // k2, chunk % k2]) <= 0)
    # a long d = 128 layer: 4.5 MB of K+V per head, one head per group, three heads per XCD; the kernels of this shape
    # keep 128 workgroups on an XCD -> 64 row blocks kept back; 4-bit codes (2.25 MB per head) and bf16 (9 MB) also give
    # groups of one head
    s4 = pb.make_shape(1, 24, 128, 13, 30, 45, 0, 64)
    live4 = rng.integers(1, 200, size=(24, k))
    rp4 = np.zeros((24, k + 1), np.int32)
    rp4[:, 1:] = np.cumsum(live4, axis=1)
    for bits, heads_per_group in ((8, 1), (4, 1), (16, 1)):
        order4 = pb.paro_schedule_rows(s4, bits, bits, rp4)
        assert np.array_equal(np.sort(order4), np.arange(24 * k))
        for x in range(8):
            chunk = order4[x * 3 * k:(x + 1) * 3 * k]
            assert len(set(chunk // k)) == 3
            _check_grouped_range(chunk, live4[chunk // k, chunk % k], (chunk // k) // heads_per_group, 64)
    # a two-row-block problem: ranges of one row block, nothing to keep back
    s5 = pb.make_shape(1, 2, 64, 1, 8, 16, 0, 64)
    assert np.array_equal(pb.paro_schedule_rows(s5, 8, 8, np.array([[0, 1, 3], [3, 5, 6]], np.int32)), np.arange(4))
    with pytest.raises(pb.ParoError):
        pb.paro_schedule_rows(s2, 5, 8, rp2)


def test_row_schedule_deals_unequal_heads_to_the_xcds_by_work():
    """Heads of equal size stay where they are (XCD x works on heads 6x .. 6x+5); heads that differ in live blocks are
    dealt so that no XCD carries much more than its share."""
    k = 275
    s = pb.make_shape(1, 48, 64, 13, 30, 45, 0, 64)

    def row_ptr_of(live):
        rp = np.zeros((48, k + 1), np.int64)
        rp[:, 1:] = np.cumsum(live, axis=1)
        rp += np.concatenate([[0], np.cumsum(live.sum(1))[:-1]])[:, None]
        return rp.astype(np.int32)

    def xcd_loads(order, live):
        return np.array([live[c // k, c % k].sum() for c in np.split(order, 8)])

    rng = np.random.default_rng(11)
    equal = np.stack([rng.permutation(np.arange(1, k + 1) % 120 + 1) for _ in range(48)])  # every head: the same multiset
    order = pb.paro_schedule_rows(s, 8, 8, row_ptr_of(equal))
    for x, chunk in enumerate(np.split(order, 8)):
        assert set(chunk // k) == set(range(6 * x, 6 * x + 6))
    # per-head density between 0.1 and 0.5, heaviest heads first: in natural order XCD 0 would carry 1.6x the mean
    dens = np.linspace(0.5, 0.1, 48)
    uneq = np.stack([rng.binomial(k, dv, size=k).clip(1) for dv in dens])
    natural = np.array([uneq[6 * x:6 * x + 6].sum() for x in range(8)])
    assert natural.max() > 1.5 * natural.mean()
    order = pb.paro_schedule_rows(s, 8, 8, row_ptr_of(uneq))
    assert np.array_equal(np.sort(order), np.arange(48 * k))
    for chunk in np.split(order, 8):
        heads = np.unique(chunk // k)
        assert len(heads) == 6 and np.all(np.bincount(chunk // k)[heads] == k)  # whole heads only
    loads = xcd_loads(order, uneq)
    assert loads.sum() == uneq.sum() and loads.max() <= 1.03 * loads.mean()
    pb.paro_check_row_order(s, order)


def test_blocklist_and_launch_order_validators():
    """Lists the library makes pass; each way a caller-made list can break the kernels' assumptions is named."""
    w = wl.Workload("chk", 1, 2, 64, 2, 6, 8, 0, 32, 0.5, 8, 8, "f32", 5, perm_choice=(0, 3))
    s = pb.shape_of(w)
    masks = wl.make_block_masks(w, lambda pid: pb.paro_perm_index(s, pid), wl.make_perm_ids(w))
    row_ptr, col_idx = pb.paro_mask_to_blocklist(w.nh, w.k, wl.pack_bitmask(masks))
    pb.paro_check_blocklist(w.nh, w.k, row_ptr, col_idx)
    order = pb.paro_schedule_rows(s, 8, 8, row_ptr)
    pb.paro_check_row_order(s, order)

    def rejected(fn, *a):
        with pytest.raises(pb.ParoError) as e:
            fn(*a)
        assert e.value.status == pb.PARO_EINVAL
        return str(e.value)

    row = next(i for i in range(w.k) if row_ptr[0, i + 1] - row_ptr[0, i] >= 2)
    beg = int(row_ptr[0, row])
    swapped = col_idx.copy()
    swapped[beg], swapped[beg + 1] = col_idx[beg + 1], col_idx[beg]
    assert "not strictly ascending" in rejected(pb.paro_check_blocklist, w.nh, w.k, row_ptr, swapped)
    dup = col_idx.copy()
    dup[beg + 1] = dup[beg]
    assert "not strictly ascending" in rejected(pb.paro_check_blocklist, w.nh, w.k, row_ptr, dup)
    far = col_idx.copy()
    far[beg] = w.k
    assert "outside" in rejected(pb.paro_check_blocklist, w.nh, w.k, row_ptr, far)
    bad_ptr = row_ptr.copy()
    bad_ptr[1, 2] = bad_ptr[1, 3] + 1
    assert "ascending range" in rejected(pb.paro_check_blocklist, w.nh, w.k, bad_ptr, col_idx)
    assert "ascending range" in rejected(pb.paro_check_blocklist, w.nh, w.k, row_ptr, col_idx[:-1])
    twice = order.copy()
    twice[3] = twice[4]
    assert "appears twice" in rejected(pb.paro_check_row_order, s, twice)
    out = order.copy()
    out[0] = order.size
    assert "outside" in rejected(pb.paro_check_row_order, s, out)


def test_row_schedule_shortens_the_simulated_drain_of_the_headline_launch():
    """What the launch order is for: on the headline masks, list scheduling onto the 256 wavefront slots of an XCD at a
    constant pace per block (which is how the one-wavefront kernel behaves: a wavefront is no faster alone) ends earlier
    with the library's order than with every head's rows simply heaviest first."""
    import heapq

    w = wl.WORKLOADS["cogvideox5b"]
    s = pb.shape_of(w)
    masks = wl.make_block_masks(w, lambda pid: pb.paro_perm_index(s, pid), wl.make_perm_ids(w))
    row_ptr, _ = pb.paro_mask_to_blocklist(w.nh, w.k, wl.pack_bitmask(masks))
    live = masks.sum(2)
    order = pb.paro_schedule_rows(s, w.bits_qk, w.bits_pv, row_ptr)

    def makespan(chunk):
        slots = [0.0] * 256
        heapq.heapify(slots)
        for item in chunk:
            heapq.heappush(slots, heapq.heappop(slots) + live[item // w.k, item % w.k] + 1.0)  # + a block's worth of set-up
        return max(slots)

    per_head = np.concatenate([h * w.k + np.argsort(-live[h], kind="stable") for h in range(w.nh)])
    new = max(makespan(c) for c in np.split(order, 8))
    old = max(makespan(c) for c in np.split(per_head, 8))
    ideal = (live.sum() + live.size) / 2048.0
    assert new < 0.985 * old, (new, old)
    assert new < 1.06 * ideal, (new, ideal)
