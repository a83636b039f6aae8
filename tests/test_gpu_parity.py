"""GPU parity: every step of the HIP path, called through the C ABI, against the CPU oracle on
identical seeded inputs.  Integer work (gather rows, codes, scales, block lists) must match bit
for bit; attention outputs within max-abs 2e-2 and relative-L2 1e-2 (the stated bar)."""
import numpy as np
import pytest

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl
from tests.helpers import (assert_equal_up_to_output_rounding, blocklist_for, check_attention, gather_fn, oracle_head,
                           same_attention_kernel_for_raw_q)

pytestmark = pytest.mark.gpu

MAX_ABS = 2e-2
REL_L2 = 1e-2


def _torch():
    import torch

    return torch


def _pb():
    from paper_2506_16054_amd import binding as pb

    return pb


def to_dev(x, dtype):
    torch = _torch()
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def tdtype(name):
    torch = _torch()
    return torch.bfloat16 if name == "bf16" else torch.float32


def host(t):
    return t.float().cpu().numpy() if t.dtype == _torch().bfloat16 else t.cpu().numpy()


def vt_to_rows(vt, block):
    """[k, d, block] in slot order -> [k*block, d] in token order (the documented PARO_VT map)."""
    pb = _pb()
    slots = np.array([pb.paro_vt_slot(block, i) for i in range(block)])
    k, d, _ = vt.shape
    return vt[:, :, slots].transpose(0, 2, 1).reshape(k * block, d)


def unpack_vt_int4(b):
    """bytes [k, d, block/2] -> int codes [k, d, block] in slot order: byte 4g+t holds slot 8g+t in
    bits 0-3 and slot 8g+4+t in bits 4-7."""
    u = b.astype(np.uint8)
    k, d, half = u.shape
    out = np.zeros((k, d, half * 2), np.int32)
    for t4 in range(half):
        g, t = divmod(t4, 4)
        out[:, :, 8 * g + t] = ((u[:, :, t4] & 0xF).astype(np.int32) ^ 8) - 8
        out[:, :, 8 * g + 4 + t] = ((u[:, :, t4] >> 4).astype(np.int32) ^ 8) - 8
    return out


def unpack_rows_int4(b):
    u = b.astype(np.uint8)
    out = np.zeros(u.shape[:-1] + (u.shape[-1] * 2,), np.int32)
    out[..., 0::2] = ((u & 0xF).astype(np.int32) ^ 8) - 8
    out[..., 1::2] = ((u >> 4).astype(np.int32) ^ 8) - 8
    return out


SMALL = {
    # several 64-blocks, ragged tail (780 = 12*64 + 12), three heads with different orders
    "video64": wl.Workload("video64", 1, 3, 64, 5, 12, 13, 0, 64, 0.4, 8, 8, "bf16", 11, perm_choice=(3, 0, 5)),
    "video64_int4": wl.Workload("video64_int4", 1, 2, 64, 5, 12, 13, 0, 64, 0.4, 8, 4, "bf16", 12, perm_choice=(1, 4)),
    "video32_f32": wl.Workload("video32_f32", 2, 2, 64, 3, 7, 9, 0, 32, 0.5, 8, 8, "f32", 13, perm_choice=(2, 5)),
    "flux128": wl.Workload("flux128", 1, 2, 128, 1, 16, 16, 64, 64, 0.3, 8, 8, "bf16", 14, perm_choice=(0, 5)),
    "flux128_b32_int4": wl.Workload("flux128_b32_int4", 1, 2, 128, 1, 8, 12, 32, 32, 0.5, 8, 4, "f32", 15, perm_choice=(5, 0)),
    "tiny": wl.WORKLOADS["tiny"],
    # bf16 unquantized block-sparse mode
    "video64_bf16": wl.Workload("video64_bf16", 1, 2, 64, 5, 12, 13, 0, 64, 0.4, 16, 16, "bf16", 16, perm_choice=(3, 5)),
    "flux128_bf16": wl.Workload("flux128_bf16", 1, 2, 128, 1, 16, 16, 64, 64, 0.3, 16, 16, "bf16", 17, perm_choice=(0, 5)),
    "video32_bf16_f32io": wl.Workload("video32_bf16_f32io", 1, 2, 64, 3, 7, 9, 0, 32, 0.5, 16, 16, "f32", 18, perm_choice=(2, 4)),
    "flux128_b32_bf16": wl.Workload("flux128_b32_bf16", 1, 1, 128, 1, 8, 12, 32, 32, 0.5, 16, 16, "bf16", 19, perm_choice=(5,)),
}
# INT4 QK^T (the paper's all-INT4 setting) and the mixed INT4 QK / INT8 PV
SMALL["video64_i4i4"] = wl.Workload("video64_i4i4", 1, 2, 64, 5, 12, 13, 0, 64, 0.4, 4, 4, "bf16", 20, perm_choice=(3, 0))
SMALL["video64_i4i8_f32"] = wl.Workload("video64_i4i8_f32", 1, 2, 64, 5, 12, 13, 0, 64, 0.4, 4, 8, "f32", 23, perm_choice=(4, 1))
SMALL["flux128_i4i8_f32"] = wl.Workload("flux128_i4i8_f32", 1, 2, 128, 1, 16, 16, 64, 64, 0.3, 4, 8, "f32", 21, perm_choice=(0, 5))
SMALL["video32_i4i4_f32"] = wl.Workload("video32_i4i4_f32", 1, 2, 64, 3, 7, 9, 0, 32, 0.5, 4, 4, "f32", 22, perm_choice=(2, 5))
REL_L2_BF16 = 5e-3  # stated bar of the unquantized mode


class Problem:
    """Inputs, oracle results and GPU results of one small workload."""

    def __init__(self, w):
        torch, pb = _torch(), _pb()
        from paper_2506_16054_amd.pipeline import ParoAttention

        self.w = w
        self.perm_ids = wl.make_perm_ids(w)
        self.masks = wl.make_block_masks(w, gather_fn(w), self.perm_ids)
        self.bits, self.row_ptr, self.col_idx = blocklist_for(w, self.masks)
        self.q, self.k, self.v = wl.make_qkv(w)
        self.oracle = [[oracle_head(w, self.q[b, h], self.k[b, h], self.v[b, h], self.perm_ids[h], self.row_ptr[h], self.col_idx)
                        for h in range(w.nh)] for b in range(w.B)]
        self.s = pb.shape_of(w)
        self.pa = ParoAttention(self.s, self.perm_ids, self.bits, w.bits_qk, w.bits_pv, tdtype(w.dtype))
        self.dq, self.dk, self.dv = (to_dev(x, w.dtype) for x in (self.q, self.k, self.v))
        # poison the outputs so that untouched elements are noticed
        for t in self.pa.xp + [self.pa.op, self.pa.o]:
            t.fill_(float("nan"))
        self.o = self.pa.run(self.dq, self.dk, self.dv)
        torch.cuda.synchronize()


_cache = {}


def problem(name):
    if name not in _cache:
        _cache[name] = Problem(SMALL[name])
    return _cache[name]


ALL = list(SMALL)


@pytest.mark.parametrize("name", ALL)
def test_blocklist_bit_exact(name):
    p = problem(name)
    assert np.array_equal(p.pa.h_row_ptr, p.row_ptr)
    assert np.array_equal(p.pa.h_col_idx, p.col_idx)


@pytest.mark.parametrize("name", ALL)
def test_permute_bit_exact(name):
    p = problem(name)
    w = p.w
    for x, xp in zip((p.q, p.k, p.v), p.pa.xp):
        got = host(xp)
        assert not np.isnan(got).any()
        for b in range(w.B):
            for h in range(w.nh):
                idx = p.oracle[b][h]["idx"]
                assert np.array_equal(got[b, h], po.permute(x[b, h], idx, w.npad))


@pytest.mark.parametrize("name", ALL)
def test_quantize_codes_and_scales_bit_exact(name):
    p = problem(name)
    w = p.w
    if w.bits_qk == 16:  # unquantized mode: operands are bf16 values, compared exactly
        qc, kc, vc = host(p.pa.qc), host(p.pa.kc), host(p.pa.vc)
        for b in range(w.B):
            for h in range(w.nh):
                r = p.oracle[b][h]
                assert np.array_equal(qc[b, h], r["qc"]) and np.array_equal(kc[b, h], r["kc"])
                assert np.array_equal(vt_to_rows(vc[b, h], w.block), r["vc"])
        return
    qc, kc = p.pa.qc.cpu().numpy(), p.pa.kc.cpu().numpy()
    vc = p.pa.vc.cpu().numpy()
    sq, sk, sv = (t.cpu().numpy() for t in (p.pa.sq, p.pa.sk, p.pa.sv))
    for b in range(w.B):
        for h in range(w.nh):
            r = p.oracle[b][h]
            g_q = unpack_rows_int4(qc[b, h]) if w.bits_qk == 4 else qc[b, h].astype(np.int32)
            g_k = unpack_rows_int4(kc[b, h]) if w.bits_qk == 4 else kc[b, h].astype(np.int32)
            assert np.array_equal(g_q, r["qc"])
            assert np.array_equal(g_k, r["kc"])
            v_slots = unpack_vt_int4(vc[b, h]) if w.bits_pv == 4 else vc[b, h].astype(np.int32)
            assert np.array_equal(vt_to_rows(v_slots, w.block), r["vc"])
            assert np.array_equal(sq[b, h], r["sq"]) and np.array_equal(sk[b, h], r["sk"]) and np.array_equal(sv[b, h], r["sv"])


@pytest.mark.parametrize("name", ALL)
def test_attention_matches_oracle(name):
    p = problem(name)
    w = p.w
    op = host(p.pa.op)
    o = host(p.o)
    assert not np.isnan(op).any() and not np.isnan(o).any()
    for b in range(w.B):
        for h in range(w.nh):
            r = p.oracle[b][h]
            # the oracle's float64 result; a bf16 output adds at most half a bf16 step to the error
            ref_p, ref = r["op"], r["o"]
            assert np.all(op[b, h, w.N:] == 0)  # padded rows are written as zeros
            rel = REL_L2_BF16 if w.bits_qk == 16 else REL_L2
            check_attention(op[b, h], ref_p, r["flip_risk"], MAX_ABS, rel, "%s b%d h%d" % (name, b, h))
            check_attention(o[b, h], ref, po.unpermute(r["flip_risk"], r["idx"]), MAX_ABS, rel)


@pytest.mark.parametrize("name", ["video64", "video32_f32"])
def test_unpermute_bit_exact(name):
    p = problem(name)
    w = p.w
    op, o = host(p.pa.op), host(p.o)
    for b in range(w.B):
        for h in range(w.nh):
            assert np.array_equal(o[b, h], po.unpermute(op[b, h], p.oracle[b][h]["idx"]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("bits,layout", [(8, "rows"), (8, "vt"), (4, "rows"), (4, "vt"), (16, "rows"), (16, "vt")])
def test_quantize_all_modes_ragged(dtype, bits, layout):
    """Every (dtype, bits, layout) of paro_quantize on a ragged shape, including garbage in the
    padded rows (which must not influence scales or codes)."""
    torch, pb = _torch(), _pb()
    rng = np.random.default_rng(bits * 7 + len(layout))
    B, nh, d, block = 1, 2, 64, 64
    F, H, W = 2, 9, 11  # N = 198 = 3*64 + 6
    s = pb.make_shape(B, nh, d, F, H, W, 0, block)
    n, k, npad = 198, 4, 256
    x = (rng.standard_normal((B, nh, npad, d)) * rng.uniform(0.2, 5, size=(B, nh, npad, 1))).astype(np.float32)
    x[0, 1, 64:128] = 0  # an all-zero block
    if dtype == "bf16":
        x = wl.bf16_round(x)
    x[:, :, n:] = 1000.0  # garbage where padding should be
    xp = to_dev(x, dtype)
    lay = pb.PARO_ROWS if layout == "rows" else pb.PARO_VT
    codes = torch.full(pb.codes_shape(s, bits, lay), -1 if bits != 16 else float("nan"),
                       dtype=torch.bfloat16 if bits == 16 else torch.int8, device="cuda:0")
    scales = torch.full((B, nh, k), float("nan"), dtype=torch.float32, device="cuda:0")
    pb.paro_quantize(s, bits, lay, xp, codes, scales)
    torch.cuda.synchronize()
    got_s = scales.cpu().numpy()
    got = host(codes)
    for h in range(nh):
        if bits == 16:
            ref = x[0, h].copy()
            ref[n:] = 0
            ref = wl.bf16_round(ref).astype(np.float32)
            rows = got[0, h] if layout == "rows" else vt_to_rows(got[0, h], block)
            assert np.array_equal(rows, ref)
            assert np.all(got_s[0, h] == 1.0)
            continue
        ref_c, ref_s = po.quantize_blocks(x[0, h], n, block, po.qmax_of(bits))
        if layout == "rows":
            rows = unpack_rows_int4(got[0, h]) if bits == 4 else got[0, h].astype(np.int32)
        else:
            slots = unpack_vt_int4(got[0, h]) if bits == 4 else got[0, h].astype(np.int32)
            rows = vt_to_rows(slots, block)
        assert np.array_equal(rows, ref_c)
        assert np.array_equal(got_s[0, h], ref_s)


def _amax_with_all_ones_scale(rng, qmax):
    """A float32 absmax whose binary32 quotient by qmax has an all-ones significand."""
    while True:
        e = int(rng.integers(-8, 8))
        target = np.float32((2.0 - 2.0 ** -23) * 2.0 ** e)
        a = np.float32(target * np.float32(qmax))
        for _ in range(64):
            if (np.float32(a / np.float32(qmax)).view(np.uint32) & np.uint32(0x7FFFFF)) == np.uint32(0x7FFFFF):
                return a
            a = np.nextafter(a, np.float32(0), dtype=np.float32)


@pytest.mark.parametrize("bits", [8, 4])
def test_quantize_codes_are_the_correctly_rounded_quotient_in_hard_cases(bits):
    """The code is rint(fl32(x / scale)) bit for bit: groups with huge and tiny magnitudes, scales whose
    significand is all ones, and elements placed on and next to rounding ties of the quotient."""
    torch, pb = _torch(), _pb()
    rng = np.random.default_rng(300 + bits)
    qmax = po.qmax_of(bits)
    B, nh, d, block = 1, 2, 64, 64
    F, H, W = 4, 8, 16  # N = 512 = 8 blocks
    s = pb.make_shape(B, nh, d, F, H, W, 0, block)
    n = npad = 512
    k = 8
    x = np.zeros((B, nh, npad, d), np.float32)
    mags = [2.0 ** -60, 2.0 ** -30, 1.0, 2.0 ** 30, 2.0 ** 60, 3e-39, 1.0, 1.0]
    for h in range(nh):
        for g in range(k):
            blk = rng.standard_normal((block, d)).astype(np.float32)
            amax = np.float32(np.abs(blk).max())
            if g >= 6:  # scale with an all-ones significand
                amax_new = _amax_with_all_ones_scale(rng, qmax)
                blk = (blk * (amax_new / amax) * np.float32(0.999)).astype(np.float32)
                blk[0, 0] = amax_new
                scale = np.float32(amax_new / np.float32(qmax))
            else:
                blk = (blk * np.float32(mags[g])).astype(np.float32)
                scale = np.float32(np.abs(blk).max() / np.float32(qmax))
            # ties of the quotient and their neighbours, without raising the absmax
            for i in range(1, 40):
                c = int(rng.integers(0, qmax - 1))
                t = np.float32(np.float32(c + 0.5) * scale)
                for j, v in enumerate((np.nextafter(t, np.float32(0)), t, np.nextafter(t, np.float32(np.inf)))):
                    blk[i, 3 * (i % 20) + j] = v if rng.random() < 0.5 else -v
            x[0, h, g * block:(g + 1) * block] = blk
    xp = to_dev(x, "f32")
    for lay, name in ((pb.PARO_ROWS, "rows"), (pb.PARO_VT, "vt")):
        codes = torch.full(pb.codes_shape(s, bits, lay), -1, dtype=torch.int8, device="cuda:0")
        scales = torch.full((B, nh, k), float("nan"), dtype=torch.float32, device="cuda:0")
        pb.paro_quantize(s, bits, lay, xp, codes, scales)
        torch.cuda.synchronize()
        got, got_s = host(codes), scales.cpu().numpy()
        for h in range(nh):
            ref_c, ref_s = po.quantize_blocks(x[0, h], n, block, qmax)
            if name == "rows":
                rows = unpack_rows_int4(got[0, h]) if bits == 4 else got[0, h].astype(np.int32)
            else:
                rows = vt_to_rows(unpack_vt_int4(got[0, h]) if bits == 4 else got[0, h].astype(np.int32), block)
            assert np.array_equal(got_s[0, h], ref_s), name
            bad = np.argwhere(rows != ref_c)
            assert bad.size == 0, "%s: %d codes differ, first at %s" % (name, len(bad), bad[:3].tolist())
        assert (np.asarray(got_s).view(np.uint32) & 0x7FFFFF == 0x7FFFFF).any()  # the all-ones case was exercised


@pytest.mark.parametrize("bits", [8, 16])
def test_row_maximum_climbing_hundreds_of_octaves(bits):
    """Keys whose magnitude grows along the sequence make the running row maximum climb by far more
    than 64 octaves between the first and the last live block, so the kernels have to re-reference
    their running sums several times; a second head has the steep end first (the maximum never moves
    after the first block)."""
    torch, pb = _torch(), _pb()
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = SMALL["video64"].replace(nh=2, perm_choice=(0, 0), bits_qk=bits, bits_pv=bits, density=1.0, dtype="f32", seed=77)
    masks = wl.make_block_masks(w, gather_fn(w))
    bm, row_ptr, col_idx = blocklist_for(w, masks)
    rng = np.random.default_rng(78)
    ramp = np.linspace(0.05, 12.0, w.N)[:, None]
    q = np.abs(rng.standard_normal((1, 2, w.N, w.d))).astype(np.float32) * 3
    k = np.abs(rng.standard_normal((1, 2, w.N, w.d))).astype(np.float32)
    k[0, 0] *= ramp          # logits grow along the sequence
    k[0, 1] *= ramp[::-1]    # logits shrink along the sequence
    v = rng.standard_normal((1, 2, w.N, w.d)).astype(np.float32)
    if bits == 16:
        q, k, v = (wl.bf16_round(x) for x in (q, k, v))
    pa = ParoAttention(pb.shape_of(w), wl.make_perm_ids(w), bm, bits, bits, torch.float32)
    o = host(pa.run_fused(*(to_dev(x, "f32") for x in (q, k, v))))
    torch.cuda.synchronize()
    for h in range(2):
        r = oracle_head(w, q[0, h], k[0, h], v[0, h], 0, row_ptr[h], col_idx)
        # the spread of the logits of one row, in octaves, far exceeds the re-referencing threshold
        logit = (q[0, h, :1].astype(np.float64) @ k[0, h].astype(np.float64).T) / np.sqrt(w.d) * np.log2(np.e)
        assert logit.max() - logit.min() > 200
        assert np.isfinite(o[0, h]).all()
        st = check_attention(o[0, h], r["o"], po.unpermute(r["flip_risk"], r["idx"]), MAX_ABS, REL_L2_BF16 if bits == 16 else REL_L2,
                             "steep head %d" % h)
        # With fp32 output the error left is that of the arithmetic.  With 8-bit P codes the kernel forms the
        # exponent as c*(B + S) + offset: the offset's rounding grows with the logit scale c (here the logits
        # span hundreds of octaves, several times a real layer's), flips more near-tie codes, and is the
        # larger part of what is left; the 16-bit mode keeps the exact exponent and rounds P to bf16 (2^-9 per
        # element, and on these rows a handful of keys carry the whole sum).
        assert st["rel_l2"] < (3e-3 if bits == 8 else 2e-3)


@pytest.mark.parametrize("scale", [1e-3, 1e-6, 30.0])
@pytest.mark.parametrize("bits_pv", [8, 4])
def test_padded_keys_get_no_mass_even_when_all_logits_are_tiny(scale, bits_pv):
    """Inputs of very small magnitude make every logit (and the scale product c) almost zero, so a
    masked key is excluded only if the kernel excludes it explicitly: on a ragged sequence the padded
    keys of the last block must still receive no probability."""
    torch, pb = _torch(), _pb()
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = SMALL["video64"].replace(nh=2, perm_choice=(3, 0), bits_pv=bits_pv, density=1.0, dtype="f32", seed=81)
    assert w.N % w.block != 0
    masks = wl.make_block_masks(w, gather_fn(w))
    bm, row_ptr, col_idx = blocklist_for(w, masks)
    q, k, v = wl.make_qkv(w)
    q, k = (q * np.float32(scale)).astype(np.float32), (k * np.float32(scale)).astype(np.float32)
    perm_ids = wl.make_perm_ids(w)
    pa = ParoAttention(pb.shape_of(w), perm_ids, bm, w.bits_qk, bits_pv, torch.float32)
    o = host(pa.run_fused(*(to_dev(x, "f32") for x in (q, k, v))))
    torch.cuda.synchronize()
    for h in range(w.nh):
        r = oracle_head(w, q[0, h], k[0, h], v[0, h], perm_ids[h], row_ptr[h], col_idx)
        check_attention(o[0, h], r["o"], po.unpermute(r["flip_risk"], r["idx"]), MAX_ABS, REL_L2, "tiny logits head %d" % h)


@pytest.mark.parametrize("name", ["video64", "video64_int4", "flux128"])
@pytest.mark.parametrize("q_dtype", ["bf16", "f32"])
def test_in_kernel_q_quantization_is_bit_identical(name, q_dtype):
    """paro_sparse_attn_unpermuted_rawq (Q reordered and quantized by the workgroup that owns the row
    block) gives exactly the output of paro_permute_quantize(Q) + paro_sparse_attn_unpermuted, for both
    input types, on ragged shapes, with text tokens and with 4-bit PV - bit for bit where both run the same
    attention kernel, to the rounding of the output where they do not (d = 128 with 8-bit codes)."""
    torch, pb = _torch(), _pb()
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = SMALL[name].replace(dtype=q_dtype)
    s = pb.shape_of(w)
    perm_ids = wl.make_perm_ids(w)
    bm = wl.pack_bitmask(wl.make_block_masks(w, gather_fn(w), perm_ids))
    q, k, v = (to_dev(x, q_dtype) for x in wl.make_qkv(w))
    q[0, 0, : w.block] *= 1e-30  # a row block of tiny magnitude (generic divide path of the quantizer)
    pa = ParoAttention(s, perm_ids, bm, 8, w.bits_pv, tdtype(q_dtype))
    assert pa.can_fuse_q
    want = pa.run_fused(q, k, v).clone()
    pa.o.fill_(float("nan"))
    got = pa.run_rawq(q, k, v)
    torch.cuda.synchronize()
    assert not torch.isnan(got).any()
    if same_attention_kernel_for_raw_q(w):
        assert torch.equal(got, want)
    else:
        assert_equal_up_to_output_rounding(got, want, name)


def test_in_kernel_q_quantization_rejects_what_it_does_not_cover():
    torch, pb = _torch(), _pb()
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = SMALL["video32_f32"]
    s = pb.shape_of(w)
    perm_ids = wl.make_perm_ids(w)
    bm = wl.pack_bitmask(wl.make_block_masks(w, gather_fn(w), perm_ids))
    pa = ParoAttention(s, perm_ids, bm, 8, 8, torch.float32)
    assert not pa.can_fuse_q
    q, k, v = (to_dev(x, "f32") for x in wl.make_qkv(w))
    with pytest.raises(pb.ParoError) as e:
        pa.run_rawq(q, k, v)
    assert e.value.status == pb.PARO_EUNSUPPORTED


def test_empty_row_block_gives_zeros():
    torch, pb = _torch(), _pb()
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = SMALL["video64"].replace(nh=1, perm_choice=(3,))
    masks = wl.make_block_masks(w, gather_fn(w))
    masks[0, 2, :] = False  # row block 2 attends nothing
    bits, row_ptr, col_idx = blocklist_for(w, masks)
    q, k, v = wl.make_qkv(w)
    pa = ParoAttention(pb.shape_of(w), wl.make_perm_ids(w), bits, 8, 8, torch.bfloat16)
    pa.run(*(to_dev(x, "bf16") for x in (q, k, v)))
    torch.cuda.synchronize()
    op = host(pa.op)[0, 0]
    r = oracle_head(w, q[0, 0], k[0, 0], v[0, 0], 3, row_ptr[0], col_idx)
    assert np.all(op[128:192] == 0)
    check_attention(op, r["op"], r["flip_risk"], MAX_ABS, REL_L2)


@pytest.mark.parametrize("name", ["video64", "video64_int4", "video32_f32", "flux128", "flux128_b32_int4", "video64_bf16", "video32_bf16_f32io",
                                  "video64_i4i4", "video64_i4i8_f32", "flux128_i4i8_f32"])
def test_fused_entry_points_are_bit_identical_to_the_separate_steps(name):
    """paro_permute_quantize == paro_permute + paro_quantize and paro_sparse_attn_unpermuted ==
    paro_sparse_attn + paro_unpermute, bit for bit (so the oracle parity of the separate steps
    carries over), including untouched padding and ragged tails."""
    torch = _torch()
    p = problem(name)
    pa = p.pa
    ref_q, ref_k, ref_v = pa.qc.clone(), pa.kc.clone(), pa.vc.clone()
    ref_s = [t.clone() for t in (pa.sq, pa.sk, pa.sv)]
    ref_o = p.o.clone()
    for t in (pa.vc,):
        t.zero_()
    for t in (pa.sq, pa.sk, pa.sv):
        t.fill_(float("nan"))
    pa.o.fill_(float("nan"))
    o = pa.run_fused(p.dq, p.dk, p.dv)
    torch.cuda.synchronize()
    fq, fk = pa._fused_buffers()
    assert torch.equal(fq.view(torch.uint8) if fq.dtype == torch.int8 else fq, ref_q.view(torch.uint8) if ref_q.dtype == torch.int8 else ref_q)
    assert torch.equal(fk.view(torch.uint8) if fk.dtype == torch.int8 else fk, ref_k.view(torch.uint8) if ref_k.dtype == torch.int8 else ref_k)
    assert torch.equal(pa.vc, ref_v)
    if p.w.bits_qk != 16:
        for got, ref in zip((pa.sq, pa.sk, pa.sv), ref_s):
            assert torch.equal(got, ref)
    assert torch.equal(o, ref_o)
    # the three quantizer launches as one
    fq.fill_(1)
    fk.fill_(1)
    pa.vc.fill_(1)
    for t in (pa.sq, pa.sk, pa.sv):
        t.fill_(float("nan"))
    pa.prepare_fused_qkv(p.dq, p.dk, p.dv)
    torch.cuda.synchronize()
    assert torch.equal(fq.view(torch.uint8) if fq.dtype == torch.int8 else fq, ref_q.view(torch.uint8) if ref_q.dtype == torch.int8 else ref_q)
    assert torch.equal(fk.view(torch.uint8) if fk.dtype == torch.int8 else fk, ref_k.view(torch.uint8) if ref_k.dtype == torch.int8 else ref_k)
    assert torch.equal(pa.vc, ref_v)
    for got, ref in zip((pa.sq, pa.sk, pa.sv), ref_s):
        assert torch.equal(got, ref) or p.w.bits_qk == 16
    if p.w.bits_qk == 16:
        assert all(bool((t == 1).all()) for t in (pa.sq, pa.sk, pa.sv))


@pytest.mark.parametrize("name", ["video64", "flux128", "video64_bf16"])
def test_row_schedule_does_not_change_results(name):
    torch, pb = _torch(), _pb()
    p = problem(name)
    pa = p.pa
    pa.attend()  # scheduled order (the pipeline's default)
    torch.cuda.synchronize()
    ref = pa.op.clone()
    pa.op.fill_(float("nan"))
    pb.paro_sparse_attn(pa.s, pa.bits_qk, pa.bits_pv, pa.qc, pa.sq, pa.kc, pa.sk, pa.vc, pa.sv, pa.row_ptr, pa.col_idx, pa.op, None)
    torch.cuda.synchronize()
    assert torch.equal(pa.op, ref)
    assert not np.array_equal(pa.h_row_order, np.arange(pa.h_row_order.size))


def test_heads_of_unequal_density_are_dealt_to_the_xcds_and_results_do_not_change():
    """Masks whose density differs from head to head (one threshold per head, Sec. 4.2 (3)): the launch order moves
    whole heads between the XCDs' ranges; the output is bit-identical to the natural order and matches the oracle."""
    torch, pb = _torch(), _pb()
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = wl.Workload("uneq", 1, 16, 64, 2, 8, 12, 0, 32, 0.25, 8, 8, "bf16", 77, perm_choice=(0, 2, 5))
    dense = w.replace(density=0.9)
    perm_ids = wl.make_perm_ids(w)
    masks = wl.make_block_masks(w, gather_fn(w), perm_ids)
    masks[:8] = wl.make_block_masks(dense, gather_fn(w), perm_ids)[:8]  # heads 0..7 dense, 8..15 sparse
    bits, row_ptr, col_idx = blocklist_for(w, masks)
    s = pb.shape_of(w)
    pa = ParoAttention(s, perm_ids, bits, w.bits_qk, w.bits_pv, tdtype(w.dtype))
    order = pa.h_row_order
    pb.paro_check_row_order(s, order)
    live = masks.sum(2)
    loads = np.array([live[c // w.k, c % w.k].sum() for c in np.split(order, 8)])
    natural = np.array([live[2 * x:2 * x + 2].sum() for x in range(8)])
    assert natural.max() > 1.3 * natural.mean() and loads.max() < 1.1 * loads.mean()
    q, k, v = wl.make_qkv(w)
    o = pa.run(*(to_dev(x, w.dtype) for x in (q, k, v))).clone()
    torch.cuda.synchronize()
    pa.op.fill_(float("nan"))
    pb.paro_sparse_attn(pa.s, pa.bits_qk, pa.bits_pv, pa.qc, pa.sq, pa.kc, pa.sk, pa.vc, pa.sv, pa.row_ptr, pa.col_idx, pa.op, None)
    torch.cuda.synchronize()
    assert torch.equal(pa.finish(), o)
    got = host(o)
    for h in (0, 7, 8, 15):
        ref = oracle_head(w, q[0, h], k[0, h], v[0, h], perm_ids[h], row_ptr[h], col_idx)
        check_attention(got[0, h], ref["o"], po.unpermute(ref["flip_risk"], ref["idx"]), MAX_ABS, REL_L2, "unequal heads, head %d" % h)
