"""Thin ctypes binding over libparo.so: same names as the C ABI (include/paro.h), argument
marshalling only.  Device tensors are torch tensors (device memory + the current HIP stream);
every step of the path runs inside the library's kernels.

The library is loaded on first use and the binding fails loudly if it has not been built
(``python -m paper_2506_16054_amd.build``): there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

PARO_OK = 0
PARO_EINVAL = -1
PARO_EUNSUPPORTED = -2
PARO_EHIP = -3
PARO_F32 = 0
PARO_BF16 = 1
PARO_ROWS = 0
PARO_VT = 1

LIBPATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libparo.so")

EXPORTS = (
    "paro_version", "paro_strerror", "paro_last_error", "paro_ntokens", "paro_nblocks", "paro_npad",
    "paro_perm_index", "paro_vt_slot", "paro_mask_to_blocklist", "paro_permute", "paro_unpermute",
    "paro_quantize", "paro_sparse_attn", "paro_permute_quantize", "paro_sparse_attn_unpermuted", "paro_schedule_rows", "paro_check_blocklist", "paro_check_row_order",
    "paro_mask_to_blocklist_device", "paro_calib_block_stats", "paro_calib_metrics", "paro_calib_choose", "paro_calib_mask",
    "paro_sparse_attn_unpermuted_rawq", "paro_blocklist_cols_device", "paro_permute_quantize_qkv",
    "paro_k_channel_mean", "paro_permute_quantize_smoothed",
)


class ParoError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("paro status %d: %s" % (status, message))
        self.status = status


class paro_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "nh", "d", "F", "Hg", "Wg", "T_text", "block")]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIBPATH):
            raise ParoError(PARO_EHIP, "%s is missing: build it with `python -m paper_2506_16054_amd.build`" % LIBPATH)
        L = ctypes.CDLL(LIBPATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        sp = ctypes.POINTER(paro_shape)
        L.paro_version.restype = i32
        L.paro_strerror.restype = ctypes.c_char_p
        L.paro_strerror.argtypes = [i32]
        L.paro_last_error.restype = ctypes.c_char_p
        for f in (L.paro_ntokens, L.paro_nblocks, L.paro_npad):
            f.restype = i64
            f.argtypes = [sp]
        L.paro_perm_index.argtypes = [sp, i32, vp]
        L.paro_vt_slot.argtypes = [i32, i32]
        L.paro_mask_to_blocklist.argtypes = [i32, i32, vp, vp, vp, i64, ctypes.POINTER(i64)]
        L.paro_permute.argtypes = [sp, i32, vp, vp, vp, vp]
        L.paro_unpermute.argtypes = [sp, i32, vp, vp, vp, vp]
        L.paro_quantize.argtypes = [sp, i32, i32, i32, vp, vp, vp, vp]
        L.paro_sparse_attn.argtypes = [sp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, i32, vp, vp]
        L.paro_schedule_rows.argtypes = [sp, i32, i32, vp, vp]
        L.paro_check_blocklist.argtypes = [i32, i32, vp, vp, i64]
        L.paro_check_row_order.argtypes = [sp, vp]
        L.paro_permute_quantize.argtypes = [sp, i32, i32, i32, vp, vp, vp, vp, vp]
        L.paro_sparse_attn_unpermuted.argtypes = [sp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, vp, i32, vp, vp]
        L.paro_mask_to_blocklist_device.argtypes = [i32, i32, vp, vp, vp, i64, vp, vp]
        f32 = ctypes.c_float
        L.paro_calib_block_stats.argtypes = [sp, vp, vp, f32, vp, vp, vp, vp]
        L.paro_calib_metrics.argtypes = [sp, vp, vp, vp, f32, vp, vp, vp]
        L.paro_calib_choose.argtypes = [i32, vp, vp, f32, vp, vp, vp]
        L.paro_calib_mask.argtypes = [sp, vp, f32, vp, vp]
        L.paro_sparse_attn_unpermuted_rawq.argtypes = [sp, i32, i32, vp, vp, vp, vp, vp, vp, vp, i64, vp, vp, i32, vp, vp]
        L.paro_blocklist_cols_device.argtypes = [i32, i32, vp, vp, vp, i64, vp]
        L.paro_permute_quantize_qkv.argtypes = [sp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.paro_k_channel_mean.argtypes = [sp, i32, vp, vp, vp]
        L.paro_permute_quantize_smoothed.argtypes = [sp, i32, i32, vp, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != PARO_OK:
        raise ParoError(status, lib().paro_last_error().decode() or lib().paro_strerror(status).decode())


def make_shape(B: int, nh: int, d: int, F: int, Hg: int, Wg: int, T_text: int, block: int) -> paro_shape:
    return paro_shape(B, nh, d, F, Hg, Wg, T_text, block)


def shape_of(w) -> paro_shape:
    """paro_shape of a workloads.Workload."""
    return paro_shape(w.B, w.nh, w.d, w.F, w.Hg, w.Wg, w.T_text, w.block)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch

    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t) -> int:
    import torch

    if t.dtype == torch.float32:
        return PARO_F32
    if t.dtype == torch.bfloat16:
        return PARO_BF16
    raise ParoError(PARO_EINVAL, "tensor dtype %s is neither float32 nor bfloat16" % t.dtype)


def _require(t, name: str, shape=None, dtype=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ParoError(PARO_EINVAL, "%s must be a contiguous device tensor" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ParoError(PARO_EINVAL, "%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    if dtype is not None and t.dtype != dtype:
        raise ParoError(PARO_EINVAL, "%s has dtype %s, expected %s" % (name, t.dtype, dtype))


# ---------------------------------------------------------------------------------------------
# host-only calls
# ---------------------------------------------------------------------------------------------
def paro_version() -> int:
    return lib().paro_version()


def paro_ntokens(s: paro_shape) -> int:
    n = lib().paro_ntokens(ctypes.byref(s))
    if n < 0:
        _check(int(n))
    return int(n)


def paro_nblocks(s: paro_shape) -> int:
    n = lib().paro_nblocks(ctypes.byref(s))
    if n < 0:
        _check(int(n))
    return int(n)


def paro_npad(s: paro_shape) -> int:
    n = lib().paro_npad(ctypes.byref(s))
    if n < 0:
        _check(int(n))
    return int(n)


def paro_perm_index(s: paro_shape, perm_id: int) -> np.ndarray:
    n = paro_ntokens(s)
    idx = np.empty(n, np.int32)
    _check(lib().paro_perm_index(ctypes.byref(s), int(perm_id), idx.ctypes.data))
    return idx


def paro_vt_slot(block: int, i: int) -> int:
    r = lib().paro_vt_slot(int(block), int(i))
    if r < 0:
        _check(r)
    return r


def paro_mask_to_blocklist(nh: int, k: int, bitmask: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """bitmask uint8 [nh, ceil(k*k/8)] -> (row_ptr int32 [nh, k+1], col_idx int32 [nnz]), host arrays."""
    bm = np.ascontiguousarray(bitmask, dtype=np.uint8)
    if bm.shape != (nh, (k * k + 7) // 8):
        raise ParoError(PARO_EINVAL, "bitmask has shape %s, expected %s" % (bm.shape, (nh, (k * k + 7) // 8)))
    row_ptr = np.empty((nh, k + 1), np.int32)
    nnz = ctypes.c_int64(0)
    st = lib().paro_mask_to_blocklist(nh, k, bm.ctypes.data, row_ptr.ctypes.data, None, 0, ctypes.byref(nnz))
    if st != PARO_OK and nnz.value == 0:
        _check(st)
    col_idx = np.empty(max(nnz.value, 1), np.int32)
    _check(lib().paro_mask_to_blocklist(nh, k, bm.ctypes.data, row_ptr.ctypes.data, col_idx.ctypes.data, col_idx.size, ctypes.byref(nnz)))
    return row_ptr, col_idx[: nnz.value]


def paro_check_blocklist(nh: int, k: int, row_ptr: np.ndarray, col_idx: np.ndarray) -> None:
    """Raises ParoError unless the host block list is what the attention kernels assume."""
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    if rp.shape != (nh, k + 1):
        raise ParoError(PARO_EINVAL, "row_ptr has shape %s, expected (%d, %d)" % (rp.shape, nh, k + 1))
    _check(lib().paro_check_blocklist(int(nh), int(k), rp.ctypes.data, ci.ctypes.data if ci.size else None, int(ci.size)))


def paro_check_row_order(s: paro_shape, row_order: np.ndarray) -> None:
    """Raises ParoError unless the host launch order is a permutation of all row blocks."""
    ro = np.ascontiguousarray(row_order, dtype=np.int32)
    total = s.B * s.nh * paro_nblocks(s)
    if ro.shape != (total,):
        raise ParoError(PARO_EINVAL, "row_order has shape %s, expected (%d,)" % (ro.shape, total))
    _check(lib().paro_check_row_order(ctypes.byref(s), ro.ctypes.data))


def paro_schedule_rows(s: paro_shape, bits_qk: int, bits_pv: int, row_ptr: np.ndarray) -> np.ndarray:
    """Launch order of the row blocks (host): int32 [B*nh*k]."""
    k = paro_nblocks(s)
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    if rp.shape != (s.nh, k + 1):
        raise ParoError(PARO_EINVAL, "row_ptr has shape %s, expected %s" % (rp.shape, (s.nh, k + 1)))
    order = np.empty(s.B * s.nh * k, np.int32)
    _check(lib().paro_schedule_rows(ctypes.byref(s), int(bits_qk), int(bits_pv), rp.ctypes.data, order.ctypes.data))
    return order


# ---------------------------------------------------------------------------------------------
# device calls (torch tensors on the GPU; enqueued on torch's current stream)
# ---------------------------------------------------------------------------------------------
def _perm_bytes(s: paro_shape, perm_ids) -> np.ndarray:
    p = np.ascontiguousarray(perm_ids, dtype=np.uint8)
    if p.shape != (s.nh,):
        raise ParoError(PARO_EINVAL, "perm_ids has shape %s, expected (%d,)" % (p.shape, s.nh))
    return p


def paro_permute(s: paro_shape, perm_ids, x, xp) -> None:
    n, npad = paro_ntokens(s), paro_npad(s)
    _require(x, "x", (s.B, s.nh, n, s.d))
    _require(xp, "xp", (s.B, s.nh, npad, s.d), x.dtype)
    p = _perm_bytes(s, perm_ids)
    _check(lib().paro_permute(ctypes.byref(s), _dtype_code(x), p.ctypes.data, _ptr(x), _ptr(xp), _stream()))


def paro_unpermute(s: paro_shape, perm_ids, op, o) -> None:
    n, npad = paro_ntokens(s), paro_npad(s)
    _require(op, "op", (s.B, s.nh, npad, s.d))
    _require(o, "o", (s.B, s.nh, n, s.d), op.dtype)
    p = _perm_bytes(s, perm_ids)
    _check(lib().paro_unpermute(ctypes.byref(s), _dtype_code(op), p.ctypes.data, _ptr(op), _ptr(o), _stream()))


def codes_shape(s: paro_shape, bits: int, layout: int) -> Tuple[int, ...]:
    """Shape of the `codes` tensor of paro_quantize (int8 bytes for bits 8/4, bf16 for bits 16)."""
    k, npad = paro_nblocks(s), paro_npad(s)
    pack = 2 if bits == 4 else 1
    if layout == PARO_ROWS:
        return (s.B, s.nh, npad, s.d // pack)
    return (s.B, s.nh, k, s.d, s.block // pack)


def paro_quantize(s: paro_shape, bits: int, layout: int, xp, codes, scales) -> None:
    import torch

    _require(xp, "xp", (s.B, s.nh, paro_npad(s), s.d))
    _require(codes, "codes", codes_shape(s, bits, layout), torch.bfloat16 if bits == 16 else torch.int8)
    _require(scales, "scales", (s.B, s.nh, paro_nblocks(s)), torch.float32)
    _check(lib().paro_quantize(ctypes.byref(s), _dtype_code(xp), int(bits), int(layout), _ptr(xp), _ptr(codes), _ptr(scales), _stream()))


def paro_permute_quantize(s: paro_shape, bits: int, layout: int, perm_ids, x, codes, scales) -> None:
    import torch

    _require(x, "x", (s.B, s.nh, paro_ntokens(s), s.d))
    _require(codes, "codes", codes_shape(s, bits, layout), torch.bfloat16 if bits == 16 else torch.int8)
    _require(scales, "scales", (s.B, s.nh, paro_nblocks(s)), torch.float32)
    p = _perm_bytes(s, perm_ids)
    _check(lib().paro_permute_quantize(ctypes.byref(s), _dtype_code(x), int(bits), int(layout), p.ctypes.data, _ptr(x), _ptr(codes),
                                       _ptr(scales), _stream()))


def paro_permute_quantize_qkv(s: paro_shape, bits_qk: int, bits_pv: int, perm_ids, q, k, v, q_codes, sq, k_codes, sk, v_codes, sv) -> None:
    import torch

    for name, x in (("q", q), ("k", k), ("v", v)):
        _require(x, name, (s.B, s.nh, paro_ntokens(s), s.d), q.dtype)
    ct_qk = torch.bfloat16 if bits_qk == 16 else torch.int8
    _require(q_codes, "q_codes", codes_shape(s, bits_qk, PARO_ROWS), ct_qk)
    _require(k_codes, "k_codes", codes_shape(s, bits_qk, PARO_ROWS), ct_qk)
    _require(v_codes, "v_codes", codes_shape(s, bits_pv, PARO_VT), torch.bfloat16 if bits_pv == 16 else torch.int8)
    for name, x in (("sq", sq), ("sk", sk), ("sv", sv)):
        _require(x, name, (s.B, s.nh, paro_nblocks(s)), torch.float32)
    p = _perm_bytes(s, perm_ids)
    _check(lib().paro_permute_quantize_qkv(ctypes.byref(s), _dtype_code(q), int(bits_qk), int(bits_pv), p.ctypes.data, _ptr(q), _ptr(k),
                                           _ptr(v), _ptr(q_codes), _ptr(sq), _ptr(k_codes), _ptr(sk), _ptr(v_codes), _ptr(sv), _stream()))


def paro_k_channel_mean(s: paro_shape, k, k_mean) -> None:
    import torch

    _require(k, "k", (s.B, s.nh, paro_ntokens(s), s.d))
    _require(k_mean, "k_mean", (s.B, s.nh, s.d), torch.float32)
    _check(lib().paro_k_channel_mean(ctypes.byref(s), _dtype_code(k), _ptr(k), _ptr(k_mean), _stream()))


def paro_permute_quantize_smoothed(s: paro_shape, bits: int, perm_ids, k, k_mean, codes, scales) -> None:
    import torch

    _require(k, "k", (s.B, s.nh, paro_ntokens(s), s.d))
    _require(k_mean, "k_mean", (s.B, s.nh, s.d), torch.float32)
    _require(codes, "codes", codes_shape(s, bits, PARO_ROWS), torch.int8)
    _require(scales, "scales", (s.B, s.nh, paro_nblocks(s)), torch.float32)
    p = _perm_bytes(s, perm_ids)
    _check(lib().paro_permute_quantize_smoothed(ctypes.byref(s), _dtype_code(k), int(bits), p.ctypes.data, _ptr(k), _ptr(k_mean),
                                                _ptr(codes), _ptr(scales), _stream()))


def paro_mask_to_blocklist_device(nh: int, k: int, bitmask, row_ptr, col_idx, nnz_out=None) -> None:
    """Device tensors: bitmask uint8 [nh, ceil(k*k/8)] -> row_ptr int32 [nh, k+1], col_idx int32 [cap]
    (cap = col_idx.numel(); may be None for the offsets only), nnz_out int32 [1] or None."""
    import torch

    _require(bitmask, "bitmask", (nh, (k * k + 7) // 8), torch.uint8)
    _require(row_ptr, "row_ptr", (nh, k + 1), torch.int32)
    if col_idx is not None:
        _require(col_idx, "col_idx", None, torch.int32)
    if nnz_out is not None:
        _require(nnz_out, "nnz_out", (1,), torch.int32)
    cap = 0 if col_idx is None else int(col_idx.numel())
    _check(lib().paro_mask_to_blocklist_device(int(nh), int(k), _ptr(bitmask), _ptr(row_ptr), _ptr(col_idx) if cap else None, cap,
                                               _ptr(nnz_out), _stream()))


def paro_blocklist_cols_device(nh: int, k: int, bitmask, row_ptr, col_idx) -> None:
    """Device tensors: bitmask uint8 [nh, ceil(k*k/8)] and row_ptr int32 [nh, k+1] (precomputed offsets) -> col_idx int32 [cap]."""
    import torch

    _require(bitmask, "bitmask", (nh, (k * k + 7) // 8), torch.uint8)
    _require(row_ptr, "row_ptr", (nh, k + 1), torch.int32)
    _require(col_idx, "col_idx", None, torch.int32)
    _check(lib().paro_blocklist_cols_device(int(nh), int(k), _ptr(bitmask), _ptr(row_ptr), _ptr(col_idx), int(col_idx.numel()), _stream()))


def paro_calib_block_stats(s: paro_shape, q16, k16, eps: float, block_sum, block_max, block_cnt) -> None:
    import torch

    kb = paro_nblocks(s)
    _require(q16, "q16", codes_shape(s, 16, PARO_ROWS), torch.bfloat16)
    _require(k16, "k16", codes_shape(s, 16, PARO_ROWS), torch.bfloat16)
    _require(block_sum, "block_sum", (s.B, s.nh, kb, kb), torch.float32)
    _require(block_max, "block_max", (s.B, s.nh, kb, kb), torch.float32)
    _require(block_cnt, "block_cnt", (s.B, s.nh, kb, kb), torch.int32)
    _check(lib().paro_calib_block_stats(ctypes.byref(s), _ptr(q16), _ptr(k16), float(eps), _ptr(block_sum), _ptr(block_max),
                                        _ptr(block_cnt), _stream()))


def paro_calib_metrics(s: paro_shape, block_sum, block_max, block_cnt, sigma: float, m_sparse, m_quant) -> None:
    import torch

    kb = paro_nblocks(s)
    _require(block_sum, "block_sum", (s.B, s.nh, kb, kb), torch.float32)
    _require(block_max, "block_max", (s.B, s.nh, kb, kb), torch.float32)
    _require(block_cnt, "block_cnt", (s.B, s.nh, kb, kb), torch.int32)
    _require(m_sparse, "m_sparse", (s.nh,), torch.float32)
    _require(m_quant, "m_quant", (s.nh,), torch.float32)
    _check(lib().paro_calib_metrics(ctypes.byref(s), _ptr(block_sum), _ptr(block_max), _ptr(block_cnt), float(sigma), _ptr(m_sparse),
                                    _ptr(m_quant), _stream()))


def paro_calib_choose(nh: int, m_sparse6, m_quant6, alpha: float, m_combined6, perm_ids) -> None:
    import torch

    for name, t in (("m_sparse6", m_sparse6), ("m_quant6", m_quant6), ("m_combined6", m_combined6)):
        _require(t, name, (6, nh), torch.float32)
    _require(perm_ids, "perm_ids", (nh,), torch.uint8)
    _check(lib().paro_calib_choose(int(nh), _ptr(m_sparse6), _ptr(m_quant6), float(alpha), _ptr(m_combined6), _ptr(perm_ids), _stream()))


def paro_calib_mask(s: paro_shape, block_sum, density: float, bitmask) -> None:
    import torch

    kb = paro_nblocks(s)
    _require(block_sum, "block_sum", (s.B, s.nh, kb, kb), torch.float32)
    _require(bitmask, "bitmask", (s.nh, (kb * kb + 7) // 8), torch.uint8)
    _check(lib().paro_calib_mask(ctypes.byref(s), _ptr(block_sum), float(density), _ptr(bitmask), _stream()))


def _attn_operands(s: paro_shape, bits_qk: int, bits_pv: int, q, sq, k, sk, v, sv, row_ptr, col_idx) -> None:
    import torch

    kb = paro_nblocks(s)
    _require(q, "q", codes_shape(s, bits_qk, PARO_ROWS))
    _require(k, "k", codes_shape(s, bits_qk, PARO_ROWS))
    _require(v, "v", codes_shape(s, bits_pv, PARO_VT))
    for name, t in (("sq", sq), ("sk", sk), ("sv", sv)):
        if t is not None:
            _require(t, name, (s.B, s.nh, kb), torch.float32)
    _require(row_ptr, "row_ptr", (s.nh, kb + 1), torch.int32)
    _require(col_idx, "col_idx", None, torch.int32)


def _order_ptr(s: paro_shape, row_order):
    import torch

    if row_order is None:
        return None
    _require(row_order, "row_order", (s.B * s.nh * paro_nblocks(s),), torch.int32)
    return _ptr(row_order)


def paro_sparse_attn_unpermuted(s: paro_shape, bits_qk: int, bits_pv: int, q, sq, k, sk, v, sv, row_ptr, col_idx, perm_ids, o,
                                row_order=None) -> None:
    _attn_operands(s, bits_qk, bits_pv, q, sq, k, sk, v, sv, row_ptr, col_idx)
    _require(o, "o", (s.B, s.nh, paro_ntokens(s), s.d))
    p = _perm_bytes(s, perm_ids)
    _check(lib().paro_sparse_attn_unpermuted(ctypes.byref(s), int(bits_qk), int(bits_pv), _ptr(q), _ptr(sq), _ptr(k), _ptr(sk), _ptr(v),
                                             _ptr(sv), _ptr(row_ptr), _ptr(col_idx) if col_idx.numel() else None,
                                             int(col_idx.numel()), _order_ptr(s, row_order), p.ctypes.data, _dtype_code(o), _ptr(o),
                                             _stream()))


def paro_sparse_attn_unpermuted_rawq(s: paro_shape, bits_pv: int, q, k, sk, v, sv, row_ptr, col_idx, perm_ids, o, row_order=None) -> None:
    """q: unquantized [B, nh, N, d] (fp32 or bf16, default order); k, v: 8-bit K codes (rows) and 8/4-bit V codes (transposed)."""
    import torch

    kb, n = paro_nblocks(s), paro_ntokens(s)
    _require(q, "q", (s.B, s.nh, n, s.d))
    _require(k, "k", codes_shape(s, 8, PARO_ROWS), torch.int8)
    _require(v, "v", codes_shape(s, bits_pv, PARO_VT), torch.int8)
    for name, t in (("sk", sk), ("sv", sv)):
        _require(t, name, (s.B, s.nh, kb), torch.float32)
    _require(row_ptr, "row_ptr", (s.nh, kb + 1), torch.int32)
    _require(col_idx, "col_idx", None, torch.int32)
    _require(o, "o", (s.B, s.nh, n, s.d))
    p = _perm_bytes(s, perm_ids)
    _check(lib().paro_sparse_attn_unpermuted_rawq(ctypes.byref(s), _dtype_code(q), int(bits_pv), _ptr(q), _ptr(k), _ptr(sk), _ptr(v),
                                                  _ptr(sv), _ptr(row_ptr), _ptr(col_idx) if col_idx.numel() else None,
                                                  int(col_idx.numel()), _order_ptr(s, row_order), p.ctypes.data, _dtype_code(o),
                                                  _ptr(o), _stream()))


def paro_sparse_attn(s: paro_shape, bits_qk: int, bits_pv: int, q, sq, k, sk, v, sv, row_ptr, col_idx, op, row_order=None) -> None:
    import torch

    kb, npad = paro_nblocks(s), paro_npad(s)
    _require(q, "q", codes_shape(s, bits_qk, PARO_ROWS))
    _require(k, "k", codes_shape(s, bits_qk, PARO_ROWS))
    _require(v, "v", codes_shape(s, bits_pv, PARO_VT))
    for name, t in (("sq", sq), ("sk", sk), ("sv", sv)):
        if t is not None:
            _require(t, name, (s.B, s.nh, kb), torch.float32)
    _require(row_ptr, "row_ptr", (s.nh, kb + 1), torch.int32)
    _require(col_idx, "col_idx", None, torch.int32)
    _require(op, "op", (s.B, s.nh, npad, s.d))
    _check(lib().paro_sparse_attn(ctypes.byref(s), int(bits_qk), int(bits_pv), _ptr(q), _ptr(sq), _ptr(k), _ptr(sk), _ptr(v),
                                  _ptr(sv), _ptr(row_ptr), _ptr(col_idx) if col_idx.numel() else None, int(col_idx.numel()),
                                  _order_ptr(s, row_order), _dtype_code(op), _ptr(op), _stream()))
