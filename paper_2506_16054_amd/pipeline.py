"""Device-side plumbing for one attention layer: owns the intermediate buffers and enqueues the
library calls of the hot path in order (reorder -> quantize -> block-sparse attention ->
inverse reorder) on torch's current stream.  No arithmetic happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as pb


class ParoAttention:
    """Buffers and block list for one problem shape; ``run(q, k, v)`` returns O [B, nh, N, d]."""

    def __init__(self, shape: pb.paro_shape, perm_ids, bitmask: np.ndarray, bits_qk: int, bits_pv: int,
                 dtype: torch.dtype, device="cuda:0"):
        self.s = shape
        self.bits_qk, self.bits_pv = bits_qk, bits_pv
        self.dtype = dtype
        self.dev = torch.device(device)
        self.perm_ids = np.ascontiguousarray(perm_ids, dtype=np.uint8)
        self.N, self.k, self.npad = pb.paro_ntokens(shape), pb.paro_nblocks(shape), pb.paro_npad(shape)
        row_ptr, col_idx = pb.paro_mask_to_blocklist(shape.nh, self.k, bitmask)
        self.h_row_ptr, self.h_col_idx = row_ptr, col_idx
        self.row_ptr = torch.from_numpy(row_ptr).to(self.dev)
        self.col_idx = torch.from_numpy(col_idx).to(self.dev)
        self.live_blocks = int(col_idx.size) * shape.B
        self.h_row_order = pb.paro_schedule_rows(shape, bits_qk, bits_pv, row_ptr)
        self.row_order = torch.from_numpy(self.h_row_order).to(self.dev)
        B, nh, d = shape.B, shape.nh, shape.d
        ct_qk = torch.bfloat16 if bits_qk == 16 else torch.int8
        ct_pv = torch.bfloat16 if bits_pv == 16 else torch.int8
        z = dict(device=self.dev)
        self.xp = [torch.empty((B, nh, self.npad, d), dtype=dtype, **z) for _ in range(3)]
        self.qc = torch.empty(pb.codes_shape(shape, bits_qk, pb.PARO_ROWS), dtype=ct_qk, **z)
        self.kc = torch.empty(pb.codes_shape(shape, bits_qk, pb.PARO_ROWS), dtype=ct_qk, **z)
        self.vc = torch.empty(pb.codes_shape(shape, bits_pv, pb.PARO_VT), dtype=ct_pv, **z)
        self.sq, self.sk, self.sv = (torch.empty((B, nh, self.k), dtype=torch.float32, **z) for _ in range(3))
        self.op = torch.empty((B, nh, self.npad, d), dtype=dtype, **z)
        self.o = torch.empty((B, nh, self.N, d), dtype=dtype, **z)

    def use_blocklist(self, row_ptr, col_idx, row_order=None) -> None:
        """Attend with another block list (device tensors), e.g. a slot of a MaskPrefetcher.  The
        length of ``col_idx`` is passed to the kernels as the bound of the list."""
        self.row_ptr, self.col_idx, self.row_order = row_ptr, col_idx, row_order

    def prepare(self, q, k, v) -> None:
        """paro_permute + paro_quantize for Q, K (row layout) and V (transposed-block layout)."""
        s = self.s
        for src, xp in zip((q, k, v), self.xp):
            pb.paro_permute(s, self.perm_ids, src, xp)
        if self.bits_qk == 16 and self.dtype == torch.bfloat16:
            self.qc, self.kc = self.xp[0], self.xp[1]  # already bf16 rows: nothing to convert
        else:
            pb.paro_quantize(s, self.bits_qk, pb.PARO_ROWS, self.xp[0], self.qc, self.sq)
            pb.paro_quantize(s, self.bits_qk, pb.PARO_ROWS, self.xp[1], self.kc, self.sk)
        pb.paro_quantize(s, self.bits_pv, pb.PARO_VT, self.xp[2], self.vc, self.sv)

    def attend(self) -> None:
        pb.paro_sparse_attn(self.s, self.bits_qk, self.bits_pv, self.qc, self.sq, self.kc, self.sk, self.vc, self.sv,
                            self.row_ptr, self.col_idx, self.op, self.row_order)

    def finish(self):
        pb.paro_unpermute(self.s, self.perm_ids, self.op, self.o)
        return self.o

    def run(self, q, k, v):
        """The path as five separate steps (reorder, quantize, attention, inverse reorder)."""
        self.prepare(q, k, v)
        self.attend()
        return self.finish()

    # ---- fused form: the reorder lives in the quantizer's load addresses and in the attention
    # kernel's store addresses; four launches, no reordered intermediates
    def _fused_buffers(self):
        if not hasattr(self, "_fq"):
            s, z = self.s, dict(device=self.dev)
            ct = torch.bfloat16 if self.bits_qk == 16 else torch.int8
            self._fq = torch.empty(pb.codes_shape(s, self.bits_qk, pb.PARO_ROWS), dtype=ct, **z)
            self._fk = torch.empty(pb.codes_shape(s, self.bits_qk, pb.PARO_ROWS), dtype=ct, **z)
        return self._fq, self._fk

    def prepare_fused(self, q, k, v) -> None:
        s = self.s
        fq, fk = self._fused_buffers()
        pb.paro_permute_quantize(s, self.bits_qk, pb.PARO_ROWS, self.perm_ids, q, fq, self.sq)
        pb.paro_permute_quantize(s, self.bits_qk, pb.PARO_ROWS, self.perm_ids, k, fk, self.sk)
        pb.paro_permute_quantize(s, self.bits_pv, pb.PARO_VT, self.perm_ids, v, self.vc, self.sv)

    def prepare_fused_qkv(self, q, k, v) -> None:
        """prepare_fused in one launch (Q, K and V quantized by one grid)."""
        fq, fk = self._fused_buffers()
        pb.paro_permute_quantize_qkv(self.s, self.bits_qk, self.bits_pv, self.perm_ids, q, k, v, fq, self.sq, fk, self.sk, self.vc, self.sv)

    def attend_fused(self):
        fq, fk = self._fused_buffers()
        pb.paro_sparse_attn_unpermuted(self.s, self.bits_qk, self.bits_pv, fq, self.sq, fk, self.sk, self.vc, self.sv,
                                       self.row_ptr, self.col_idx, self.perm_ids, self.o, self.row_order)
        return self.o

    def run_fused(self, q, k, v):
        self.prepare_fused(q, k, v)
        return self.attend_fused()

    # ---- optional pre-conditioning of K: the per-channel mean over the tokens is removed in the quantizer's loads
    def prepare_fused_smooth_k(self, q, k, v) -> None:
        """prepare_fused with paro_k_channel_mean + paro_permute_quantize_smoothed for K (integer K codes only)."""
        s = self.s
        fq, fk = self._fused_buffers()
        if not hasattr(self, "k_mean"):
            self.k_mean = torch.empty((s.B, s.nh, s.d), dtype=torch.float32, device=self.dev)
        pb.paro_k_channel_mean(s, k, self.k_mean)
        pb.paro_permute_quantize(s, self.bits_qk, pb.PARO_ROWS, self.perm_ids, q, fq, self.sq)
        pb.paro_permute_quantize_smoothed(s, self.bits_qk, self.perm_ids, k, self.k_mean, fk, self.sk)
        pb.paro_permute_quantize(s, self.bits_pv, pb.PARO_VT, self.perm_ids, v, self.vc, self.sv)

    def run_fused_smooth_k(self, q, k, v):
        self.prepare_fused_smooth_k(q, k, v)
        return self.attend_fused()

    # ---- shortest form (block 64, 8-bit QK): Q is reordered and quantized inside the attention kernel,
    # by the workgroup that owns the row block; three launches
    @property
    def can_fuse_q(self) -> bool:
        return self.bits_qk == 8 and self.s.block == 64

    def prepare_kv(self, k, v) -> None:
        _, fk = self._fused_buffers()
        pb.paro_permute_quantize(self.s, 8, pb.PARO_ROWS, self.perm_ids, k, fk, self.sk)
        pb.paro_permute_quantize(self.s, self.bits_pv, pb.PARO_VT, self.perm_ids, v, self.vc, self.sv)

    def attend_rawq(self, q):
        _, fk = self._fused_buffers()
        pb.paro_sparse_attn_unpermuted_rawq(self.s, self.bits_pv, q, fk, self.sk, self.vc, self.sv, self.row_ptr, self.col_idx,
                                            self.perm_ids, self.o, self.row_order)
        return self.o

    def run_rawq(self, q, k, v):
        self.prepare_kv(k, v)
        return self.attend_rawq(q)


class MaskPrefetcher:
    """Two device slots for the block list of the attention call at hand and of the next one
    (paper Sec. 4.2 (1), App. C "Overhead of Prefetch").  All masks stay in pinned host memory, each as
    one record [bitmask | row offsets | launch order]: the offsets and the order are functions of the
    static mask and are computed once, here, when the store is built.  ``prefetch(slot, t)`` copies
    record ``t`` to slot ``slot`` on a second stream (one transfer, on the copy engine) and writes the
    column list there with paro_blocklist_cols_device (one small kernel), while the compute stream is
    busy with the other slot.  Ordering is by events only:

        slot.ready   recorded on the copy stream after the expansion; the compute stream waits on
                     it in ``acquire`` before the attention call that reads the slot;
        slot.free    recorded on the compute stream in ``release`` after that attention call; the
                     copy stream waits on it before it overwrites the slot.

    ``lists_on_host=True`` trades host memory for device work: the record also holds the expanded column list
    (4 bytes per live block instead of 1 bit per block), ``prefetch`` is the one transfer and no kernel runs on
    the second stream at all.

    Both streams have the default priority.  No arithmetic happens here."""

    def __init__(self, shape: pb.paro_shape, h_bitmasks: np.ndarray, h_row_orders=None, cap=None, device="cuda:0",
                 lists_on_host: bool = False):
        self.lists_on_host = bool(lists_on_host)
        self.s = shape
        self.dev = torch.device(device)
        self.k = pb.paro_nblocks(shape)
        nh, k = shape.nh, self.k
        nbytes = (k * k + 7) // 8
        bm = np.ascontiguousarray(h_bitmasks, dtype=np.uint8)
        if bm.ndim != 3 or bm.shape[1:] != (nh, nbytes):
            raise pb.ParoError(pb.PARO_EINVAL, "h_bitmasks has shape %s, expected (T, %d, %d)" % (bm.shape, nh, nbytes))
        self.T = bm.shape[0]
        n_order = shape.B * nh * k
        ro = None
        if h_row_orders is not None:
            ro = np.ascontiguousarray(h_row_orders, dtype=np.int32)
            if ro.shape != (self.T, n_order):
                raise pb.ParoError(pb.PARO_EINVAL, "h_row_orders has shape %s, expected (%d, %d)" % (ro.shape, self.T, n_order))
        # record layout, every part 16-byte aligned
        align = lambda n: (n + 15) // 16 * 16
        self._off_ptr = align(nh * nbytes)
        self._off_ord = self._off_ptr + align(nh * (k + 1) * 4)
        self._off_col = self._off_ord + (align(n_order * 4) if ro is not None else 0)
        lists = [pb.paro_mask_to_blocklist(nh, k, bm[t]) for t in range(self.T)]
        nnz_max = max(1, max(int(ci.size) for _, ci in lists))
        self.cap = int(cap) if cap is not None else nnz_max
        if self.cap < nnz_max:
            raise pb.ParoError(pb.PARO_EINVAL, "cap=%d is smaller than the longest block list (%d)" % (self.cap, nnz_max))
        self._rec = self._off_col + (align(self.cap * 4) if self.lists_on_host else 0)
        host = np.zeros((self.T, self._rec), np.uint8)
        for t, (row_ptr, col_idx) in enumerate(lists):
            host[t, : nh * nbytes] = bm[t].reshape(-1)
            host[t, self._off_ptr: self._off_ptr + row_ptr.nbytes] = row_ptr.reshape(-1).view(np.uint8)
            if ro is not None:
                host[t, self._off_ord: self._off_ord + ro[t].nbytes] = ro[t].view(np.uint8)
            if self.lists_on_host:
                host[t, self._off_col: self._off_col + col_idx.nbytes] = col_idx.view(np.uint8)
        self.h_records = torch.empty(host.shape, dtype=torch.uint8, pin_memory=True)
        self.h_records.copy_(torch.from_numpy(host))
        self.copy_stream = torch.cuda.Stream(self.dev)
        z = dict(device=self.dev)
        self.slots = []
        for _ in range(2):
            rec = torch.zeros((self._rec,), dtype=torch.uint8, **z)
            self.slots.append({
                "record": rec,
                "bitmask": rec[: nh * nbytes].view(nh, nbytes),
                "row_ptr": rec[self._off_ptr: self._off_ptr + nh * (k + 1) * 4].view(torch.int32).view(nh, k + 1),
                "row_order": None if ro is None else rec[self._off_ord: self._off_ord + n_order * 4].view(torch.int32),
                "col_idx": (rec[self._off_col: self._off_col + self.cap * 4].view(torch.int32) if self.lists_on_host
                            else torch.zeros((self.cap,), dtype=torch.int32, **z)),
                "ready": torch.cuda.Event(),
                "free": torch.cuda.Event(),
            })
        torch.cuda.current_stream().synchronize()  # the slots exist before the copy stream touches them

    def prefetch(self, slot: int, t: int) -> None:
        """Enqueue, on the copy stream, the load of record ``t`` into ``slot`` and the expansion of its mask."""
        sl = self.slots[slot]
        with torch.cuda.stream(self.copy_stream):
            self.copy_stream.wait_event(sl["free"])
            sl["record"].copy_(self.h_records[t], non_blocking=True)
            if not self.lists_on_host:
                pb.paro_blocklist_cols_device(self.s.nh, self.k, sl["bitmask"], sl["row_ptr"], sl["col_idx"])
            sl["ready"].record(self.copy_stream)

    def acquire(self, slot: int):
        """Make the current stream wait for the slot's block list; returns (row_ptr, col_idx, row_order)."""
        sl = self.slots[slot]
        torch.cuda.current_stream().wait_event(sl["ready"])
        return sl["row_ptr"], sl["col_idx"], sl["row_order"]

    def release(self, slot: int) -> None:
        """Call after the attention launch that read the slot: the slot may be refilled once it is done."""
        self.slots[slot]["free"].record(torch.cuda.current_stream())


def calibrate(shape: pb.paro_shape, q, k, eps: float = 1e-3, sigma: float = 0.9, alpha: float = 0.5, density: float = 0.3):
    """Offline calibration of one attention layer (paper Sec. 4.1, Sec. 4.2 (3)) from calibration
    samples q, k [B, nh, N, d]: enqueues the library calls and returns device tensors
    ``perm_ids`` uint8 [nh], ``bitmask`` uint8 [nh, ceil(k*k/8)], ``m_sparse``, ``m_quant``,
    ``m_combined`` float32 [6, nh], and the chosen orders' ``block_sum`` [B, nh, k, k].  The only
    host step is the copy of the nh chosen order ids, which the reorder entry points take on the host."""
    dev = q.device
    nh, kb = shape.nh, pb.paro_nblocks(shape)
    z = dict(device=dev)
    q16 = torch.empty(pb.codes_shape(shape, 16, pb.PARO_ROWS), dtype=torch.bfloat16, **z)
    k16 = torch.empty_like(q16)
    unused_scales = torch.empty((shape.B, nh, kb), dtype=torch.float32, **z)
    bsum = torch.empty((shape.B, nh, kb, kb), dtype=torch.float32, **z)
    bmax = torch.empty_like(bsum)
    bcnt = torch.empty((shape.B, nh, kb, kb), dtype=torch.int32, **z)
    ms = torch.empty((6, nh), dtype=torch.float32, **z)
    mq = torch.empty_like(ms)
    mc = torch.empty_like(ms)
    perm_ids = torch.empty((nh,), dtype=torch.uint8, **z)
    bitmask = torch.empty((nh, (kb * kb + 7) // 8), dtype=torch.uint8, **z)

    def stats_for(ids):
        pb.paro_permute_quantize(shape, 16, pb.PARO_ROWS, ids, q, q16, unused_scales)
        pb.paro_permute_quantize(shape, 16, pb.PARO_ROWS, ids, k, k16, unused_scales)
        pb.paro_calib_block_stats(shape, q16, k16, eps, bsum, bmax, bcnt)

    for t in range(6):
        stats_for(np.full(nh, t, np.uint8))
        pb.paro_calib_metrics(shape, bsum, bmax, bcnt, sigma, ms[t], mq[t])
    pb.paro_calib_choose(nh, ms, mq, alpha, mc, perm_ids)
    h_perm_ids = perm_ids.cpu().numpy()  # synchronises: the reorder calls take the ids on the host
    stats_for(h_perm_ids)
    pb.paro_calib_mask(shape, bsum, density, bitmask)
    return {"perm_ids": perm_ids, "h_perm_ids": h_perm_ids, "bitmask": bitmask, "m_sparse": ms, "m_quant": mq, "m_combined": mc,
            "block_sum": bsum}
