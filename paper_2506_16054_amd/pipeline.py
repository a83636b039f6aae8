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

    def attend_fused(self):
        fq, fk = self._fused_buffers()
        pb.paro_sparse_attn_unpermuted(self.s, self.bits_qk, self.bits_pv, fq, self.sq, fk, self.sk, self.vc, self.sv,
                                       self.row_ptr, self.col_idx, self.perm_ids, self.o, self.row_order)
        return self.o

    def run_fused(self, q, k, v):
        self.prepare_fused(q, k, v)
        return self.attend_fused()
