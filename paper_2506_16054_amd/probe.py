"""ctypes binding of lib/libparo_probe.so, the measurement aids of bench.py (csrc/probe/): the matrix
rate the GPU sustains, the issue cost of single vector-ALU instructions, and a register-only replica
of one live block of the INT8 attention kernel.  Not part of the product library; nothing under
``binding`` or ``pipeline`` loads it.

    python -m paper_2506_16054_amd.probe                      # prints the issue-cost table as markdown
    python -m paper_2506_16054_amd.probe --timeline flux [records.npy]   # when the wavefronts of one attention launch start and end

The second form loads lib/libparo_timeline.so (the product sources with sparse_attn.hip compiled under
-DPARO_TIMELINE=1) in place of the product library, in this process only.
"""
from __future__ import annotations

import ctypes
import os
import sys

LIBPATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libparo_probe.so")
_lib = None

# parts of the block replica that can be left out (paro_probe_block), and their size per wave-block at d = 64
BLOCK_PARTS = {
    "all": 63,
    "without the 8 matrix instructions": 62,
    "without the 32 exp2": 61,
    "without conversion + packing (16 cvt_pknorm + 8 perm -> 24 xor)": 59,
    "without the row maximum (16 max3)": 55,
    "without the accumulator update (60 of 64 sub/fma)": 47,
    "without the row sum (31 add)": 31,
    "logit fma and bookkeeping only": 0,
}


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        import torch  # noqa: F401  (first: the library must bind to the HIP runtime that torch has loaded)

        if not os.path.exists(LIBPATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2506_16054_amd.build`" % LIBPATH)
        L = ctypes.CDLL(LIBPATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        L.paro_probe_mfma.restype = i64
        L.paro_probe_mfma.argtypes = [i32, i32, vp, i64, vp]
        L.paro_probe_last_error.restype = ctypes.c_char_p
        L.paro_probe_issue_kinds.restype = i32
        L.paro_probe_issue_name.restype = ctypes.c_char_p
        L.paro_probe_issue_name.argtypes = [i32]
        L.paro_probe_issue.argtypes = [i32, i32, i32, i32, i32, vp, vp, i64, vp]
        L.paro_probe_block.argtypes = [i32, i32, i32, i32, vp, vp, i64, vp]
        L.paro_probe_pair.argtypes = [i32, i32, i32, vp, vp, i64, vp]
        L.paro_probe_copy.restype = i64
        L.paro_probe_copy.argtypes = [vp, vp, i64, i32, i32, vp]
        _lib = L
    return _lib


def _stream() -> int:
    import torch

    return torch.cuda.current_stream().cuda_stream


def compute_units() -> int:
    import torch

    return int(torch.cuda.get_device_properties(0).multi_processor_count)


def kinds():
    L = lib()
    return [L.paro_probe_issue_name(k).decode() for k in range(L.paro_probe_issue_kinds())]


def sustained_mfma_rate(bits: int) -> float:
    """TOP/s (bits 8) or TFLOP/s (bits 16) of a kernel that only issues dense matrix instructions."""
    import torch

    out = torch.empty(4096, dtype=torch.int32, device="cuda:0")

    def launch():
        ops = lib().paro_probe_mfma(int(bits), 4000, out.data_ptr(), out.numel(), _stream())
        if ops < 0:
            raise RuntimeError("paro_probe_mfma failed with status %d: %s" % (ops, lib().paro_probe_last_error().decode()))
        return ops

    for _ in range(3):
        launch()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    ops = sum(launch() for _ in range(10))
    e1.record()
    torch.cuda.synchronize()
    return ops / (e0.elapsed_time(e1) * 1e-3) / 1e12


def sustained_copy_rate(write_every: int, mbytes_read: int = 512, groups_per_cu: int = 8) -> float:
    """TB/s (bytes read + written per second) of a plain streaming copy: write_every 1 = one byte written per byte
    read, 2 = one per two (the quantizer's mix).  Best of the workgroup counts tried."""
    import torch

    n_read = mbytes_read * (1 << 20) // 16
    src = torch.empty(n_read * 16, dtype=torch.uint8, device="cuda:0").fill_(3)
    dst = torch.empty(n_read * 16 // write_every, dtype=torch.uint8, device="cuda:0")
    best = 0.0
    for per_cu in (groups_per_cu, 2 * groups_per_cu, 4 * groups_per_cu):
        groups = compute_units() * per_cu

        def launch():
            moved = lib().paro_probe_copy(src.data_ptr(), dst.data_ptr(), n_read, write_every, groups, _stream())
            if moved < 0:
                raise RuntimeError("paro_probe_copy failed with status %d: %s" % (moved, lib().paro_probe_last_error().decode()))
            return moved

        for _ in range(3):
            launch()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        moved = sum(launch() for _ in range(10))
        e1.record()
        torch.cuda.synchronize()
        best = max(best, moved / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return best


def _times(launch, per_wave_work: float, timed_per_simd: int):
    """Runs ``launch(times, sink, capacity)`` twice (the second run is read).  The SIMD's arbiter serves its
    oldest wavefront first, so the wavefronts of a SIMD finish one after the other and the LAST one's elapsed
    cycles are the time the SIMD needed for all of them: cost per unit of work = that / (work per wavefront x
    timed wavefronts per SIMD).  Returns (cost in shader cycles, clock in GHz, matrix instructions a companion
    wavefront issued per 1000 cycles meanwhile or None)."""
    import torch

    cap = 4096 * 4
    times = torch.zeros((cap, 4), dtype=torch.int64, device="cuda:0")
    sink = torch.zeros((cap,), dtype=torch.int32, device="cuda:0")
    n = 0
    for _ in range(2):
        times.zero_()
        n = launch(times.data_ptr(), sink.data_ptr(), cap)
        if n < 0:
            raise RuntimeError("probe launch failed with status %d: %s" % (n, lib().paro_probe_last_error().decode()))
        torch.cuda.synchronize()
    full = times[:n].cpu().numpy()
    timed = full[full[:, 0] > 0]
    comp = full[full[:, 0] == 0]
    # per SIMD (placement register: XCC, shader engine, array, compute unit, SIMD): the slowest timed wavefront
    hw = timed[:, 3] & 0xFFFFFFFF
    simd = ((timed[:, 3] >> 32) & 0xF) << 20 | (hw & 0xFFF0)
    last = {}
    first = {}
    count = {}
    for key, c in zip(simd.tolist(), timed[:, 0].tolist()):
        last[key] = max(last.get(key, 0), c)
        first[key] = min(first.get(key, c), c)
        count[key] = count.get(key, 0) + 1
    if set(count.values()) != {timed_per_simd}:
        raise RuntimeError("expected %d timed wavefronts on every SIMD, found %s" % (timed_per_simd, sorted(set(count.values()))))
    import numpy as np

    cycles = float(np.median(list(last.values())))
    ghz = float((timed[:, 0] / (timed[:, 1] * 10.0)).mean())  # ticks of 10 ns
    mfma_rate = None
    if len(comp):
        mfma_rate = float(comp[:, 1].mean()) * 8.0 / cycles * 1000.0
    return cycles / (per_wave_work * timed_per_simd), ghz, mfma_rate, float(np.median(list(first.values()))) / per_wave_work


def issue_cost(kind: int, waves_per_simd: int, with_mfma: bool = False, iters: int = 8000):
    """(shader cycles one wavefront instruction of ``kind`` costs its SIMD, clock in GHz, companion matrix rate)."""
    timed = waves_per_simd - (1 if with_mfma else 0)
    return _times(lambda t, s, cap: lib().paro_probe_issue(kind, compute_units(), waves_per_simd, iters, int(with_mfma), t, s, cap, _stream()),
                  iters * 32.0, timed)


def block_cost(parts: int, waves_per_simd: int, iters: int = 1500):
    """(shader cycles one replica block costs its SIMD, clock in GHz, None)."""
    return _times(lambda t, s, cap: lib().paro_probe_block(parts, compute_units(), waves_per_simd, iters, t, s, cap, _stream()),
                  float(iters), waves_per_simd)


PAIR_MODES = {
    0: "program order: QK(0) softmax(0) PV(0) update(0) QK(1) softmax(1) PV(1) update(1)",
    1: "QK(1) among softmax(0), PV(0) among softmax(1), PV(1) among update(0)",
    2: "as 1, and QK(0) of the next visit among update(1)",
    3: "one matrix instruction in front of every 8 x (logit fma, exp2): QK(1) in softmax(0), PV(0) in softmax(1)",
    4: "the pieces of 3 in the same order, matrix instructions not moved in",
    5: "as 3, skewed: each matrix instruction directly followed by 8 exp2, the next run's 8 logit fma behind them",
}


def pair_cost(mode: int, iters: int = 1500):
    """(shader cycles per half-block per SIMD of the two-halves replica, two wavefronts per SIMD, clock, None, first)."""
    return _times(lambda t, s, cap: lib().paro_probe_pair(mode, compute_units(), iters, t, s, cap, _stream()), 2.0 * iters, 2)


def issue_table() -> dict:
    """All measurements behind profiles/valu_issue_costs.md as a dictionary."""
    names = kinds()
    single = {name: {w: issue_cost(k, w) for w in (2, 3, 4)} for k, name in enumerate(names)}
    beside = {name: issue_cost(k, 4, with_mfma=True) for k, name in enumerate(names) if "mfma" not in name}
    blocks = {label: {w: block_cost(parts, w) for w in (2, 3, 4)} for label, parts in BLOCK_PARTS.items()}
    pairs = {label: pair_cost(mode) for mode, label in PAIR_MODES.items()}
    return {"single": single, "beside_mfma": beside, "block": blocks, "pair": pairs}


def markdown(tab: dict) -> str:
    out = ["| instruction | cycles at 2 waves/SIMD | 3 | 4 | pace of the first wave to finish, 2 waves/SIMD | clock GHz | 3 waves + a wave of matrix instructions: cycles | matrix instructions per 1000 cycles meanwhile (alone: 30.3) |",
           "|---|---|---|---|---|---|---|---|"]
    for name, row in tab["single"].items():
        b = tab["beside_mfma"].get(name)
        out.append("| `%s` | %.2f | %.2f | %.2f | %.2f | %.2f | %s | %s |" % (name, row[2][0], row[3][0], row[4][0], row[2][3], row[3][1],
                                                                        "%.2f" % b[0] if b else "-", "%.1f" % b[2] if b else "-"))
    out += ["", "| block replica (cycles per wave-block per SIMD) | 2 waves/SIMD | 3 | 4 | clock GHz |", "|---|---|---|---|---|"]
    for label, row in tab["block"].items():
        out.append("| %s | %.0f | %.0f | %.0f | %.2f |" % (label, row[2][0], row[3][0], row[4][0], row[3][1]))
    out += ["", "| two-halves replica, 2 waves/SIMD (cycles per half-block per SIMD) | cycles | first wave to finish | clock GHz |", "|---|---|---|---|"]
    for label, row in tab["pair"].items():
        out.append("| %s | %.0f | %.0f | %.2f |" % (label, row[0], row[3], row[1]))
    return "\n".join(out)


def timeline(workload: str, step_us: float | None = None, records_path: str | None = None) -> str:
    """Markdown summary of one attention launch of the named workload: per class of row block (few / many column
    blocks) when its wavefronts start and end and what a block costs them, and how many wavefronts are resident over time."""
    import numpy as np
    import torch

    from . import binding as pb
    from . import workloads as wl
    from .pipeline import ParoAttention

    if pb._lib is not None:
        raise RuntimeError("the product library is already loaded in this process")
    pb.LIBPATH = os.path.join(os.path.dirname(LIBPATH), "libparo_timeline.so")
    w = wl.WORKLOADS[workload]
    s = pb.shape_of(w)
    perm_ids = wl.make_perm_ids(w)
    bitmask = wl.pack_bitmask(wl.make_block_masks(w, lambda pid: pb.paro_perm_index(s, pid), perm_ids))
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    q = torch.empty((w.B, w.nh, w.N, w.d), dtype=tdt, device=dev)
    k, v = torch.empty_like(q), torch.empty_like(q)
    for h in range(w.nh):
        for dst, src in zip((q, k, v), wl.make_head_qkv(w, 0, h)):
            dst[0, h] = torch.from_numpy(src).to(dev)
    pa = ParoAttention(s, perm_ids, bitmask, w.bits_qk, w.bits_pv, tdt, dev)
    pa.prepare_fused_qkv(q, k, v)  # the launches bench.py times
    for _ in range(60):
        pa.attend_fused()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    pa.attend_fused()
    e1.record()
    torch.cuda.synchronize()
    waves_per_wg = 4 if (w.d == 128 and w.bits_qk == 8 and w.bits_pv == 8) else 1
    if not (w.block == 64 and w.bits_qk == 8 and (waves_per_wg == 4 or w.d == 64)):
        raise RuntimeError("only the one-wavefront (d = 64) and the four-wavefront (d = 128, 8-bit) kernels record a timeline")
    slots = waves_per_wg * w.B * w.nh * w.k
    rec = np.zeros((slots, 8), dtype=np.int64)
    read = pb.lib().paro_timeline_read
    read.restype = ctypes.c_int64
    khz = read(ctypes.c_void_p(rec.ctypes.data), ctypes.c_int64(slots))
    if khz <= 0:
        raise RuntimeError("paro_timeline_read: %d" % khz)
    if records_path:
        # [slot][start clock, end clock, column blocks, shader cycles of phases 0..3 of the block loop, of the part in front of
        # it]; slot = row block x wavefronts per block + wavefront
        np.save(records_path, rec)
    t0 = rec[:, 0].min()
    start, end, cnt = (rec[:, 0] - t0) * 1e3 / khz, (rec[:, 1] - t0) * 1e3 / khz, rec[:, 2]
    heavy = 2 * cnt > w.k
    out = ["workload %s: %d wavefronts (%d per row block), launch %.1f us by HIP events, %.1f us from the first start to the last end"
           % (workload, slots, waves_per_wg, 1e3 * e0.elapsed_time(e1), end.max()), "",
           "| row blocks | wavefronts | column blocks | start us (min / median / max) | end us (min / median / max) | us per block (median) |",
           "|---|---|---|---|---|---|"]
    for label, sel in (("more than half of all column blocks live", heavy), ("the others", ~heavy)):
        if sel.any():
            per = ((end - start) / np.maximum(cnt, 1))[sel]
            out.append("| %s | %d | %d ... %d | %.1f / %.1f / %.1f | %.1f / %.1f / %.1f | %.2f |" % (
                label, sel.sum(), cnt[sel].min(), cnt[sel].max(), start[sel].min(), np.median(start[sel]), start[sel].max(),
                end[sel].min(), np.median(end[sel]), end[sel].max(), np.median(per)))
    if waves_per_wg == 4:  # the four-wavefront kernel also records where a block's cycles go
        names = ("K reads, QK^T products, row maximum, share of the tile exponent", "wait for the tiles and the other wavefronts (barrier)",
                 "exponentials, row sum, codes", "PV products, accumulator update, next requests")
        out += ["", "| shader cycles per block (median over the wavefronts) | " + " | ".join(names) + " | sum | in front of the loop (per wavefront) |",
                "|---|---|---|---|---|---|---|"]
        for label, sel in (("more than half of all column blocks live", heavy), ("the others, started in the first 5 us", ~heavy & (start < 5.0)),
                           ("the others, started later", ~heavy & (start >= 5.0))):
            if sel.any():
                per = rec[sel, 3:7] / np.maximum(cnt[sel], 1)[:, None]
                out.append("| %s | %s | %.0f | %.0f |" % (label, " | ".join("%.0f" % x for x in np.median(per, axis=0)), np.median(per.sum(1)), np.median(rec[sel, 7])))
    # the kernels give launch positions [x * per_xcd, (x + 1) * per_xcd) to XCD x; row_order maps positions to row blocks
    total = w.B * w.nh * w.k
    per_xcd = (total + 7) // 8
    order = pa.row_order.cpu().numpy() if pa.row_order is not None else np.arange(total)
    xcd_of_item = np.empty(total, dtype=np.int64)
    xcd_of_item[order] = np.arange(total) // per_xcd
    xcd = np.repeat(xcd_of_item, waves_per_wg)
    out += ["", "| XCD | row blocks | column blocks visited | last start us | last end us | median end us of its last 5 % of wavefronts to end |", "|---|---|---|---|---|---|"]
    for x in range(8):
        sel = xcd == x
        if sel.any():
            ends = np.sort(end[sel])
            out.append("| %d | %d | %d | %.1f | %.1f | %.1f |" % (x, sel.sum() // waves_per_wg, cnt[sel].sum() // waves_per_wg, start[sel].max(), ends[-1],
                                                                np.median(ends[-max(1, len(ends) // 20):])))
    out += ["", "| at us | wavefronts resident | of them: many-block rows | wavefronts started so far |", "|---|---|---|---|"]
    if step_us is None:  # about forty rows
        step_us = max(5.0, 5.0 * round(end.max() / 200.0))
    for t in np.arange(0.0, end.max() + step_us, step_us):
        run = (start <= t) & (end > t)
        out.append("| %.0f | %d | %d | %d |" % (t, run.sum(), (run & heavy).sum(), (start <= t).sum()))
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "--timeline":
        sys.stdout.write(timeline(sys.argv[2] if len(sys.argv) > 2 else "flux", records_path=sys.argv[3] if len(sys.argv) > 3 else None) + "\n")
        sys.exit(0)
    sys.stdout.write(markdown(issue_table()) + "\n")
    sys.stdout.write("\n| plain streaming copy, 512 MB read | TB/s (read + written) |\n|---|---|\n")
    sys.stdout.write("| one byte written per byte read | %.2f |\n| one byte written per two read (the quantizer's mix) | %.2f |\n"
                     % (sustained_copy_rate(1), sustained_copy_rate(2)))
