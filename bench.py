"""Benchmark of the PAROAttention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

One "step" is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: reorder Q, K, V -> block quantize -> block-sparse INT8 attention -> inverse
reorder, in the fused form (the reorder rides on the quantizer's loads and on the attention
kernel's stores; Q, K and V are quantized by one launch: two launches per step).  The block list of the static mask is built once, outside
the timed region, as the method does offline.  The same path as five separate steps is timed
afterwards for reference (`separate_steps_ms`).  Prints ONE JSON line.  The headline workload is the CogVideoX-5B-shaped
layer: 48 heads, N = 17550, d = 64, 30 % density, INT8 QK^T and INT8 PV.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0  # MI355X dense INT8 MFMA, published: 5.0 POP/s
PEAK_BF16_TFLOPS = 2500.0


def attention_kernel_symbol(w):
    """(mangled symbol, demangled name as the profiler prints it, wavefronts per row-block visit, wavefronts per SIMD)
    of the kernel that paro_sparse_attn launches for an integer workload."""
    t, tn = ("t", "unsigned short") if w.dtype == "bf16" else ("f", "float")
    if w.block == 64 and w.d == 64 and w.bits_qk == 8:
        return ("_ZN4paro18attn_i8_w64_kernelILi%dE%sLi0EEEvNS_8AttnArgsE" % (w.bits_pv, t),
                "paro::attn_i8_w64_kernel<%d, %s, 0>" % (w.bits_pv, tn), 1, 2)
    if w.block == 64 and w.d == 64 and w.bits_qk == 4:
        return ("_ZN4paro22attn_i8_w64_qk4_kernelILi%dE%sEEvNS_8AttnArgsE" % (w.bits_pv, t),
                "paro::attn_i8_w64_qk4_kernel<%d, %s>" % (w.bits_pv, tn), 1, 2)
    if w.block == 64 and w.d == 128 and w.bits_qk == 8 and w.bits_pv == 8:
        return ("_ZN4paro18attn_i8_q16_kernelI%sEEvNS_8AttnArgsE" % t, "paro::attn_i8_q16_kernel<%s>" % tn, 4, 4)
    return ("_ZN4paro14attn_i8_kernelILi%dELi%dELi%dELi%dE%sLi0EEEvNS_8AttnArgsE" % (w.block, w.d, w.bits_qk, w.bits_pv, t),
            "paro::attn_i8_kernel<%d, %d, %d, %d, %s, 0>" % (w.block, w.d, w.bits_qk, w.bits_pv, tn), w.block // 32, 3 if w.d == 64 else 2)


def static_loop_counts(w):
    """Vector instructions per loop iteration (one visit of a live block by one wavefront) of the built attention
    kernel, by issue class, from the compiler's listing (lib/attn_loop_counts.json, written by the build).  Of the
    kernel's loop variants the one with the fewest instructions is the folded-exponent form that 8-bit P codes take."""
    path = os.path.join(ROOT, "paper_2506_16054_amd", "lib", "attn_loop_counts.json")
    try:
        loops = json.load(open(path)).get(attention_kernel_symbol(w)[0])
    except OSError:
        return None
    if not loops:
        return None
    return min(loops, key=lambda c: sum(c.values()))


def recorded_counters(w, live_blocks):
    """SQ_INSTS_VALU per launch of the attention kernel and HBM bytes per launch, as recorded from rocprofv3 runs
    summarised under profiles/ - but only if that record is of the kernel this build launches: the summary must
    name the same kernel and its instruction count must agree (3 %) with the built kernel's loop.  Otherwise the
    record is reported as stale and not used."""
    import re

    out = {"valu_instructions": None, "traffic": None, "stale": None}
    _, name, waves, _ = attention_kernel_symbol(w)
    static = static_loop_counts(w)
    path = os.path.join(ROOT, "profiles", "attn_i8_%s_sq_counters.md" % w.name)
    try:
        text = open(path).read()
        m = re.search(r"\| SQ_INSTS_VALU \| ([0-9.e+]+) \|", text)
        if m and static:
            measured = float(m.group(1))
            expected = sum(static.values()) * live_blocks * waves
            out["stale"] = name not in text or abs(measured / expected - 1.0) > 0.03
            if not out["stale"]:
                out["valu_instructions"] = measured
    except OSError:
        pass
    path = os.path.join(ROOT, "profiles", "hot_path_%s_hbm_traffic.md" % w.name)
    try:
        text = open(path).read()
        m = re.search(r"traffic_bytes_per_launch paro_sparse_attn %s = (\d+)" % re.escape(w.name), text)
        if m and name in text:
            out["traffic"] = int(m.group(1))
    except OSError:
        pass
    return out


PROBE_OF_CLASS = {"fma": "v_fma_f32", "add_mul": "v_add_f32", "int_simple": "v_add_u32", "half_rate": "v_max3_i32",
                  "transcendental": "v_exp_f32", "permlane_swap": "v_permlane32_swap_b32", "mfma": "v_mfma_i32_32x32x32_i8",
                  "mfma_16x16": "v_mfma_i32_16x16x64_i8"}


def valu_issue_roofline(w, live_blocks, attn_ms, n_cus):
    """What binds the integer attention kernels: instruction issue.  Model time = sum over issue classes of
    (instructions of the class per loop iteration, from the compiler's listing) x (what one such wavefront
    instruction costs a SIMD, measured now by the issue probe at the kernel's occupancy, in nanoseconds at the clock
    the probe's load runs at) x iterations / SIMDs.  frac = model / measured: 1 means the kernel runs at the summed
    issue cost of its own instructions with nothing hidden and nothing lost."""
    from paper_2506_16054_amd import probe

    static = static_loop_counts(w)
    if not static:
        return None
    _, name, waves, occupancy = attention_kernel_symbol(w)
    kinds = probe.kinds()
    cost_cycles, cost_ns = {}, {}
    for cls in static:
        cyc, ghz = probe.issue_cost(kinds.index(PROBE_OF_CLASS[cls]), occupancy)[:2]
        cost_cycles[cls], cost_ns[cls] = cyc, cyc / ghz
    iterations = live_blocks * waves
    simds = 4 * n_cus
    model_ms = sum(static[c] * cost_ns[c] for c in static) * iterations / simds * 1e-6
    model_no_mfma_ms = sum(static[c] * cost_ns[c] for c in static if not c.startswith("mfma")) * iterations / simds * 1e-6
    return {
        "bound": "valu_issue",
        "kernel": name,
        "frac": model_ms / attn_ms,
        "frac_vector_only": model_no_mfma_ms / attn_ms,
        "model_ms": model_ms,
        "measured_ms": attn_ms,
        "instructions_per_iteration": static,
        "cost_cycles_per_wave_instruction": {k: round(v, 2) for k, v in cost_cycles.items()},
        "wavefronts_per_simd": occupancy,
        "iterations_per_launch": iterations,
        "note": "iteration = one live block visited by one wavefront; costs from lib/libparo_probe.so in this run; "
                "frac_vector_only leaves the matrix instructions out (they overlap with vector work only in part)",
    }


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed steps; the GPU clock takes some tens of milliseconds of load to settle")
    ap.add_argument("--workload", default="cogvideox5b")
    ap.add_argument("--density", type=float, default=None, help="override the workload's mask density (density sweep)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefetch", action="store_true", help="skip the mask-prefetch overhead measurement")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target wall time of the oracle sample")
    return ap.parse_args()


# ---------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands, on a bounded sample of the same workload
# ---------------------------------------------------------------------------------------------
_ORACLE_CTX = {}


def _oracle_rows(row_blocks):
    from oracle import paro_oracle as po

    c = _ORACLE_CTX
    po.sparse_attention_head(c["qc"], c["sq"], c["kc"], c["sk"], c["vc"], c["sv"], c["N"], c["block"], c["row_ptr"],
                             c["col_idx"], c["qmax_p"], row_blocks)
    return len(row_blocks)


def cpu_baseline(w, perm_ids, row_ptr, col_idx, target_seconds):
    """Times the float64 oracle, head after head (reorder + quantize of the head on one process,
    then its attention with the row blocks split over the host cores), until about
    ``target_seconds`` of wall time are spent.  Returns the JSON object; throughput is in the
    metric's unit (dense-equivalent TOPS) over the heads that were completed."""
    import multiprocessing as mp

    from oracle import paro_oracle as po
    from paper_2506_16054_amd import workloads as wl

    try:
        from threadpoolctl import threadpool_limits

        threadpool_limits(1)
    except Exception:
        pass
    # at most 16 worker processes: that is the CPU share of one GPU on the benchmark boxes, whatever the
    # affinity mask shows
    cores = max(1, min(len(os.sched_getaffinity(0)), 16, w.k))
    heads_done, live_done = 0, 0
    t_prep = t_attn = 0.0
    t_start = time.perf_counter()
    while heads_done < w.nh and (heads_done == 0 or time.perf_counter() - t_start < target_seconds):
        h = heads_done
        q, k, v = wl.make_head_qkv(w, 0, h)  # input generation is not timed
        t0 = time.perf_counter()
        idx = po.perm_index(w.F, w.Hg, w.Wg, w.T_text, int(perm_ids[h]))
        qc, sq = po.prepare_operand(q, idx, w.npad, w.block, w.bits_qk)
        kc, sk = po.prepare_operand(k, idx, w.npad, w.block, w.bits_qk)
        vc, sv = po.prepare_operand(v, idx, w.npad, w.block, w.bits_pv)
        t1 = time.perf_counter()
        _ORACLE_CTX.update(qc=qc, sq=sq, kc=kc, sk=sk, vc=vc, sv=sv, N=w.N, block=w.block, row_ptr=row_ptr[h],
                           col_idx=col_idx, qmax_p=None if w.bits_pv in (0, 16) else po.qmax_of(w.bits_pv))
        chunks = [list(range(c, w.k, cores)) for c in range(cores)]
        if cores > 1:
            with mp.get_context("fork").Pool(cores) as pool:  # forked after the context is set
                pool.map(_oracle_rows, chunks)
        else:
            _oracle_rows(chunks[0])
        t2 = time.perf_counter()
        t_prep += t1 - t0
        t_attn += t2 - t1
        live_done += int(row_ptr[h][w.k]) - int(row_ptr[h][0])
        heads_done += 1
    dense_ops = 4.0 * float(w.N) ** 2 * w.d * heads_done
    return {
        "value": dense_ops / (t_prep + t_attn) / 1e12,
        "unit": "dense-equivalent TOPS",
        "cores": cores,
        "kind": "oracle",
        "sample": "heads 0..%d of %d of %s (%d live blocks): attention %.1f s on %d processes (capped at 16, one GPU's CPU share "
                  "on the box), reorder+quantize %.1f s on 1; block list from the library's host routine (bit-identical to the oracle's)"
                  % (heads_done - 1, w.nh, w.name, live_done, t_attn, cores, t_prep),
    }


# ---------------------------------------------------------------------------------------------
# Mask prefetch (Sec. 4.2 (1), App. C): the path with a different mask at every step, loaded from
# pinned host memory and expanded on the GPU behind the previous step's attention, against the
# same sequence with every block list already resident.  Outside the headline's timed region.
# ---------------------------------------------------------------------------------------------
def prefetch_overhead(args, w, s, pa, perm_ids, q, k, v):
    import numpy as np
    import torch

    from paper_2506_16054_amd import binding as pb
    from paper_2506_16054_amd import workloads as wl
    from paper_2506_16054_amd.pipeline import MaskPrefetcher

    T = 4
    cache = {}
    rel = (1.0, 0.9, 1.1, 1.0)
    bitmasks = [wl.pack_bitmask(wl.make_block_masks(w.replace(density=min(1.0, w.density * r), seed=w.seed + 100 * t),
                                                    lambda pid: pb.paro_perm_index(s, pid), perm_ids, cache)) for t, r in enumerate(rel)]
    lists = [pb.paro_mask_to_blocklist(w.nh, w.k, bm) for bm in bitmasks]
    orders = [pb.paro_schedule_rows(s, w.bits_qk, w.bits_pv, rp) for rp, _ in lists]
    dev = q.device
    resident = [(torch.from_numpy(rp).to(dev), torch.from_numpy(ci).to(dev), torch.from_numpy(o).to(dev)) for (rp, ci), o in zip(lists, orders)]
    pf = MaskPrefetcher(s, np.stack(bitmasks), np.stack(orders), cap=max(ci.size for _, ci in lists), device=dev)
    pf_lists = MaskPrefetcher(s, np.stack(bitmasks), np.stack(orders), cap=max(ci.size for _, ci in lists), device=dev, lists_on_host=True)
    saved = (pa.row_ptr, pa.col_idx, pa.row_order)
    steps = max(T, args.steps // T * T)

    def run_resident():
        for i in range(steps):
            pa.prepare_fused_qkv(q, k, v)
            pa.use_blocklist(*resident[i % T])
            pa.attend_fused()

    def run_with(p):
        p.prefetch(0, 0)
        for i in range(steps):
            slot = i & 1
            if i + 1 < steps:
                p.prefetch(slot ^ 1, (i + 1) % T)
            pa.prepare_fused_qkv(q, k, v)
            pa.use_blocklist(*p.acquire(slot))
            pa.attend_fused()
            p.release(slot)

    def run_prefetched():
        run_with(pf)

    def run_lists():
        run_with(pf_lists)

    run_prefetched()  # untimed: first use of the copy stream, the pinned records and the expansion kernels
    run_lists()
    times = {}
    for name, fn in (("resident", run_resident), ("prefetched", run_prefetched), ("lists", run_lists), ("resident2", run_resident),
                     ("prefetched2", run_prefetched), ("lists2", run_lists), ("resident3", run_resident), ("prefetched3", run_prefetched),
                     ("lists3", run_lists)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        times[name] = (time.perf_counter() - t0) * 1e3 / steps
    # device time of one load + expansion, on the copy stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(pf.copy_stream):
        e0.record(pf.copy_stream)
    pf.prefetch(0, 1)
    with torch.cuda.stream(pf.copy_stream):
        e1.record(pf.copy_stream)
    torch.cuda.synchronize()
    pa.use_blocklist(*saved)
    # best of three alternating repetitions each: the host enqueues more per step on the prefetched
    # path, and a single repetition now and then catches a slow spell of the host
    res = min(times["resident"], times["resident2"], times["resident3"])
    pre = min(times["prefetched"], times["prefetched2"], times["prefetched3"])
    pre_lists = min(times["lists"], times["lists2"], times["lists3"])
    return {
        "masks": T,
        "steps": steps,
        "ms_per_step_resident_lists": res,
        "ms_per_step_prefetched": pre,
        "overhead_frac": pre / res - 1.0,
        "ms_per_step_prefetched_expanded_lists": pre_lists,
        "overhead_frac_expanded_lists": pre_lists / res - 1.0,
        "bytes_per_mask_expanded_lists": int(pf_lists.h_records.shape[1]),
        "note": "overhead_frac: 1-bit masks in pinned host memory, one transfer + one expansion kernel per step on a second stream "
                "(Sec. 4.2 (1)); overhead_frac_expanded_lists: the expanded column lists in pinned host memory, one transfer, no kernel",
        "repetitions_ms": {k: round(v, 4) for k, v in times.items()},
        "load_and_expand_us": e0.elapsed_time(e1) * 1e3,
        "bytes_per_mask": int(pf.h_records.shape[1]),
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards over heads with no exchange; "
              "no multi-GPU launch is part of it). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2506_16054_amd import binding as pb
    from paper_2506_16054_amd import workloads as wl
    from paper_2506_16054_amd.pipeline import ParoAttention

    w = wl.WORKLOADS[args.workload]
    if args.density is not None:
        w = w.replace(density=args.density)
    s = pb.shape_of(w)

    # ---- static per-head data (host): axis orders, block masks, block list
    perm_ids = wl.make_perm_ids(w)
    masks = wl.make_block_masks(w, lambda pid: pb.paro_perm_index(s, pid), perm_ids)
    bitmask = wl.pack_bitmask(masks)

    # ---- CPU baseline first: it forks worker processes, which must happen before this process
    # initialises the GPU runtime
    cpu = None
    if not args.no_cpu_baseline:
        h_row_ptr, h_col_idx = pb.paro_mask_to_blocklist(w.nh, w.k, bitmask)
        cpu = cpu_baseline(w, perm_ids, h_row_ptr, h_col_idx, args.cpu_seconds)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32

    # ---- synthetic inputs, generated on the host from the seed and moved to HBM once
    q = torch.empty((w.B, w.nh, w.N, w.d), dtype=tdt, device=dev)
    k = torch.empty_like(q)
    v = torch.empty_like(q)
    for b in range(w.B):
        for h in range(w.nh):
            hq, hk, hv = wl.make_head_qkv(w, b, h)
            q[b, h] = torch.from_numpy(hq).to(dev)
            k[b, h] = torch.from_numpy(hk).to(dev)
            v[b, h] = torch.from_numpy(hv).to(dev)
    pa = ParoAttention(s, perm_ids, bitmask, w.bits_qk, w.bits_pv, tdt, dev)
    live = pa.live_blocks
    live_ops = live * 4.0 * w.block * w.block * w.d
    dense_ops = 4.0 * w.B * w.nh * float(w.N) ** 2 * w.d

    for _ in range(args.warmup):
        pa.prepare_fused_qkv(q, k, v)
        pa.attend_fused()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; HIP events around each attention launch on the same stream
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        pa.prepare_fused_qkv(q, k, v)
        ev[i][0].record()
        pa.attend_fused()
        ev[i][1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- for reference, outside the timed region: the same path as separate steps
    pa.run(q, k, v)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for i in range(min(args.steps, 10)):
        pa.run(q, k, v)
    torch.cuda.synchronize()
    separate_ms = (time.perf_counter() - t2) * 1e3 / min(args.steps, 10)
    # and the form in which Q is reordered and quantized inside the attention kernel (K, V quantizers + attention)
    rawq_ms = None
    if pa.can_fuse_q:
        for _ in range(10):
            pa.run_rawq(q, k, v)
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for i in range(args.steps):
            pa.run_rawq(q, k, v)
        torch.cuda.synchronize()
        rawq_ms = (time.perf_counter() - t3) * 1e3 / args.steps
    attn_ms = sorted(a.elapsed_time(b) for a, b in ev)
    attn_avg = sum(attn_ms) / len(attn_ms)
    # the quantizer launch of step i lies between the end of attention i-1 and the start of attention i (gap included)
    quant_ms = sorted(ev[i - 1][1].elapsed_time(ev[i][0]) for i in range(1, len(ev)))
    quant_avg = sum(quant_ms) / len(quant_ms) if quant_ms else None

    prefetch = None if args.no_prefetch else prefetch_overhead(args, w, s, pa, perm_ids, q, k, v)

    quantized = w.bits_qk in (8, 4)
    # compulsory HBM bytes of one attention launch: Q, K, V operands read once, output written once
    qk_bytes = {4: 0.5, 8: 1, 16: 2}[w.bits_qk]
    v_bytes = 0.5 if w.bits_pv == 4 else (1 if w.bits_pv == 8 else 2)
    algorithmic_bytes = int(w.B * w.nh * w.npad * w.d * (2 * qk_bytes + v_bytes) + w.B * w.nh * w.N * w.d * (2 if w.dtype == "bf16" else 4))
    peak = PEAK_INT8_TOPS if quantized else PEAK_BF16_TFLOPS
    achieved = live_ops / (attn_avg * 1e-3) / 1e12
    from paper_2506_16054_amd import probe

    sustained = probe.sustained_mfma_rate(8 if quantized else 16)
    rec = recorded_counters(w, live) if quantized else {"valu_instructions": None, "traffic": None, "stale": None}
    n_cus = int(torch.cuda.get_device_properties(0).multi_processor_count)
    issue = valu_issue_roofline(w, live, attn_avg, n_cus) if quantized else None
    # second kernel of a step: the one-grid quantizer, bound by HBM (Q, K, V read once, their codes written once)
    in_bytes = 2 if w.dtype == "bf16" else 4
    quant_bytes = int(w.B * w.nh * (3 * w.N * w.d * in_bytes + w.npad * w.d * (2 * qk_bytes + v_bytes)))
    quant_roofline = None
    if quant_avg:
        copy_rate = probe.sustained_copy_rate(2 if in_bytes == 2 else 1)
        quant_roofline = {
            "kernel": "paro_permute_quantize_qkv", "bound": "hbm", "achieved": quant_bytes / (quant_avg * 1e-3) / 1e9, "peak": 8000.0,
            "unit": "GB/s", "frac": quant_bytes / (quant_avg * 1e-3) / 8e12, "ms_avg": quant_avg, "ms_min": quant_ms[0],
            "algorithmic_bytes": quant_bytes, "plain_copy_sustained": copy_rate * 1e3,
            "frac_of_plain_copy": quant_bytes / (quant_avg * 1e-3) / 1e12 / copy_rate,
            "note": "time from the end of one attention launch to the start of the next (HIP events), i.e. the quantizer launch and "
                    "its two launch gaps; plain_copy_sustained = a streaming copy with the same read:write mix, measured in this run",
        }
    out = {
        "metric": "dense_equivalent_TOPS",
        "value": dense_ops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TOPS (4*B*heads*N^2*d / step time; whole path: reorder + quantize + sparse attention + inverse reorder)",
        "separate_steps_ms": separate_ms,
        "q_quantized_in_attention_ms_per_step": rawq_ms,
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8" if quantized else "bf16",
        "data": "synthetic",
        "config": {
            "workload": "%s: B=%d heads=%d N=%d d=%d block=%d density=%.3f QK int%d PV int%d, %s in/out"
                        % (w.name, w.B, w.nh, w.N, w.d, w.block, live / (w.B * w.nh * w.k * w.k), w.bits_qk, w.bits_pv, w.dtype),
            "live_blocks": live,
            "seed": w.seed,
        },
        "attention_kernel": {
            "ms_avg": attn_avg,
            "ms_min": attn_ms[0],
            "ms_median": attn_ms[len(attn_ms) // 2],
            "dense_equivalent_TOPS": dense_ops / (attn_avg * 1e-3) / 1e12,
            "live_TOPS": achieved,
        },
        "roofline": {
            "kernel": "paro_sparse_attn_unpermuted",
            "bound": "mfma",
            "achieved": achieved,
            "peak": peak,
            "unit": "TOP/s" if quantized else "TFLOP/s",
            "frac": achieved / peak,
            "traffic": rec["traffic"],
            "traffic_unit": "bytes per launch (HBM read + write, rocprofv3 counters scaled by a known copy; null if profiles/ holds no record of the kernel this build launches)",
            "algorithmic_bytes": algorithmic_bytes,
            "peak_sustained": sustained,
            "frac_of_sustained": achieved / sustained,
            "peak_sustained_note": "rate of a kernel that only issues this matrix instruction, measured in this run",
        },
    }
    if issue is not None:
        issue["recorded_SQ_INSTS_VALU_per_launch"] = rec["valu_instructions"]
        issue["profiles_record_stale"] = rec["stale"]
        out["roofline_valu_issue"] = issue
    if quant_roofline is not None:
        out["roofline_quantizer"] = quant_roofline
    if prefetch is not None:
        out["mask_prefetch"] = prefetch
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
