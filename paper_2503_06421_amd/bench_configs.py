"""Measurements of the other workload configurations (bench.py at the repository root times the
Llama2-7B-shaped headline workload).

    python -m paper_2503_06421_amd.bench_configs --config single|13b|churn|70b|overlap|merging|apply|coldstart|pitch|probe

Each prints one JSON line.  Kernel times come from the library's HIP events around each launch
(TIDAL_FLAG_KERNEL_TIMING); call-level times from events on the compute stream.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np
import torch

from . import binding as tb
from . import harness as hz
from . import workloads as wl_mod

HBM_PEAK = 8000.0


def log(*a):
    print("[bench_configs]", *a, file=sys.stderr, flush=True)


def ev():
    return torch.cuda.Event(enable_timing=True)


def lora_bytes(wl, rank_old, rank_new):
    return 4 * wl.lora_w_elements + (hz.packed_adapter_bytes(wl, rank_old) if rank_old else 0) + \
        (hz.packed_adapter_bytes(wl, rank_new) if rank_new else 0)


def bench_single(args):
    """Configuration 1: one 4096 x 4096 fp32 layer, r = 8.  W (32 MiB) fits in the 256 MB Infinity
    Cache, so back-to-back timing of the same matrix measures the cache; a second set of numbers
    rotates over 24 distinct copies (768 MiB) so every pass comes from HBM."""
    wl = wl_mod.single_linear()
    copies = 24
    shapes = wl.shapes * copies
    pool = hz.HostPool(wl)
    ad = [hz.pinned_adapter(wl, a) for a in (0, 1)]
    T = hz.DeviceTemplate(shapes, max_adapter_bytes=hz.packed_adapter_bytes(wl), flags=tb.TIDAL_FLAG_KERNEL_TIMING)
    out = {"config": "single_linear_4096_fp32_r8"}
    try:
        src0 = pool.sources()[0]
        # materialise (PCIe): 64 MiB of fp32 -> one chunk
        times = []
        for rep in range(6):
            e0, e1 = ev(), ev()
            e0.record(T.compute_stream)
            tb.tidal_materialize(T.h, [(rep % copies, src0[1], src0[2])], T.copy_stream, T.compute_stream)
            e1.record(T.compute_stream)
            T.sync()
            times.append(e0.elapsed_time(e1))
        out["materialize_ms"] = round(float(np.median(times[1:])), 4)
        out["materialize_GBps"] = round(wl.source_bytes / np.median(times[1:]) / 1e6, 2)
        tb.tidal_materialize(T.h, [(i, src0[1], src0[2]) for i in range(copies)], T.copy_stream, T.compute_stream)
        T.sync()

        def targets(a, slot):
            s, al, A, B = ad[a][0][0]
            return tb.targets_from_arrays([(slot, al, A, B)])

        # (a) same matrix again and again, call-level (includes the upload), on a template without the
        # kernel-timing flag (its two event records per launch would count as part of the invocation).
        # "isolated": one event pair around each call; "back_to_back": 50 invocations between one
        # pair of events, the rate a keep-alive function under load sees.
        T2 = hz.DeviceTemplate(wl.shapes, max_adapter_bytes=hz.packed_adapter_bytes(wl))
        try:
            tb.tidal_materialize(T2.h, [(0, src0[1], src0[2])], T2.copy_stream, T2.compute_stream)
            T2.sync()
            call_ms = {"attach": [], "swap": [], "detach": []}
            for rep in range(12):
                e = [ev() for _ in range(4)]
                e[0].record(T2.compute_stream)
                tb.tidal_lora_attach(T2.h, targets(0, 0), T2.compute_stream)
                e[1].record(T2.compute_stream)
                tb.tidal_lora_swap(T2.h, targets(1, 0), T2.compute_stream)
                e[2].record(T2.compute_stream)
                tb.tidal_lora_detach(T2.h, T2.compute_stream)
                e[3].record(T2.compute_stream)
                T2.sync()
                if rep >= 2:
                    for k, name in enumerate(("attach", "swap", "detach")):
                        call_ms[name].append(e[k].elapsed_time(e[k + 1]))
            n_loop = 50
            pair_ms, swap_ms = [], []
            for rep in range(4):
                e0, e1 = ev(), ev()
                e0.record(T2.compute_stream)
                for _ in range(n_loop):
                    tb.tidal_lora_attach(T2.h, targets(0, 0), T2.compute_stream)
                    tb.tidal_lora_detach(T2.h, T2.compute_stream)
                e1.record(T2.compute_stream)
                T2.sync()
                pair_ms.append(e0.elapsed_time(e1) / n_loop)
                tb.tidal_lora_attach(T2.h, targets(0, 0), T2.compute_stream)
                e0, e1 = ev(), ev()
                e0.record(T2.compute_stream)
                for k in range(n_loop):
                    tb.tidal_lora_swap(T2.h, targets(1 - k % 2, 0), T2.compute_stream)
                e1.record(T2.compute_stream)
                T2.sync()
                swap_ms.append(e0.elapsed_time(e1) / n_loop)
                tb.tidal_lora_detach(T2.h, T2.compute_stream)
                T2.sync()
            out["cache_resident"] = {
                "isolated": {"attach_ms_per_invocation": round(float(np.median(call_ms["attach"])), 4),
                             "swap_ms_per_invocation": round(float(np.median(call_ms["swap"])), 4),
                             "detach_ms_per_invocation": round(float(np.median(call_ms["detach"])), 4)},
                "back_to_back": {"attach_plus_detach_ms": round(float(np.median(pair_ms[1:])), 4),
                                 "swap_ms_per_invocation": round(float(np.median(swap_ms[1:])), 4)},
                "note": "32 MiB W stays in the Infinity Cache between passes; adapters come from pinned host memory each call"}
        finally:
            T2.close()
        # (b) rotate over distinct copies with resident adapters: HBM-fed kernel time
        mems, handles = [], []
        for slot in range(copies):
            for a in (0, 1):
                tg = targets(a, slot)
                nb = tb.tidal_adapter_required_bytes(T.h, tg)
                mem = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
                handles.append(tb.tidal_adapter_upload(T.h, tg, mem, nb, T.compute_stream))
                mems.append(mem)
        T.sync()
        tb.tidal_reset_stats(T.h)
        for rep in range(3):
            for slot in range(copies):
                tb.tidal_lora_attach_adapter(T.h, handles[2 * slot], T.compute_stream)
                tb.tidal_lora_swap_adapter(T.h, handles[2 * slot + 1], T.compute_stream)
                tb.tidal_lora_detach(T.h, T.compute_stream)
        T.sync()
        st = tb.tidal_get_stats(T.h)
        kms = st["lora_kernel_ms"] / st["lora_launches"]
        out["hbm_fed"] = {"kernel_ms_avg": round(kms, 5), "kernel_GBps": round(lora_bytes(wl, 0, 8) / kms / 1e6, 1),
                          "frac_of_hbm_peak": round(lora_bytes(wl, 0, 8) / kms / 1e6 / HBM_PEAK, 4),
                          "note": "rotating over %d copies of W (%d MiB) so no pass is served from cache" % (copies, copies * 32)}
        for h in handles:
            tb.tidal_adapter_destroy(h)
    finally:
        T.close()
    return out


def bench_stack(args, wl, pool_limit=None):
    """materialise + attach for a whole stack (13B-shaped, 70B-shaped)."""
    pool = hz.HostPool(wl, limit_bytes=pool_limit)
    log("host pool ready in %.1f s (%s)" % (pool.draw_seconds, "wrapped" if pool.wrapped else "full"))
    items, keep = hz.pinned_adapter(wl, 0)
    flags = tb.TIDAL_FLAG_KERNEL_TIMING | (tb.TIDAL_FLAG_SERIAL_UPLOAD if args.serial_upload else 0)
    T = hz.DeviceTemplate(wl.shapes, max_adapter_bytes=hz.packed_adapter_bytes(wl), flags=flags)
    out = {"config": wl.name + ("_serial_upload" if args.serial_upload else ""), "source_GB": round(wl.source_bytes / 1e9, 3), "host_pool": "wrapped into %.1f GiB" % (pool_limit / 2**30) if pool.wrapped else "full"}
    try:
        probe = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        peak = tb.tidal_h2d_peak(probe, 1 << 30, 3, T.copy_stream)
        del probe
        srcs = pool.sources()
        mat, att, det = [], [], []
        tg = tb.targets_from_arrays(items)
        for rep in range(args.reps + 1):
            e = [ev() for _ in range(4)]
            tb.tidal_reset_stats(T.h)
            e[0].record(T.compute_stream)
            tb.tidal_materialize(T.h, srcs, T.copy_stream, T.compute_stream)
            e[1].record(T.compute_stream)
            tb.tidal_lora_attach(T.h, tg, T.compute_stream)
            e[2].record(T.compute_stream)
            T.sync()
            st = tb.tidal_get_stats(T.h)
            if rep > 0 or args.reps == 0:
                mat.append(e[0].elapsed_time(e[1]))
                att.append((e[1].elapsed_time(e[2]), st["lora_kernel_ms"], st["lora_launches"]))
            log("rep %d: materialize %.1f ms, attach %.2f ms (kernels %.3f ms in %d launches)" %
                (rep, e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2]), st["lora_kernel_ms"], st["lora_launches"]))
        mat_ms = float(np.median(mat))
        att_ms = float(np.median([a[0] for a in att]))
        k_ms = float(np.median([a[1] for a in att]))
        b = lora_bytes(wl, 0, wl.rank)
        out.update({
            "materialize_ms": round(mat_ms, 2), "materialize_GBps": round(wl.source_bytes / mat_ms / 1e6, 2),
            "h2d_peak_measured": round(peak, 2), "frac_of_measured_peak": round(wl.source_bytes / mat_ms / 1e6 / peak, 4),
            "attach_ms_per_invocation": round(att_ms, 3), "attach_kernel_ms": round(k_ms, 4),
            "attach_launches": att[-1][2], "lora_algorithmic_GB": round(b / 1e9, 3),
            "lora_kernel_GBps": round(b / k_ms / 1e6, 1), "frac_of_hbm_peak": round(b / k_ms / 1e6 / HBM_PEAK, 4)})
    finally:
        T.close()
    return out


def bench_pitch(args):
    """One merge launch per shape, warm (back-to-back attach / detach of a resident adapter): the
    4096-wide power-of-two row pitch next to the three shapes of the 13B-shaped stack, each with the
    bare read-modify-write probe in the same tiling and walk length beside it.  The run the
    memory-side counters are collected on (one dispatch per shape and direction)."""
    shapes = [(4096, 4096, 64), (5120, 5120, 80), (13824, 5120, 80), (5120, 13824, 40)]
    r = args.rank
    out = {"config": "merge_by_row_pitch_r%d" % r, "shapes": []}
    for rows, cols, n in shapes:
        T = hz.DeviceTemplate([(rows, cols)] * n, flags=tb.TIDAL_FLAG_KERNEL_TIMING)
        try:
            rng = np.random.default_rng(rows + cols)
            w = torch.from_numpy(rng.normal(0, 0.02, (rows, cols)).astype(np.float16)).pin_memory()
            tb.tidal_materialize(T.h, [(i, tb.TIDAL_F16, w.data_ptr()) for i in range(n)], T.copy_stream, T.compute_stream)
            T.sync()
            A = rng.normal(0, 0.01, (r, cols)).astype(np.float16)
            B = rng.normal(0, 0.01, (rows, r)).astype(np.float16)
            tg = [(i, r, 2.0 * r, tb.TIDAL_F16, A.ctypes.data, B.ctypes.data) for i in range(n)]   # one device copy per slot
            nb = tb.tidal_adapter_required_bytes(T.h, tg)
            mem = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
            a = tb.tidal_adapter_upload(T.h, tg, mem, nb, T.compute_stream)
            T.sync()
            info = tb.tidal_lora_launch_info(T.h, rows, cols, n, 0, r)
            ms = []
            for rep in range(args.reps + 1):
                tb.tidal_reset_stats(T.h)
                tb.tidal_lora_attach_adapter(T.h, a, T.compute_stream)
                tb.tidal_lora_detach(T.h, T.compute_stream)
                T.sync()
                if rep:
                    ms.append(tb.tidal_get_stats(T.h)["lora_kernel_ms"] / 2)
            rp = 16 if r <= 16 else (32 if r <= 32 else 64)
            byt = 4.0 * n * rows * cols + n * 2 * rp * (rows + cols)
            k_ms = float(np.median(ms))
            p0, _ = tb.tidal_template_slot_ptr(T.h, 0)
            bare = tb.tidal_hbm_rmw_peak(p0, rows, cols, n, info["blocks_per_walk"], 4, T.compute_stream)
            bare1 = tb.tidal_hbm_rmw_peak(p0, rows, cols, n, 1, 4, T.compute_stream)
            rec = {"shape": "%d x %d x %d" % (n, rows, cols), "row_pitch_bytes": 2 * cols, "kernel": info["kernel"],
                   "blocks_per_walk": info["blocks_per_walk"], "kernel_ms": round(k_ms, 4),
                   "GBps": round(byt / k_ms / 1e6, 1), "frac_of_hbm_peak": round(byt / k_ms / 1e6 / HBM_PEAK, 4),
                   "bare_rmw_same_walk_GBps": round(bare, 1), "frac_of_bare_rmw": round(byt / k_ms / 1e6 / bare, 4),
                   "bare_rmw_one_block_per_wave_GBps": round(bare1, 1)}
            out["shapes"].append(rec)
            log(json.dumps(rec))
            tb.tidal_adapter_destroy(a)
        finally:
            T.close()
        del T
        torch.cuda.empty_cache()
    return out


def bench_probe(args):
    """What this memory system makes of a row pitch and a walk length, with the LoRA kernels' tiling and no arithmetic:
    about 4 GiB of matrices per width, each 256-column strip walked down in runs of 1, 4 or 16 blocks of 32 rows, as
    loads only, stores only and read-modify-write (tidal_hbm_probe)."""
    widths = [4096, 5120, 8192, 11008, 13824, 28672]
    out = {"config": "hbm_probe_by_row_pitch", "widths": []}
    for cols in widths:
        rows = 4096
        n = max(1, (4 << 30) // (rows * cols * 2))
        mem = torch.zeros(n * rows * cols, dtype=torch.int16, device="cuda:0")
        rec = {"cols": cols, "row_pitch_bytes": 2 * cols, "matrices": n, "GiB": round(n * rows * cols * 2 / 2 ** 30, 2)}
        for mode, name in ((tb.TIDAL_PROBE_READ, "read"), (tb.TIDAL_PROBE_WRITE, "write"), (tb.TIDAL_PROBE_RMW, "rmw")):
            for walk in (1, 4, 16):
                rec["%s_walk%d_GBps" % (name, walk)] = round(tb.tidal_hbm_probe(mem, rows, cols, n, walk, mode, 4), 1)
        out["widths"].append(rec)
        log(json.dumps(rec))
        del mem
        torch.cuda.empty_cache()
    return out


def bench_coldstart(args):
    """Cold start of the Llama2-7B-shaped function with its adapter known at load time: the load
    followed by an attach, against tidal_materialize_attach, which folds the adapter into the
    conversion (one rounding from the fp16 source, no read-modify-write pass)."""
    wl = wl_mod.llama2_7b()
    pool = hz.HostPool(wl)
    items, keep = hz.pinned_adapter(wl, 0)
    T = hz.DeviceTemplate(wl.shapes, max_adapter_bytes=hz.packed_adapter_bytes(wl), flags=tb.TIDAL_FLAG_KERNEL_TIMING)
    out = {"config": wl.name + "_coldstart", "source_GB": round(wl.source_bytes / 1e9, 3)}
    try:
        srcs = pool.sources()
        tg = tb.targets_from_arrays(items)
        res = {"two_calls": [], "fused": []}
        for rep in range(args.reps + 1):
            for mode in ("two_calls", "fused"):
                tb.tidal_reset_stats(T.h)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                if mode == "fused":
                    tb.tidal_materialize_attach(T.h, srcs, tg, T.copy_stream, T.compute_stream)
                else:
                    tb.tidal_materialize(T.h, srcs, T.copy_stream, T.compute_stream)
                    tb.tidal_lora_attach(T.h, tg, T.compute_stream)
                T.sync()
                ms = (time.perf_counter() - t0) * 1e3
                st = tb.tidal_get_stats(T.h)
                log("rep %d %s: %.2f ms (convert kernels %.2f ms, LoRA kernels %.3f ms, %d LoRA launches)" %
                    (rep, mode, ms, st["convert_kernel_ms"], st["lora_kernel_ms"], st["lora_launches"]))
                if rep > 0:
                    res[mode].append((ms, st["convert_kernel_ms"], st["lora_kernel_ms"]))
        for mode, r in res.items():
            out[mode] = {"ms": round(float(np.median([x[0] for x in r])), 2),
                         "GBps": round(wl.source_bytes / float(np.median([x[0] for x in r])) / 1e6, 2),
                         "convert_kernel_ms": round(float(np.median([x[1] for x in r])), 2),
                         "lora_kernel_ms": round(float(np.median([x[2] for x in r])), 3)}
    finally:
        T.close()
    return out


def bench_churn(args):
    """Configuration 4: resident 7B-shaped bf16 base, pool of 32 resident adapters (ranks from
    {8,16,32,64}, alpha = 2r, targets q,k,v,o), 200 invocations by Zipf(1.1): step 0 attaches,
    every later step is one fused swap."""
    ch = wl_mod.adapter_churn()
    wl = ch.base
    # the base's values do not matter for timing: stream it from a wrapped pool
    pool = hz.HostPool(wl, limit_bytes=2 << 30)
    T = hz.DeviceTemplate(wl.shapes, flags=tb.TIDAL_FLAG_KERNEL_TIMING)
    out = {"config": "adapter_churn_llama2_7b_shaped", "pool": len(ch.ranks), "steps": len(ch.schedule)}
    try:
        tb.tidal_materialize(T.h, pool.sources(), T.copy_stream, T.compute_stream)
        T.sync()
        handles, mems = [], []
        t0 = time.perf_counter()
        for a, r in enumerate(ch.ranks):
            items, keep = hz.pinned_adapter(wl, a, rank=r, alpha=ch.alphas[a])
            tg = tb.targets_from_arrays(items)
            nb = tb.tidal_adapter_required_bytes(T.h, tg)
            mem = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
            handles.append(tb.tidal_adapter_upload(T.h, tg, mem, nb, T.compute_stream))
            mems.append(mem)
            T.sync()
        log("uploaded %d adapters (%.2f GB packed) in %.1f s" % (len(handles), sum(m.numel() for m in mems) / 1e9, time.perf_counter() - t0))
        per_step = []
        cur = None
        for step, a in enumerate(ch.schedule):
            tb.tidal_reset_stats(T.h)
            e0, e1 = ev(), ev()
            e0.record(T.compute_stream)
            if step == 0:
                tb.tidal_lora_attach_adapter(T.h, handles[a], T.compute_stream)
            else:
                tb.tidal_lora_swap_adapter(T.h, handles[a], T.compute_stream)
            e1.record(T.compute_stream)
            T.sync()
            st = tb.tidal_get_stats(T.h)
            r_old = ch.ranks[cur] if cur is not None else 0
            per_step.append((r_old, ch.ranks[a], e0.elapsed_time(e1), st["lora_kernel_ms"], a == cur))
            cur = a
        swaps = per_step[1:]
        call = np.array([s[2] for s in swaps])
        kern = np.array([s[3] for s in swaps])
        by = {}
        for r0, r1, c, k, same in swaps:
            by.setdefault((r0, r1), []).append(k)
        byte_of = lambda r0, r1: lora_bytes(wl, r0, r1)
        total_bytes = sum(byte_of(r0, r1) for r0, r1, *_ in swaps)
        out.update({
            "swap_ms_per_invocation": {"mean": round(float(call.mean()), 4), "p50": round(float(np.median(call)), 4),
                                       "p95": round(float(np.percentile(call, 95)), 4)},
            "swap_kernel_ms": {"mean": round(float(kern.mean()), 4), "p50": round(float(np.median(kern)), 4),
                               "p95": round(float(np.percentile(kern, 95)), 4)},
            "swap_GBps_overall": round(total_bytes / kern.sum() / 1e6, 1),
            "frac_of_hbm_peak": round(total_bytes / kern.sum() / 1e6 / HBM_PEAK, 4),
            "first_attach_ms": round(per_step[0][2], 4),
            "repeats_of_attached_adapter": int(sum(1 for s in swaps if s[4])),
            "by_rank_pair_GBps": {"%d->%d" % k: round(byte_of(*k) / float(np.median(v)) / 1e6, 0) for k, v in sorted(by.items())},
            "by_rank_pair_count": {"%d->%d" % k: len(v) for k, v in sorted(by.items())}})
        tb.tidal_lora_detach(T.h, T.compute_stream)
        T.sync()
        # the same schedule through a copy-on-write fork: every step rewrites the private copies of
        # the 128 targeted slots from the pristine template (no unmerge, no accumulated rounding)
        need = tb.tidal_fork_required_bytes(T.h, wl.lora_slots)
        fmem = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        F = tb.tidal_fork_create(T.h, wl.lora_slots, fmem, need)
        fk, fbytes = [], 0
        for step, a in enumerate(ch.schedule):
            tb.tidal_reset_stats(T.h)
            tb.tidal_fork_apply(F, handles[a], T.compute_stream)
            T.sync()
            st = tb.tidal_get_stats(T.h)
            if step:
                fk.append(st["lora_kernel_ms"])
                fbytes += lora_bytes(wl, 0, ch.ranks[a])
        fk = np.array(fk)
        out["fork_apply_kernel_ms"] = {"mean": round(float(fk.mean()), 4), "p50": round(float(np.median(fk)), 4),
                                       "p95": round(float(np.percentile(fk, 95)), 4)}
        out["fork_apply_GBps_overall"] = round(fbytes / fk.sum() / 1e6, 1)
        out["fork_extra_GB"] = round(need / 1e9, 3)
        tb.tidal_fork_destroy(F)
        for h in handles:
            tb.tidal_adapter_destroy(h)
    finally:
        T.close()
    return out


def bench_overlap(args):
    """Sec. 5.2 of the paper on this hardware: time-to-finish of a consumer that reads every slot in
    access order (stand-in for the first inference; its duration is set by the number of passes over
    each slot) while the template streams in, (C) from nothing in access order, (D) from nothing in
    reverse order, (E) with the leading M_prefetch bytes of Eq. 1 already resident.  Expectation:
    C ~ max(load, compute) + first slot, D ~ load + compute, E ~ compute."""
    wl = wl_mod.llama2_7b()
    pool = hz.HostPool(wl, limit_bytes=2 << 30)
    T = hz.DeviceTemplate(wl.shapes, flags=tb.TIDAL_FLAG_SLOT_EVENTS)
    consumer = torch.cuda.Stream()
    n = len(wl.shapes)
    sums = torch.zeros(n, dtype=torch.int64, device="cuda:0")
    srcs = pool.sources()
    out = {"config": "overlap_llama2_7b_shaped", "model_GB": round(wl.source_bytes / 1e9, 3), "cases": []}

    def load(which):
        tb.tidal_materialize(T.h, which, T.copy_stream, T.compute_stream)

    def consume(passes):
        for i in range(n):
            tb.tidal_slot_checksum(T.h, i, passes, consumer, sums[i:])

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        T.sync()
        consumer.synchronize()
        return (time.perf_counter() - t0) * 1e3

    try:
        load(srcs); T.sync()                                           # warm-up, everything resident
        t_load = min(timed(lambda: load(srcs)) for _ in range(2))
        t_c1 = min(timed(lambda: consume(1)) for _ in range(2))
        t_c9 = min(timed(lambda: consume(9)) for _ in range(2))
        per_pass = max((t_c9 - t_c1) / 8.0, 1e-3)
        link = wl.source_bytes / (t_load * 1e-3)
        out["load_ms"] = round(t_load, 2)
        out["link_GBps"] = round(link / 1e9, 2)
        out["consume_ms_first_pass"] = round(t_c1, 3)
        out["consume_ms_per_extra_pass"] = round(per_pass, 3)
        for ratio in (0.5, 1.0, 2.0):
            passes = max(1, 1 + int(round((ratio * t_load - t_c1) / per_pass)))
            t_c = min(timed(lambda: consume(passes)) for _ in range(2))
            t_cold = timed(lambda: (load(srcs), consume(passes)))
            t_rev = timed(lambda: (load(srcs[::-1]), consume(passes)))
            pre = tb.tidal_prefetch_bytes(wl.source_bytes, t_c * 1e-3, link)
            n_res, res_bytes = tb.tidal_template_resident_prefix(T.h, pre)
            # the resident part is the template; only the rest is loaded at invocation time
            t_pre = timed(lambda: ((load(srcs[n_res:]) if n_res < n else None), consume(passes)))
            out["cases"].append({
                "compute_over_load": ratio, "passes": passes, "compute_ms": round(t_c, 2),
                "cold_access_order_ms": round(t_cold, 2), "cold_reverse_order_ms": round(t_rev, 2),
                "reverse_over_access": round(t_rev / t_cold, 3),
                "eq1_prefetch_GB": round(pre / 1e9, 3), "resident_slots": n_res, "resident_GB": round(res_bytes / 1e9, 3),
                "with_prefetch_ms": round(t_pre, 2),
                "max_load_compute_ms": round(max(t_load, t_c), 2), "load_plus_compute_ms": round(t_load + t_c, 2)})
            log(json.dumps(out["cases"][-1]))
    finally:
        T.close()
    return out


def bench_merging(args):
    """Tensor-merging study (Sec. 6 / Sec. 7.4 of the paper): 1,202 tensors of a 70B-shaped TP-8
    shard, streamed with and without merging neighbouring copies, for several chunk sizes."""
    wl = wl_mod.llama70b_tp8_shard_many_tensors()
    pool = hz.HostPool(wl, limit_bytes=4 << 30)
    srcs = pool.sources()
    out = {"config": wl.name, "tensors": len(wl.tensors), "source_GB": round(wl.source_bytes / 1e9, 3), "runs": []}
    for merge in (True, False):
        for mib in (16, 64, 256):
            flags = 0 if merge else tb.TIDAL_FLAG_NO_COPY_MERGE
            T = hz.DeviceTemplate(wl.shapes, chunk_bytes=mib << 20, flags=flags)
            try:
                ms = []
                for rep in range(3):
                    tb.tidal_reset_stats(T.h)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    tb.tidal_materialize(T.h, srcs, T.copy_stream, T.compute_stream)
                    T.sync()
                    ms.append((time.perf_counter() - t0) * 1e3)
                st = tb.tidal_get_stats(T.h)
                run = {"merge": merge, "chunk_mib": mib, "ms": round(min(ms[1:]), 2),
                       "GBps": round(wl.source_bytes / min(ms[1:]) / 1e6, 2), "h2d_copies": st["h2d_copies"],
                       "chunks": st["chunks"], "gathered_MB": round(st["gathered_bytes"] / 1e6, 3)}
                out["runs"].append(run)
                log(json.dumps(run))
            finally:
                T.close()
    return out


def bench_apply(args):
    """Unmerged adapters on mixed batches (the paper's dynamic function keeps adapters as separate
    weights, Sec. 3 / Sec. 5.2): y += (alpha/r) B bf16(A x) on the 4096 x 4096 query projection of
    32 layers, one call per layer, so that a pass touches 32 distinct sets of factors and
    activations (more than the 256 MB Infinity Cache holds for the larger batches).  A pool of 32
    adapters with ranks {8, 16, 32, 64} and Zipf(1.1) popularity, as in the churn configuration."""
    layers, hidden = args.layers, 4096
    ch = wl_mod.adapter_churn()
    rng = np.random.default_rng(0)
    shapes = [(hidden, hidden)] * layers
    T = hz.DeviceTemplate(shapes, max_adapter_bytes=0)
    out = {"config": "apply_q_proj_4096_x%d_layers_pool32" % layers, "cases": []}
    keep, handles = [], []
    try:
        host = {}
        for r in sorted(set(ch.ranks)):
            A = torch.empty((r, hidden), dtype=torch.float32, pin_memory=True)
            B = torch.empty((hidden, r), dtype=torch.float32, pin_memory=True)
            A.numpy()[...] = rng.normal(0, 0.02, (r, hidden))
            B.numpy()[...] = rng.normal(0, 0.02, (hidden, r))
            host[r] = (A, B)
        for a, r in enumerate(ch.ranks):
            A, B = host[r]
            tg = [(s, r, ch.alphas[a], tb.TIDAL_F32, A.data_ptr(), B.data_ptr()) for s in range(layers)]
            nb = tb.tidal_adapter_required_bytes(T.h, tg)
            mem = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
            handles.append(tb.tidal_adapter_upload(T.h, tg, mem, nb, T.compute_stream))
            keep.append(mem)
        T.sync()
        sched = ch.schedule

        def requests(lengths):
            segs, t = [], 0
            for i, n in enumerate(lengths):
                segs.append((sched[i % len(sched)], t, t + n))
                t += n
            return segs, t

        cases = [("decode_64_requests_x1_token", [1] * 64), ("decode_256_requests_x1_token", [1] * 256),
                 ("prefill_8_requests_x512_tokens", [512] * 8), ("mixed_4x512_prefill_plus_60_decode", [512] * 4 + [1] * 60),
                 ("prompt_16384_tokens_one_adapter", [16384])]
        for name, lengths in cases:
            if args.case and args.case not in name:
                continue
            segs, n = requests(lengths)
            X = [torch.randn((n, hidden), device="cuda:0").to(torch.bfloat16) for _ in range(layers)]
            Y = [torch.randn((n, hidden), device="cuda:0").to(torch.bfloat16) for _ in range(layers)]
            nb = tb.tidal_lora_apply_workspace_bytes(n)
            ws = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
            used = sorted({a for a, _, _ in segs})
            factor_bytes = sum(2 * (ch.ranks[a] * hidden + hidden * max(16, 1 << (ch.ranks[a] - 1).bit_length())) for a in used)
            alg = n * hidden * 2 + n * hidden * 4 + factor_bytes       # x once, y read + written, factors once
            best = None
            aarr, sarr = tb.lora_apply_arrays(handles, segs)          # marshalled once, as a server would
            xp = [t_.data_ptr() for t_ in X]
            yp = [t_.data_ptr() for t_ in Y]
            wp, sp = ws.data_ptr(), T.compute_stream.cuda_stream
            host_us = None
            for rep in range(args.reps + 1):
                e0, e1 = ev(), ev()
                e0.record(T.compute_stream)
                h0 = time.perf_counter()
                for l in range(layers):
                    tb.tidal_lora_apply(T.h, l, aarr, sarr, xp[l], yp[l], n, wp, nb, sp)
                h1 = time.perf_counter()
                e1.record(T.compute_stream)
                T.sync()
                ms = e0.elapsed_time(e1) / layers
                if rep > 0:
                    best = ms if best is None else min(best, ms)
                    hu = (h1 - h0) * 1e6 / layers                 # the host's share: marshalling, planning, launches
                    host_us = hu if host_us is None else min(host_us, hu)
            # the layer loop captured once in a HIP graph (the allocation-free entry point: kernel launches only) and
            # replayed: the GPU's time per call with the host's share taken out
            graph_us = None
            if n <= tb.tidal_lora_apply_static_max_tokens():
                for l in range(layers):                                  # eager once: the adapters' uploads are seen done
                    tb.tidal_lora_apply_static(T.h, l, aarr, sarr, xp[l], yp[l], n, sp)
                T.sync()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=T.compute_stream):
                    cs = torch.cuda.current_stream().cuda_stream
                    for l in range(layers):
                        tb.tidal_lora_apply_static(T.h, l, aarr, sarr, xp[l], yp[l], n, cs)
                torch.cuda.synchronize()
                with torch.cuda.stream(T.compute_stream):
                    for rep in range(args.reps + 1):
                        e0, e1 = ev(), ev()
                        e0.record()
                        g.replay()
                        e1.record()
                        torch.cuda.synchronize()
                        if rep > 0:
                            us = e0.elapsed_time(e1) * 1e3 / layers
                            graph_us = us if graph_us is None else min(graph_us, us)
                del g
            # the q, k and v targets of a layer in one call: slots l, l+1, l+2 (mod layers) stand in for them
            best3 = None
            if n <= 4096:
                nb3 = tb.tidal_lora_apply_workspace_bytes(3 * n)
                ws3 = torch.empty(nb3, dtype=torch.uint8, device="cuda:0")
                for rep in range(args.reps + 1):
                    e0, e1 = ev(), ev()
                    e0.record(T.compute_stream)
                    for l in range(layers):
                        sl = [l, (l + 1) % layers, (l + 2) % layers]
                        tb.tidal_lora_apply_multi(T.h, sl, aarr, sarr, xp[l], [yp[i] for i in sl], n, ws3.data_ptr(), nb3, sp)
                    e1.record(T.compute_stream)
                    T.sync()
                    ms = e0.elapsed_time(e1) / layers
                    if rep > 0:
                        best3 = ms if best3 is None else min(best3, ms)
            case = {"case": name, "tokens": n, "requests": len(lengths), "adapters_used": len(used),
                    "us_per_layer_call": round(best * 1e3, 2), "host_us_per_call": round(host_us, 2),
                    "us_per_call_graph_replay": round(graph_us, 2) if graph_us else None, "algorithmic_MB": round(alg / 1e6, 3),
                    "GBps": round(alg / best / 1e6, 1), "hbm_frac": round(alg / best / 1e6 / HBM_PEAK, 4),
                    "us_per_call_3_targets": round(best3 * 1e3, 2) if best3 else None}
            out["cases"].append(case)
            log(json.dumps(case))
            del X, Y, ws
    finally:
        for h in handles:
            tb.tidal_adapter_destroy(h)
        T.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", required=True, choices=["single", "13b", "churn", "70b", "overlap", "merging", "apply", "coldstart", "pitch", "probe"])
    ap.add_argument("--rank", type=int, default=64, help="pitch: rank of the merged adapter")
    ap.add_argument("--reps", type=int, default=2)
    ap.add_argument("--pool-gib", type=float, default=0.0, help="wrap the host pool into this many GiB (70b default: 24)")
    ap.add_argument("--serial-upload", action="store_true", help="13b / 70b: TIDAL_FLAG_SERIAL_UPLOAD")
    ap.add_argument("--layers", type=int, default=32, help="apply: distinct layers (sets of factors and activations) per pass")
    ap.add_argument("--case", default="", help="apply: only cases whose name contains this")
    args = ap.parse_args()
    assert torch.cuda.is_available(), "needs a GPU (there is no CPU path)"
    torch.cuda.set_device(0)
    if args.config == "single":
        out = bench_single(args)
    elif args.config == "13b":
        out = bench_stack(args, wl_mod.llama2_13b(), int(args.pool_gib * 2**30) if args.pool_gib else None)
    elif args.config == "70b":
        out = bench_stack(args, wl_mod.llama3_70b(), int((args.pool_gib or 24.0) * 2**30))
    elif args.config == "probe":
        out = bench_probe(args)
    elif args.config == "overlap":
        out = bench_overlap(args)
    elif args.config == "merging":
        out = bench_merging(args)
    elif args.config == "apply":
        out = bench_apply(args)
    elif args.config == "coldstart":
        out = bench_coldstart(args)
    elif args.config == "pitch":
        out = bench_pitch(args)
    else:
        out = bench_churn(args)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
