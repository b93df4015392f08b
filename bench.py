#!/usr/bin/env python3
"""Benchmark of the template-materialisation + LoRA attach/swap hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

The headline workload is the largest one that fits one GPU: the Llama-3-70B-shaped stack (562 bf16
tensors, 141.1 GB, streamed from a pinned host pool the tensors are mapped into modulo its size)
with LoRA r = 16 on all seven projections of its 80 layers (560 targets).  One *step* is one pass
of the whole path over it:
  tidal_materialize   host tensors -> bf16 template slots (chunked pinned H2D on a copy stream,
                      conversion kernel on a second stream where the host dtype is not bf16),
  tidal_lora_attach   adapter upload + in-place merge W += (alpha/r) B A on every targeted slot.
The other four workloads (single 4096^2 layer; 7B-shaped stack with attach + swap; 13B-shaped stack
with r = 64 on 280 targets; adapter churn, 200 swaps of resident adapters) run after it with a few
repetitions each and are reported in the same shape under "configs".

The line printed at the end is JSON.  `value` is the LoRA merge throughput of the headline
workload with W and the packed adapters resident in HBM: algorithmic bytes (4 B per targeted W
element, plus the packed A/B read once) divided by the duration of the read-modify-write kernels,
which the library brackets with HIP events on the launch stream.  The PCIe-inclusive
materialisation rate is reported next to it under "materialize" (never as `value`), with the
host->device link peak measured in the same run.  "cpu_baseline" times the CPU oracle, as it
stands, on a bounded sample of the same work (conversion and LoRA passes on bands of rows of
sampled slots); the same bands are compared with what the GPU produced, and a mismatch beyond the
stated bound makes the run fail.
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
TOL = 2.0 ** -7                 # max |W_gpu - W_oracle| / max |W_oracle| per compared band
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")   # written by paper_2503_06421_amd.pmc_traffic


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def padded_rank(r):
    return 0 if r <= 0 else (16 if r <= 16 else (32 if r <= 32 else 64))


def factor_bytes(wl, slots, r):
    """What a LoRA kernel reads of one adapter: bf16 A^T (in x rp) and B (out x rp) per target."""
    rp = padded_rank(r)
    return sum(2 * rp * (wl.tensors[s].rows + wl.tensors[s].cols) for s in slots)


def measured_traffic(key):
    """HBM bytes per launch of the dominant kernel from the last counter run on this workload
    (profiles/hbm_traffic.json), or None if there is none."""
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f).get(key, {}).get("hbm_bytes_per_launch")
    except (OSError, ValueError):
        return None


def f64(bits, np):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


class OracleSample:
    """Times the oracle on bands of rows and compares them with the GPU's result.  Everything that
    touches oracle/ lives here (bench.py's cpu_baseline leg)."""

    def __init__(self, budget_s):
        from oracle import tidal_oracle as orc
        self.orc = orc
        self.budget = budget_s
        self.convert_bytes = self.convert_s = 0.0
        self.lora_bytes = self.lora_s = 0.0
        self.bands = 0
        self.worst = 0.0
        self.mismatch = 0.0
        self.exact_convert = True

    def spent(self):
        return self.convert_s + self.lora_s

    def convert(self, src):
        """bf16 bits of a host array, timed (the materialisation's arithmetic)."""
        c0 = time.perf_counter()
        out = self.orc.convert_to_bf16(src)
        self.convert_s += time.perf_counter() - c0
        self.convert_bytes += src.size * src.itemsize
        return out

    def passes(self, W, steps):
        """steps: list of (sign, alpha, A_bits, B_bits_band).  In place on W (bf16 bits), timed."""
        for sign, alpha, A, B in steps:
            c0 = time.perf_counter()
            self.orc.lora_merge(W, A, B, alpha, sign)
            self.lora_s += time.perf_counter() - c0
            r = A.shape[0]
            self.lora_bytes += 4.0 * W.size + 2.0 * padded_rank(r) * (A.shape[1] + B.shape[0])

    def compare(self, got, want, np, exact=False):
        self.bands += 1
        if exact:
            self.exact_convert = self.exact_convert and bool(np.array_equal(got, want))
            return
        g, w = f64(got, np), f64(want, np)
        self.worst = max(self.worst, float(np.max(np.abs(g - w)) / np.max(np.abs(w))))
        self.mismatch = max(self.mismatch, float(np.mean(got != want)))

    def records(self, what, cores_total):
        conv = self.convert_bytes / self.convert_s / 1e9 if self.convert_s > 0 else None
        lora = self.lora_bytes / self.lora_s / 1e9 if self.lora_s > 0 else None
        cpu = {"value": round(lora, 4) if lora else None, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "%s: %d bands, %.1f s of LoRA passes (4 B per W element + factors) and %.1f s of conversion; "
                         "rates are those of the sample, extrapolated to the whole workload they give its CPU time; "
                         "host has %d logical cores, the oracle uses one" % (what, self.bands, self.lora_s, self.convert_s, cores_total),
               "materialize_value": round(conv, 4) if conv else None, "materialize_unit": "GB/s of source bytes converted to bf16"}
        parity = {"bands_checked": self.bands, "max_abs_err_over_max_abs_w": self.worst, "bound": TOL,
                  "worst_fraction_of_elements_differing": self.mismatch, "conversion_bit_exact": self.exact_convert,
                  "ok": bool(self.worst <= TOL and self.exact_convert)}
        return cpu, parity


def band_of(rows, k, band_rows):
    """k-th band of a slot: top, a ragged place in the middle, bottom."""
    band_rows = min(band_rows, rows)
    starts = [0, max(0, (rows // 2 // 64) * 64 - 29), rows - band_rows]
    r0 = min(starts[k % 3], rows - band_rows)
    return r0, r0 + band_rows


def run_stack(tag, wl, args, pcie_peak, pool_limit, steps, warmup, with_swap, cpu_seconds, traffic_key):
    """materialize + attach (+ swap) on a whole stack.  Returns the record of this configuration."""
    import numpy as np
    import torch
    from paper_2503_06421_amd import binding as tb
    from paper_2503_06421_amd import harness as hz

    pool = hz.HostPool(wl, limit_bytes=pool_limit)
    log("%s: host pool of %.1f GB ready in %.1f s (%s)" % (tag, pool.buf.numel() / 1e9, pool.draw_seconds,
                                                          "tensors mapped into it modulo its size" if pool.wrapped else "every tensor drawn"))
    ads = [hz.pinned_adapter(wl, a) for a in ((0, 1) if with_swap else (0,))]
    targets = [tb.targets_from_arrays(items) for items, _ in ads]
    # Two templates over one arena: the plain one gives the call-level times (ms per invocation, materialise
    # rate, wall time per step); the one with TIDAL_FLAG_KERNEL_TIMING gives the kernel durations -- its two
    # event records around every launch would otherwise count as part of an invocation.
    T = hz.DeviceTemplate(wl.shapes, chunk_bytes=args.chunk_mib << 20, max_adapter_bytes=hz.packed_adapter_bytes(wl),
                          flags=tb.TIDAL_FLAG_KERNEL_TIMING)
    Tp = hz.DeviceTemplate(wl.shapes, arena=T.arena, chunk_bytes=args.chunk_mib << 20, max_adapter_bytes=hz.packed_adapter_bytes(wl))
    srcs = pool.sources()
    ev = lambda: torch.cuda.Event(enable_timing=True)
    rec = {"config": tag}
    try:
        def step(tpl, e=None):
            comp = tpl.compute_stream
            if e:
                e[0].record(comp)
            tb.tidal_materialize(tpl.h, srcs, tpl.copy_stream, comp)
            if e:
                e[1].record(comp)
            tb.tidal_lora_attach(tpl.h, targets[0], comp)
            if e:
                e[2].record(comp)
            if with_swap:
                tb.tidal_lora_swap(tpl.h, targets[1], comp)
            if e:
                e[3].record(comp)

        # ---- call level (--kernel-level-only: skipped, so that a profile holds nothing but the kernel-level pass)
        call_steps, call_warm = (0, 0) if args.kernel_level_only else (steps, warmup)
        for _ in range(call_warm):
            step(Tp)
        Tp.sync()
        evs = [[ev() for _ in range(4)] for _ in range(call_steps)]
        t0 = time.perf_counter()
        for k in range(call_steps):
            step(Tp, evs[k])
        Tp.sync()
        wall_ms = (time.perf_counter() - t0) * 1e3 / max(1, call_steps)
        stp = tb.tidal_get_stats(Tp.h)
        med = lambda x: float(np.median(x)) if x else float("nan")
        mat_ms = med([e[0].elapsed_time(e[1]) for e in evs])
        att_ms = med([e[1].elapsed_time(e[2]) for e in evs])
        swp_ms = med([e[2].elapsed_time(e[3]) for e in evs]) if with_swap else None
        n_calls = (call_steps + call_warm) * (2 if with_swap else 1)
        launches_per_call = stp["lora_launches"] / max(1, n_calls)
        # ---- kernel level: the same rows of the path with the adapter uploaded first and merged afterwards by one
        # launch per shape (tidal_adapter_upload + tidal_lora_attach_adapter), so that the read-modify-write kernel
        # runs with nothing else on the GPU and its duration, bracketed by the library's events, is its own.  (In the
        # pipelined call above its launches are cut into groups and share HBM with the copy engine and the pack kernel.)
        comp = T.compute_stream
        amem = [torch.empty(tb.tidal_adapter_required_bytes(T.h, t_), dtype=torch.uint8, device="cuda:0") for t_ in targets]
        live = []

        def kstep():
            tb.tidal_materialize(T.h, srcs, T.copy_stream, comp)          # resets the template: nothing attached afterwards
            for h in live:
                tb.tidal_adapter_destroy(h)
            live.clear()
            live.append(tb.tidal_adapter_upload(T.h, targets[0], amem[0], amem[0].numel(), comp))
            tb.tidal_lora_attach_adapter(T.h, live[0], comp)
            if with_swap:
                live.append(tb.tidal_adapter_upload(T.h, targets[1], amem[1], amem[1].numel(), comp))
                tb.tidal_lora_swap_adapter(T.h, live[1], comp)

        kstep()
        T.sync()
        tb.tidal_reset_stats(T.h)
        for k in range(steps):
            kstep()
        T.sync()
        st = tb.tidal_get_stats(T.h)

        fb = factor_bytes(wl, wl.lora_slots, wl.rank)
        attach_bytes = 4 * wl.lora_w_elements + fb
        swap_bytes = 4 * wl.lora_w_elements + 2 * fb
        launches = st["lora_launches"]
        bytes_per_launch = steps * (attach_bytes + (swap_bytes if with_swap else 0)) / max(1, launches)
        avg_ms = st["lora_kernel_ms"] / max(1, launches)
        gbps = bytes_per_launch / (avg_ms * 1e-3) / 1e9
        mat_gbps = wl.source_bytes / (mat_ms * 1e-3) / 1e9

        # ---- keep-alive regime: the adapter stays resident, detach / attach back to back, kernels only
        tb.tidal_reset_stats(T.h)
        for _ in range(2):
            tb.tidal_lora_detach(T.h, comp)
            tb.tidal_lora_attach_adapter(T.h, live[-1], comp)
        T.sync()
        stw = tb.tidal_get_stats(T.h)
        warm_ms = stw["lora_kernel_ms"] / max(1, stw["lora_launches"])
        warm_gbps = 4 * attach_bytes / max(1, stw["lora_launches"]) / (warm_ms * 1e-3) / 1e9

        info = tb.tidal_lora_launch_info(T.h, wl.tensors[wl.lora_slots[0]].rows, wl.tensors[wl.lora_slots[0]].cols,
                                         min(128, len(wl.lora_slots)), 0, wl.rank)
        rec.update({
            "workload": "%s: %d tensors, %.2f GB %s host -> bf16 slots%s; LoRA r=%d alpha=%g on %d targets; step = materialize + attach%s" % (
                wl.name, len(wl.tensors), wl.source_bytes / 1e9, {0: "fp32", 1: "fp16", 2: "bf16"}[wl.host_dtype],
                " (host pool wrapped into %.0f GiB)" % (pool_limit / 2 ** 30) if pool.wrapped else "",
                wl.rank, wl.alpha, len(wl.lora_slots), " + swap" if with_swap else ""),
            "steps": steps, "ms_per_step": round(wall_ms, 3),
            "materialize": {"value": round(mat_gbps, 2), "unit": "GB/s (source bytes over PCIe, H2D+convert)", "ms": round(mat_ms, 2),
                            "h2d_peak_measured": round(pcie_peak, 2), "frac_of_measured_peak": round(mat_gbps / pcie_peak, 4),
                            "chunks_per_step": stp["chunks"] // max(1, call_steps + call_warm), "h2d_copies_per_step": stp["h2d_copies"] // max(1, call_steps + call_warm),
                            "convert_kernel_ms_per_step": round(st["convert_kernel_ms"] / max(1, steps), 3)},
            "lora": {"attach_ms_per_invocation": round(att_ms, 4),
                     "swap_ms_per_invocation": round(swp_ms, 4) if swp_ms is not None else None,
                     "note": "tidal_lora_attach / _swap with host pointers: per-invocation times include the adapter's upload over PCIe "
                             "and its packing, overlapped with the merge in groups of targets (launches_per_invocation)",
                     "launches_per_invocation": launches_per_call,
                     "upload_groups_targets": tb.tidal_lora_upload_plan(Tp.h, targets[0]),
                     "kernel_ms_per_invocation_alone": round(st["lora_kernel_ms"] / (steps * (2 if with_swap else 1)), 4),
                     "keep_alive_kernel_GBps": round(warm_gbps, 1), "keep_alive_frac_of_hbm_peak": round(warm_gbps / HBM_PEAK_GBPS, 4),
                     "keep_alive_note": "the same adapter resident in HBM, detach / attach issued back to back after the steps (the kept-alive "
                                        "function of Sec. 5.2): one launch per shape, nothing crossing the link; the first pass after a load or "
                                        "an idle gap also runs a few percent slower than the ones that follow"},
            "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(traffic_key),
                         "kernel": info["kernel"], "avg_launch_ms": round(avg_ms, 4), "launches": launches,
                         "algorithmic_bytes_per_launch": bytes_per_launch},
            "value": round(gbps, 1)})
        log("%s: materialize %.1f ms (%.1f GB/s), attach %.3f ms/invocation, LoRA kernels %.1f GB/s (%.1f%% of peak; keep-alive %.1f%%)" %
            (tag, mat_ms, mat_gbps, att_ms, gbps, gbps / 80, warm_gbps / 80))

        # ---- oracle on bands of sampled targets: conversion, attach (+ swap), then the keep-alive passes are undone first
        # bring the template back to the state right after the last step: it now holds base + last adapter, as then
        if cpu_seconds > 0:
            smp = OracleSample(cpu_seconds)
            by_shape = {}
            for idx, s in enumerate(wl.lora_slots):
                by_shape.setdefault((wl.tensors[s].rows, wl.tensors[s].cols), []).append(idx)
            order = []                       # first, last, middle, then further targets of every shape, round robin over shapes,
            for frac in (0.0, 1.0, 0.5, 0.25, 0.75, 0.125, 0.875, 0.375, 0.625, 0.0625, 0.9375):   # until the time budget is spent
                for shape, idxs in by_shape.items():
                    order.append(idxs[min(len(idxs) - 1, int(frac * (len(idxs) - 1) + 0.5))])
            seen = set()
            for k, idx in enumerate(order):
                if idx in seen:
                    continue
                seen.add(idx)
                s = wl.lora_slots[idx]
                t = wl.tensors[s]
                r0, r1 = band_of(t.rows, k, 256)
                src = np.ascontiguousarray(pool.views[s][r0:r1])
                W = smp.convert(src)
                chain = []
                for a, (items, _) in enumerate(ads):
                    _, al, A, B = items[idx]
                    Ab = smp.orc.convert_to_bf16(A)
                    Bb = smp.orc.convert_to_bf16(np.ascontiguousarray(B[r0:r1]))
                    if a == 1:
                        chain.append((-1, chain[0][1], chain[0][2], chain[0][3]))
                    chain.append((+1, al, Ab, Bb))
                smp.passes(W, chain)
                # the keep-alive section left base + last adapter merged twice more (detach, attach): the oracle follows
                last = chain[-1]
                smp.passes(W, [(-1, last[1], last[2], last[3]), (+1, last[1], last[2], last[3])] * 2)
                got = T.slot_bytes(s)[2 * r0 * t.cols: 2 * r1 * t.cols].cpu().numpy().view(np.uint16).reshape(r1 - r0, t.cols)
                smp.compare(got, W, np)
                if smp.spent() > cpu_seconds and len(seen) >= len(by_shape):
                    break
            # conversion and placement bit for bit on untargeted slots (and on targeted ones before any merge:
            # covered by the tests; here the first and last tensor, whole rows)
            for s in (0, len(wl.tensors) - 1):
                t = wl.tensors[s]
                r0, r1 = band_of(t.rows, 1, 128)
                want = smp.convert(np.ascontiguousarray(pool.views[s][r0:r1]))
                got = T.slot_bytes(s)[2 * r0 * t.cols: 2 * r1 * t.cols].cpu().numpy().view(np.uint16).reshape(r1 - r0, t.cols)
                smp.compare(got, want, np, exact=True)
            rec["cpu_baseline"], rec["parity"] = smp.records("%s, bands of 256 rows of %d targeted slots" % (wl.name, len(seen)), os.cpu_count() or 0)
            log("%s: oracle %.3f GB/s (LoRA), parity worst %.3g (bound %.3g), conversion bit-exact: %s" %
                (tag, rec["cpu_baseline"]["value"] or 0.0, smp.worst, TOL, smp.exact_convert))
        else:
            rec["cpu_baseline"], rec["parity"] = None, None
    finally:
        torch.cuda.synchronize()
        tb.tidal_template_destroy(T.h)           # the resident adapter is still attached: the template goes first
        T.h = None
        Tp.close()
    del pool, T, Tp
    torch.cuda.empty_cache()
    return rec


def run_single(args, pcie_peak, cpu_seconds):
    """Configuration 1: one 4096 x 4096 fp32 layer, r = 8: materialize, attach, swap.  W (32 MiB) fits the
    Infinity Cache, so the kernel rate is measured rotating over 24 distinct copies."""
    import numpy as np
    import torch
    from paper_2503_06421_amd import binding as tb
    from paper_2503_06421_amd import harness as hz
    from paper_2503_06421_amd import workloads as wl_mod

    wl = wl_mod.single_linear()
    copies = 24
    pool = hz.HostPool(wl)
    ads = [hz.pinned_adapter(wl, a) for a in (0, 1)]
    T = hz.DeviceTemplate(wl.shapes * copies, max_adapter_bytes=hz.packed_adapter_bytes(wl), flags=tb.TIDAL_FLAG_KERNEL_TIMING)
    comp = T.compute_stream
    ev = lambda: torch.cuda.Event(enable_timing=True)
    src0 = pool.sources()[0]
    rec = {"config": "1 single linear layer"}
    try:
        def tg(a, slot):
            _, al, A, B = ads[a][0][0]
            return tb.targets_from_arrays([(slot, al, A, B)])

        mat, att, swp = [], [], []
        for rep in range(8):
            slot = rep % copies
            e = [ev() for _ in range(4)]
            e[0].record(comp)
            tb.tidal_materialize(T.h, [(slot, src0[1], src0[2])], T.copy_stream, comp)
            e[1].record(comp)
            tb.tidal_lora_attach(T.h, tg(0, slot), comp)
            e[2].record(comp)
            tb.tidal_lora_swap(T.h, tg(1, slot), comp)
            e[3].record(comp)
            T.sync()
            if rep >= 2:
                mat.append(e[0].elapsed_time(e[1])); att.append(e[1].elapsed_time(e[2])); swp.append(e[2].elapsed_time(e[3]))
            if rep < 7:
                tb.tidal_lora_detach(T.h, comp)
                T.sync()
        # kernel rate fed from HBM: resident adapters, rotating over distinct copies of W
        tb.tidal_lora_detach(T.h, comp)
        tb.tidal_materialize(T.h, [(i, src0[1], src0[2]) for i in range(copies)], T.copy_stream, comp)
        T.sync()
        mems, handles = [], []
        for slot in range(copies):
            for a in (0, 1):
                t_ = tg(a, slot)
                nb = tb.tidal_adapter_required_bytes(T.h, t_)
                mem = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
                handles.append(tb.tidal_adapter_upload(T.h, t_, mem, nb, comp))
                mems.append(mem)
        T.sync()
        tb.tidal_reset_stats(T.h)
        reps = 3
        for rep in range(reps):
            for slot in range(copies):
                tb.tidal_lora_attach_adapter(T.h, handles[2 * slot], comp)
                tb.tidal_lora_swap_adapter(T.h, handles[2 * slot + 1], comp)
                tb.tidal_lora_detach(T.h, comp)
        T.sync()
        st = tb.tidal_get_stats(T.h)
        fb = factor_bytes(wl, [0], wl.rank)
        total_bytes = reps * copies * (2 * (4 * wl.lora_w_elements + fb) + (4 * wl.lora_w_elements + 2 * fb))
        avg_ms = st["lora_kernel_ms"] / st["lora_launches"]
        gbps = total_bytes / st["lora_launches"] / (avg_ms * 1e-3) / 1e9
        mat_ms = float(np.median(mat))
        info = tb.tidal_lora_launch_info(T.h, 4096, 4096, 1, 0, wl.rank)
        rec.update({
            "workload": "single_linear: W 4096x4096 fp32 host U[-0.02,0.02] -> bf16; LoRA r=8 alpha=16; materialize, attach, swap to a second adapter",
            "materialize": {"value": round(wl.source_bytes / mat_ms / 1e6, 2), "unit": "GB/s (source bytes over PCIe, H2D+convert)", "ms": round(mat_ms, 4),
                            "h2d_peak_measured": round(pcie_peak, 2), "frac_of_measured_peak": round(wl.source_bytes / mat_ms / 1e6 / pcie_peak, 4)},
            "lora": {"attach_ms_per_invocation": round(float(np.median(att)), 4), "swap_ms_per_invocation": round(float(np.median(swp)), 4),
                     "note": "a 64 MiB pass: the invocation is bound by launch and PCIe latency of the 256 KB of factors, not by bandwidth"},
            "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4),
                         "traffic": None, "kernel": info["kernel"], "avg_launch_ms": round(avg_ms, 5), "launches": st["lora_launches"],
                         "algorithmic_bytes_per_launch": total_bytes / st["lora_launches"],
                         "note": "resident adapters, rotating over %d copies of W (%d MiB) so that no pass is served from the Infinity Cache" % (copies, 32 * copies)},
            "value": round(gbps, 1)})
        if cpu_seconds > 0:
            smp = OracleSample(cpu_seconds)
            W = smp.convert(pool.views[0])
            a0 = [smp.orc.convert_to_bf16(x) for x in ads[0][0][0][2:]]
            a1 = [smp.orc.convert_to_bf16(x) for x in ads[1][0][0][2:]]
            al = wl.alpha
            seq = []
            for rep in range(reps):                                # what every copy went through in the rotation
                seq += [(+1, al, a0[0], a0[1]), (-1, al, a0[0], a0[1]), (+1, al, a1[0], a1[1]), (-1, al, a1[0], a1[1])]
            smp.passes(W, seq)
            smp.compare(T.slot_host(copies - 1), W, np)
            rec["cpu_baseline"], rec["parity"] = smp.records("single_linear, the whole 4096 x 4096 tensor", os.cpu_count() or 0)
        for h in handles:
            tb.tidal_adapter_destroy(h)
        log("single: materialize %.3f ms, attach %.1f us, swap %.1f us per invocation; HBM-fed kernels %.1f GB/s" %
            (mat_ms, 1e3 * float(np.median(att)), 1e3 * float(np.median(swp)), gbps))
    finally:
        T.close()
    return rec


def run_churn(args, cpu_seconds):
    """Configuration 4: resident 7B-shaped bf16 base, pool of 32 resident adapters (ranks from {8,16,32,64},
    alpha = 2r, targets q,k,v,o), 200 invocations by Zipf(1.1): step 0 attaches, every later one is a fused swap."""
    import numpy as np
    import torch
    from paper_2503_06421_amd import binding as tb
    from paper_2503_06421_amd import harness as hz
    from paper_2503_06421_amd import workloads as wl_mod

    ch = wl_mod.adapter_churn()
    wl = ch.base
    pool = hz.HostPool(wl, limit_bytes=2 << 30)            # the base's values do not matter here: a wrapped pool
    T = hz.DeviceTemplate(wl.shapes, flags=tb.TIDAL_FLAG_KERNEL_TIMING)
    comp = T.compute_stream
    ev = lambda: torch.cuda.Event(enable_timing=True)
    rec = {"config": "4 adapter churn"}
    handles, mems, host = {}, [], {}
    try:
        tb.tidal_materialize(T.h, pool.sources(), T.copy_stream, comp)
        T.sync()
        for a in sorted(set(ch.schedule)):
            items, keep = hz.pinned_adapter(wl, a, rank=ch.ranks[a], alpha=ch.alphas[a])
            t_ = tb.targets_from_arrays(items)
            nb = tb.tidal_adapter_required_bytes(T.h, t_)
            mem = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
            handles[a] = tb.tidal_adapter_upload(T.h, t_, mem, nb, comp)
            T.sync()
            mems.append(mem)
            host[a] = (items, keep)
        sample_slots = [wl.lora_slots[0], wl.lora_slots[len(wl.lora_slots) // 2], wl.lora_slots[-1]]
        per_step, cur = [], None
        before_last = None
        for step, a in enumerate(ch.schedule):
            if step == len(ch.schedule) - 1:
                before_last = {s: T.slot_host(s)[1000:1256].copy() for s in sample_slots}
            tb.tidal_reset_stats(T.h)
            e0, e1 = ev(), ev()
            e0.record(comp)
            if step == 0:
                tb.tidal_lora_attach_adapter(T.h, handles[a], comp)
            else:
                tb.tidal_lora_swap_adapter(T.h, handles[a], comp)
            e1.record(comp)
            T.sync()
            st = tb.tidal_get_stats(T.h)
            per_step.append((ch.ranks[cur] if cur is not None else 0, ch.ranks[a], e0.elapsed_time(e1), st["lora_kernel_ms"], cur))
            prev, cur = cur, a
        swaps = per_step[1:]
        call = np.array([s[2] for s in swaps])
        kern = np.array([s[3] for s in swaps])
        byte_of = lambda r0, r1: 4 * wl.lora_w_elements + factor_bytes(wl, wl.lora_slots, r0) + factor_bytes(wl, wl.lora_slots, r1)
        total_bytes = sum(byte_of(r0, r1) for r0, r1, *_ in swaps)
        gbps = total_bytes / kern.sum() / 1e6
        by = {}
        for r0, r1, c, k, _ in swaps:
            by.setdefault((r0, r1), []).append(k)
        rec.update({
            "workload": "adapter_churn: resident 7B-shaped bf16 base, pool of 32 resident adapters (ranks from {8,16,32,64}, alpha=2r) on q,k,v,o "
                        "of 32 layers (128 targets of 4096x4096), 200 invocations by Zipf(1.1): 1 attach + 199 fused swaps",
            "lora": {"swap_ms_per_invocation": {"mean": round(float(call.mean()), 4), "p50": round(float(np.median(call)), 4),
                                                "p95": round(float(np.percentile(call, 95)), 4)},
                     "first_attach_ms": round(per_step[0][2], 4),
                     "by_rank_pair_GBps": {"%d->%d" % k: round(byte_of(*k) / float(np.median(v)) / 1e6, 0) for k, v in sorted(by.items())}},
            "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4),
                         "traffic": measured_traffic("adapter_churn"), "kernel": "lora_mfma_kernel / lora_mfma_lds_kernel (by rank pair)", "avg_launch_ms": round(float(kern.mean()), 4),
                         "launches": len(swaps), "algorithmic_bytes_per_launch": total_bytes / len(swaps)},
            "value": round(gbps, 1)})
        log("churn: %.3f ms per swap (p95 %.3f), kernels %.1f GB/s (%.1f%% of peak)" % (float(call.mean()), float(np.percentile(call, 95)), gbps, gbps / 80))
        if cpu_seconds > 0:
            smp = OracleSample(cpu_seconds)
            a_old, a_new = ch.schedule[-2], ch.schedule[-1]
            for s in sample_slots:
                idx = wl.lora_slots.index(s)
                W = before_last[s].copy()
                seq = []
                for sign, a in ((-1, a_old), (+1, a_new)):
                    _, al, A, B = host[a][0][idx]
                    seq.append((sign, al, smp.orc.convert_to_bf16(A), smp.orc.convert_to_bf16(np.ascontiguousarray(B[1000:1256]))))
                smp.passes(W, seq)
                smp.compare(T.slot_host(s)[1000:1256], W, np)
                if smp.spent() > cpu_seconds:
                    break
            rec["cpu_baseline"], rec["parity"] = smp.records("adapter_churn, the last swap (ranks %d -> %d) on rows 1000..1255 of sampled slots" %
                                                             (ch.ranks[a_old], ch.ranks[a_new]), os.cpu_count() or 0)
        tb.tidal_lora_detach(T.h, comp)
        T.sync()
    finally:
        torch.cuda.synchronize()
        for h in handles.values():
            try:
                tb.tidal_adapter_destroy(h)
            except tb.TidalError:
                pass
        T.close()
    return rec


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--chunk-mib", type=int, default=128)
    ap.add_argument("--pool-gib", type=float, default=8.0, help="pinned host pool the 70B- and 13B-shaped stacks are mapped into")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget for the oracle baseline of the headline workload (a third of it for each other one); 0 = skip")
    ap.add_argument("--kernel-level-only", action="store_true",
                    help="skip the call-level pass of the stack workloads (their per-invocation figures are then NaN): for "
                         "profiling runs whose counters should cover the kernel-level pass and nothing else")
    ap.add_argument("--only", default="", help="comma-separated subset of 70b,single,7b,13b,churn (the headline needs 70b)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch

    from paper_2503_06421_amd import binding as tb
    from paper_2503_06421_amd import workloads as wl_mod

    if not os.path.exists(tb.LIB_PATH):
        from paper_2503_06421_amd import build
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU path)"
    torch.cuda.set_device(0)
    only = set(x for x in args.only.split(",") if x) or {"70b", "single", "7b", "13b", "churn"}

    # ---- link peak and stand-alone conversion (same run, same box) ------------------------------------
    probe_bytes = 1 << 30
    probe_buf = torch.empty(probe_bytes, dtype=torch.uint8, device="cuda:0")
    s0 = torch.cuda.Stream()
    pcie_peak = tb.tidal_h2d_peak(probe_buf, probe_bytes, 5, s0)
    log("measured host->device peak: %.1f GB/s (1 GiB pinned hipMemcpyAsync, best of 5)" % pcie_peak)
    n_conv = probe_bytes // 2
    conv_dst = torch.empty(n_conv, dtype=torch.int16, device="cuda:0")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(2):
        tb.tidal_convert_device(conv_dst, probe_buf, tb.TIDAL_F16, n_conv, s0)
    ev[0].record(s0)
    for _ in range(10):
        tb.tidal_convert_device(conv_dst, probe_buf, tb.TIDAL_F16, n_conv, s0)
    ev[1].record(s0)
    torch.cuda.synchronize()
    conv_ms = ev[0].elapsed_time(ev[1]) / 10
    conv_gbps = 4.0 * n_conv / (conv_ms * 1e-3) / 1e9
    del conv_dst, probe_buf
    torch.cuda.empty_cache()

    pool_limit = int(args.pool_gib * 2 ** 30)
    head = None
    configs = []
    t_all = time.perf_counter()
    if "70b" in only:
        head = run_stack("5 llama3-70b-shaped", wl_mod.llama3_70b(), args, pcie_peak, pool_limit, args.steps, args.warmup, False,
                         args.cpu_seconds, "llama3_70b_shaped")
    sub = args.cpu_seconds / 3.0
    if "single" in only:
        configs.append(run_single(args, pcie_peak, sub))
    if "7b" in only:
        configs.append(run_stack("2 llama2-7b-shaped", wl_mod.llama2_7b(), args, pcie_peak, None, 2, 1, True, sub, "llama2_7b_shaped"))
    if "13b" in only:
        configs.append(run_stack("3 llama2-13b-shaped", wl_mod.llama2_13b(), args, pcie_peak, pool_limit, 2, 1, False, sub, "llama2_13b_shaped"))
    if "churn" in only:
        configs.append(run_churn(args, sub))
    log("all configurations done in %.0f s" % (time.perf_counter() - t_all))
    if head is None:
        head = configs[0]

    parity_ok = all(c["parity"] is None or c["parity"]["ok"] for c in [head] + configs if "parity" in c)
    out = {
        "metric": "weights materialized GB/s (H2D+convert) and LoRA merge/swap GB/s; ms/invocation",
        "value_is": "LoRA merge GB/s of the headline workload with W and packed adapters resident in HBM (materialize GB/s, PCIe-inclusive, is under 'materialize')",
        "value": head["value"] if parity_ok else None,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": head.get("steps", args.steps),
        "warmup": args.warmup,
        "ms_per_step": head.get("ms_per_step"),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": head["workload"], "chunk_mib": args.chunk_mib},
        "roofline": head["roofline"],
        "cpu_baseline": head.get("cpu_baseline"),
        "materialize": head.get("materialize"),
        "lora": head.get("lora"),
        "convert_standalone": {"value": round(conv_gbps, 1), "unit": "GB/s (fp16 in + bf16 out)", "ms_per_GiB_src": round(conv_ms, 4),
                               "frac_of_hbm_peak": round(conv_gbps / HBM_PEAK_GBPS, 4)},
        "parity": head.get("parity"),
        "parity_ok": parity_ok,
        "configs": configs,
    }
    print(json.dumps(out), flush=True)
    if not parity_ok:
        log("PARITY FAILURE: a compared band differs from the oracle beyond the bound; see 'parity' of each configuration")
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
