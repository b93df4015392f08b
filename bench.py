#!/usr/bin/env python3
"""Benchmark of the template-materialisation + LoRA attach/swap hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One *step* is one pass of the whole path over the Llama2-7B-shaped workload:
  tidal_materialize   226 fp16 host tensors (13.48 GB, pinned pool) -> bf16 template slots,
                      chunked pinned H2D on a copy stream overlapped with the convert kernel,
  tidal_lora_attach   adapter 0 (r=16, alpha=32 on q and v of all 32 layers): upload + merge,
  tidal_lora_swap     adapter 1 of the same shape: upload + fused unmerge/merge.

The line printed at the end is JSON.  `value` is the LoRA merge/swap throughput with W and
the packed adapters resident in HBM: algorithmic bytes (4 B per targeted W element, plus the
packed A/B read once) divided by the duration of the read-modify-write kernels, which the
library brackets with HIP events on the launch stream.  The PCIe-inclusive materialisation
rate is reported next to it under "materialize" (never as `value`), with the host->device
link peak measured in the same run.  "cpu_baseline" times the CPU oracle on a bounded sample
of the same LoRA work.
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
# HBM bytes per lora_mfma_kernel launch on the default workload (32 layers, r=16, 64 targets), from
# the two rocprofv3 --pmc runs (FETCH_SIZE x 2.0 calibration factor + WRITE_SIZE x 1.0) whose
# summary is kept under profiles/: mean of the attach and the fused-swap launch.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = 4_320_981_000


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--layers", type=int, default=32, help="fewer layers for a quick functional run (not a valid score)")
    ap.add_argument("--chunk-mib", type=int, default=128)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget for the oracle baseline; 0 = skip")
    ap.add_argument("--pipelined-upload", action="store_true",
                    help="TIDAL_FLAG_PIPELINED_UPLOAD: adapter upload overlapped with the merge in three groups (not the default run)")
    ap.add_argument("--threads", type=int, default=0, help="host threads for drawing the synthetic tensors")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2503_06421_amd import binding as tb
    from paper_2503_06421_amd import workloads as wl_mod

    if not os.path.exists(tb.LIB_PATH):
        from paper_2503_06421_amd import build
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU path)"
    torch.cuda.set_device(0)
    threads = args.threads or min(16, os.cpu_count() or 1)

    # ---- workload: pinned host pool, tensors back to back like a template server's pool ----
    wl = wl_mod.llama2_7b(layers=args.layers)
    t0 = time.perf_counter()
    isz = wl_mod.ITEMSIZE[wl.host_dtype]
    npdt = wl_mod.NP_DTYPE[wl.host_dtype]
    pool = torch.empty(wl.source_bytes, dtype=torch.uint8, pin_memory=True)
    pool_np = pool.numpy()
    views, off = [], 0
    for t in wl.tensors:
        n = t.numel * isz
        views.append(pool_np[off:off + n].view(npdt).reshape(t.rows, t.cols))
        off += n
    wl_mod.draw_all(wl, views, threads=threads)
    log("drew %d tensors, %.2f GB, in %.1f s (%d threads)" % (len(views), wl.source_bytes / 1e9,
                                                              time.perf_counter() - t0, threads))

    adapters = []           # two adapters, host dtype of the base, each one contiguous pinned block
    keep = []               # (A, B of target 0, A, B of target 1, ...) like an adapter checkpoint in a host pool
    for a in (0, 1):
        mats = []
        for s in wl.lora_slots:
            mats.extend(wl_mod.draw_adapter(wl, a, s))
        blob = torch.empty(sum(m.size * m.itemsize for m in mats), dtype=torch.uint8, pin_memory=True)
        keep.append(blob)
        items, o = [], 0
        for m in mats:
            v = blob.numpy()[o:o + m.size * m.itemsize].view(m.dtype).reshape(m.shape)
            v[...] = m
            items.append(v)
            o += m.size * m.itemsize
        adapters.append([(s, wl.alpha, items[2 * i], items[2 * i + 1]) for i, s in enumerate(wl.lora_slots)])
    targets = [tb.targets_from_arrays(ad) for ad in adapters]

    # ---- template ----------------------------------------------------------------------------
    probe_cfg = tb.make_config(chunk_bytes=args.chunk_mib << 20, max_adapter_bytes=0)
    need0 = tb.tidal_template_required_bytes(wl.shapes, probe_cfg)
    arena0 = torch.empty(need0, dtype=torch.uint8, device="cuda:0")
    t_probe = tb.tidal_template_create(wl.shapes, arena0, need0, probe_cfg)
    adapter_bytes = tb.tidal_adapter_required_bytes(t_probe, targets[0])
    tb.tidal_template_destroy(t_probe)
    del arena0
    cfg = tb.make_config(chunk_bytes=args.chunk_mib << 20, max_adapter_bytes=adapter_bytes,
                         flags=tb.TIDAL_FLAG_KERNEL_TIMING | (tb.TIDAL_FLAG_PIPELINED_UPLOAD if args.pipelined_upload else 0))
    need = tb.tidal_template_required_bytes(wl.shapes, cfg)
    arena = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    T = tb.tidal_template_create(wl.shapes, arena, need, cfg)
    copy_s, comp_s = torch.cuda.Stream(), torch.cuda.Stream()
    srcs = [(i, wl.host_dtype, tb.host_ptr(v)) for i, v in enumerate(views)]

    # ---- link peak (same run, same box) ---------------------------------------------------------
    probe_bytes = 1 << 30
    probe_buf = torch.empty(probe_bytes, dtype=torch.uint8, device="cuda:0")
    pcie_peak = tb.tidal_h2d_peak(probe_buf, probe_bytes, 5, copy_s)
    log("measured host->device peak: %.1f GB/s (1 GiB pinned hipMemcpyAsync, best of 5)" % pcie_peak)

    # ---- standalone convert kernel (device-resident source) ----------------------------------------
    n_conv = probe_bytes // 2
    conv_dst = torch.empty(n_conv, dtype=torch.int16, device="cuda:0")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(2):
        tb.tidal_convert_device(conv_dst, probe_buf, tb.TIDAL_F16, n_conv, comp_s)
    ev[0].record(comp_s)
    for _ in range(10):
        tb.tidal_convert_device(conv_dst, probe_buf, tb.TIDAL_F16, n_conv, comp_s)
    ev[1].record(comp_s)
    torch.cuda.synchronize()
    conv_ms = ev[0].elapsed_time(ev[1]) / 10
    conv_gbps = 4.0 * n_conv / (conv_ms * 1e-3) / 1e9
    del conv_dst, probe_buf

    # ---- steps ---------------------------------------------------------------------------------------
    def step(events=None):
        if events:
            events[0].record(comp_s)
        tb.tidal_materialize(T, srcs, copy_s, comp_s)
        if events:
            events[1].record(comp_s)
        tb.tidal_lora_attach(T, targets[0], comp_s)
        if events:
            events[2].record(comp_s)
        tb.tidal_lora_swap(T, targets[1], comp_s)
        if events:
            events[3].record(comp_s)

    for _ in range(args.warmup):
        step()
    tb.tidal_template_sync(T)
    torch.cuda.synchronize()
    tb.tidal_reset_stats(T)

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    lora_ms = []                      # kernel time per step, attach and swap separately
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    tb.tidal_template_sync(T)
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    st = tb.tidal_get_stats(T)
    ms_per_step = (t_end - t_start) * 1e3 / args.steps

    mat_ms = float(np.median([e[0].elapsed_time(e[1]) for e in evs]))
    att_ms = float(np.median([e[1].elapsed_time(e[2]) for e in evs]))
    swp_ms = float(np.median([e[2].elapsed_time(e[3]) for e in evs]))

    w_elems = wl.lora_w_elements
    # what the kernel reads of an adapter: bf16 A^T (in x rp) and B (out x rp), rank padded to 16
    packed = sum(2 * 16 * (wl.tensors[s].rows + wl.tensors[s].cols) for s in wl.lora_slots)
    attach_bytes = 4 * w_elems + packed
    swap_bytes = 4 * w_elems + 2 * packed
    launches = st["lora_launches"]
    kernel_ms_total = st["lora_kernel_ms"]
    avg_kernel_ms = kernel_ms_total / max(1, launches)
    # every timed step is one attach and one swap, however many launches the library makes of them
    bytes_per_launch = args.steps * (attach_bytes + swap_bytes) / max(1, launches)
    lora_gbps = bytes_per_launch / (avg_kernel_ms * 1e-3) / 1e9
    mat_gbps = wl.source_bytes / (mat_ms * 1e-3) / 1e9

    # ---- CPU oracle baseline on a bounded sample + parity of the sampled slots --------------------------
    cpu_baseline = None
    parity = None
    if args.cpu_seconds > 0:
        from oracle import tidal_oracle as orc
        done_bytes, done_s, n_done, max_rel = 0.0, 0.0, 0, 0.0
        for idx, s in enumerate(wl.lora_slots):
            Wo = orc.convert_to_bf16(views[s])
            a0 = [orc.convert_to_bf16(x) for x in adapters[0][idx][2:]]
            a1 = [orc.convert_to_bf16(x) for x in adapters[1][idx][2:]]
            c0 = time.perf_counter()
            orc.lora_merge(Wo, a0[0], a0[1], wl.alpha, +1)
            orc.lora_swap(Wo, a0[0], a0[1], wl.alpha, a1[0], a1[1], wl.alpha)
            done_s += time.perf_counter() - c0
            elems = wl.tensors[s].numel
            per_slot_packed = packed / len(wl.lora_slots)
            done_bytes += 2 * 4 * elems + 3 * per_slot_packed
            n_done += 1
            p, nb = tb.tidal_template_slot_ptr(T, s)
            o = p - arena.data_ptr()
            got = arena[o:o + nb].cpu().numpy().view(np.uint16).reshape(Wo.shape)
            g = (got.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
            r = (Wo.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
            max_rel = max(max_rel, float(np.max(np.abs(g - r)) / np.max(np.abs(r))))
            if done_s * (n_done + 1) / n_done > args.cpu_seconds:
                break
        cpu_baseline = {"value": round(done_bytes / done_s / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
                        "sample": "attach+swap on the first %d of %d targeted 4096x4096 slots, %.1f s, "
                                  "host has %d logical cores" % (n_done, len(wl.lora_slots), done_s, os.cpu_count() or 0)}
        parity = {"slots_checked": n_done, "max_abs_err_over_max_abs_w": max_rel, "bound": 2.0 ** -7}
        if not max_rel <= 2.0 ** -7:
            log("PARITY FAILURE: %g" % max_rel)

    tb.tidal_template_destroy(T)

    out = {
        "metric": "weights materialized GB/s (H2D+convert) and LoRA merge/swap GB/s; ms/invocation",
        "value_is": "LoRA merge/swap GB/s with W and packed adapters resident in HBM (materialize GB/s, PCIe-inclusive, is under 'materialize')",
        "value": round(lora_gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: %d layers, %d tensors fp16 N(0,0.02) -> bf16 slots; LoRA r=%d alpha=%g on q,v "
                               "(%d targets); step = materialize + attach + swap" %
                               (wl.name, args.layers, len(wl.tensors), wl.rank, wl.alpha, len(wl.lora_slots)),
                   "chunk_mib": args.chunk_mib},
        "roofline": {"bound": "hbm", "achieved": round(lora_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(lora_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH if (args.layers == 32 and wl.rank == 16) else None,
                     "kernel": "lora_mfma_kernel", "avg_launch_ms": round(avg_kernel_ms, 4),
                     "launches": launches, "algorithmic_bytes_per_launch": bytes_per_launch},
        "cpu_baseline": cpu_baseline,
        "materialize": {"value": round(mat_gbps, 2), "unit": "GB/s (source bytes over PCIe, H2D+convert)",
                        "ms": round(mat_ms, 2), "h2d_peak_measured": round(pcie_peak, 2),
                        "frac_of_measured_peak": round(mat_gbps / pcie_peak, 4),
                        "chunks_per_step": st["chunks"] // max(1, args.steps),
                        "h2d_copies_per_step": st["h2d_copies"] // max(1, args.steps),
                        "convert_kernel_ms_per_step": round(st["convert_kernel_ms"] / max(1, args.steps), 3)},
        "lora": {"attach_ms_per_invocation": round(att_ms, 4), "swap_ms_per_invocation": round(swp_ms, 4),
                 "note": "per-invocation times include the adapter upload over PCIe and packing",
                 "kernel_ms_avg": round(avg_kernel_ms, 4)},
        "convert_standalone": {"value": round(conv_gbps, 1), "unit": "GB/s (fp16 in + bf16 out)", "ms_per_GiB_src": round(conv_ms, 4),
                               "frac_of_hbm_peak": round(conv_gbps / HBM_PEAK_GBPS, 4)},
        "parity": parity,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
