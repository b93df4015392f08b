"""Plumbing shared by bench.py and the per-configuration benchmark: pinned host pools, device
arenas and adapter blobs come from PyTorch; every operation on them goes through the C ABI.
Nothing here computes on tensor data."""
from __future__ import annotations

import os
import time

import numpy as np
import torch

from . import binding as tb
from . import workloads as wl_mod


def host_threads() -> int:
    return min(16, os.cpu_count() or 1)


class HostPool:
    """The workload's host tensors back to back in one pinned allocation (what a template
    server's host memory pool looks like to the copy engine).  If `limit_bytes` is smaller than
    the workload, tensors are mapped into the pool modulo its size at distinct offsets, so the
    whole stack can be streamed without holding all of it in host memory; contents then repeat
    (placement is still checkable, every tensor starts at its own offset)."""

    def __init__(self, wl: wl_mod.Workload, limit_bytes: int | None = None, draw: bool = True, threads: int = 0):
        self.wl = wl
        isz = wl_mod.ITEMSIZE[wl.host_dtype]
        npdt = wl_mod.NP_DTYPE[wl.host_dtype]
        total = wl.source_bytes
        self.wrapped = limit_bytes is not None and limit_bytes < total
        size = limit_bytes if self.wrapped else total
        self.buf = torch.empty(size, dtype=torch.uint8, pin_memory=True)
        raw = self.buf.numpy()
        self.views = []
        t0 = time.perf_counter()
        if not self.wrapped:
            off = 0
            for t in wl.tensors:
                n = t.numel * isz
                self.views.append(raw[off:off + n].view(npdt).reshape(t.rows, t.cols))
                off += n
            if draw:
                wl_mod.draw_all(wl, self.views, threads=threads or host_threads())
        else:
            # fill the pool once from one stream, then hand out windows
            if draw:
                from concurrent.futures import ThreadPoolExecutor
                flat = raw.view(npdt)
                nseg = 256
                step = -(-flat.size // nseg)
                with ThreadPoolExecutor(max_workers=threads or host_threads()) as ex:
                    list(ex.map(lambda k: wl_mod.draw_into(flat[k * step:(k + 1) * step], wl.wid, (1 << 40) + k,
                                                           "normal", 0.02, wl.host_dtype), range(nseg)))
            off = 0
            for t in wl.tensors:
                n = t.numel * isz
                assert n <= size, "pool smaller than the largest tensor"
                if off + n > size:
                    off = (off + n) % 4096 * 16      # wrap to a small, tensor-specific offset
                self.views.append(raw[off:off + n].view(npdt).reshape(t.rows, t.cols))
                off += n
        self.draw_seconds = time.perf_counter() - t0

    def sources(self):
        return [(i, self.wl.host_dtype, tb.host_ptr(v)) for i, v in enumerate(self.views)]


def pinned_adapter(wl: wl_mod.Workload, adapter_id: int, rank: int | None = None, alpha: float | None = None):
    """One adapter as a contiguous pinned blob (A, B of target 0, A, B of target 1, ...), the way an
    adapter checkpoint sits in a host pool.  Returns (items, keepalive) with items =
    [(slot, alpha, A, B)]."""
    mats = []
    for s in wl.lora_slots:
        mats.extend(wl_mod.draw_adapter(wl, adapter_id, s, rank=rank))
    nbytes = sum(m.size * m.itemsize for m in mats)
    blob = torch.empty(max(nbytes, 1), dtype=torch.uint8, pin_memory=True)
    raw = blob.numpy()
    items, o = [], 0
    for m in mats:
        n = m.size * m.itemsize
        v = raw[o:o + n].view(m.dtype).reshape(m.shape)
        v[...] = m
        items.append(v)
        o += n
    al = wl.alpha if alpha is None else alpha
    return [(s, al, items[2 * i], items[2 * i + 1]) for i, s in enumerate(wl.lora_slots)], blob


def packed_adapter_bytes(wl: wl_mod.Workload, rank: int | None = None) -> int:
    """Size of the packed device copy of one adapter: per target A transposed (in rounded up to 256
    columns) and B (out rounded up to 32 rows), rp bf16 each, 256-B aligned."""
    r = wl.rank if rank is None else rank
    rp = 0 if r <= 0 else (16 if r <= 16 else (32 if r <= 32 else 64))
    total = 0
    for s in wl.lora_slots:
        t = wl.tensors[s]
        total += -(-2 * (-(-t.cols // 256) * 256) * rp // 256) * 256 + -(-2 * (-(-t.rows // 32) * 32) * rp // 256) * 256
    return total


class DeviceTemplate:
    """Template over a torch-allocated arena, with its two streams."""

    def __init__(self, shapes, arena=None, **cfg):
        """arena: reuse another template's device memory (same shapes and sizes in cfg; one of the
        two templates is in use at a time), else a new allocation."""
        self.cfg = tb.make_config(**cfg)
        self.need = tb.tidal_template_required_bytes(shapes, self.cfg)
        if self.need == 0:
            raise ValueError("invalid template configuration")
        if arena is not None and arena.numel() < self.need:
            raise ValueError("shared arena too small")
        self.arena = arena if arena is not None else torch.empty(self.need, dtype=torch.uint8, device="cuda:0")
        self.h = tb.tidal_template_create(shapes, self.arena, self.need, self.cfg)
        self.copy_stream = torch.cuda.Stream()
        self.compute_stream = torch.cuda.Stream()
        self.shapes = list(shapes)

    def slot_bytes(self, i: int) -> torch.Tensor:
        p, nb = tb.tidal_template_slot_ptr(self.h, i)
        o = p - self.arena.data_ptr()
        return self.arena[o:o + nb]

    def slot_host(self, i: int) -> np.ndarray:
        return self.slot_bytes(i).cpu().numpy().view(np.uint16).reshape(self.shapes[i])

    def sync(self):
        tb.tidal_template_sync(self.h)
        torch.cuda.synchronize()

    def close(self):
        if self.h:
            torch.cuda.synchronize()
            tb.tidal_template_destroy(self.h)
            self.h = None
