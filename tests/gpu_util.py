"""Helpers for the GPU parity tests: device arena and streams come from torch (plumbing),
every operation goes through the C ABI binding."""
from __future__ import annotations

import numpy as np
import torch

from paper_2503_06421_amd import binding as tb

NP_OF_CODE = {tb.TIDAL_F32: np.float32, tb.TIDAL_F16: np.float16, tb.TIDAL_BF16: np.uint16}


def pinned_like(arr: np.ndarray):
    """A pinned host copy of `arr`: returns (torch tensor that owns it, numpy view)."""
    t = torch.empty(arr.size * arr.itemsize, dtype=torch.uint8, pin_memory=True)
    view = t.numpy().view(arr.dtype).reshape(arr.shape)
    view[...] = arr
    return t, view


def pinned_empty(shape, dtype):
    n = int(np.prod(shape)) * np.dtype(dtype).itemsize
    t = torch.empty(max(n, 1), dtype=torch.uint8, pin_memory=True)
    return t, t.numpy()[:n].view(dtype).reshape(shape)


class Template:
    """A template over a torch-allocated arena."""

    def __init__(self, shapes, **cfg):
        self.shapes = [tuple(s) for s in shapes]
        self.cfg = tb.make_config(**cfg)
        need = tb.tidal_template_required_bytes(self.shapes, self.cfg)
        assert need > 0
        self.arena = torch.zeros(need, dtype=torch.uint8, device="cuda:0")
        assert self.arena.data_ptr() % 256 == 0
        self.h = tb.tidal_template_create(self.shapes, self.arena, need, self.cfg)
        self.copy_stream = torch.cuda.Stream()
        self.compute_stream = torch.cuda.Stream()
        self._keep = []
        self._adapters = []

    def close(self):
        if self.h:
            for a in self._adapters:
                try:
                    tb.tidal_adapter_destroy(a)
                except tb.TidalError:
                    pass
            tb.tidal_template_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        torch.cuda.synchronize()
        self.close()

    # -- materialise ---------------------------------------------------------------------
    def materialize(self, arrays: dict, pinned: bool = True, sync: bool = True):
        """arrays: {slot: numpy array}; pinned=True stages them in pinned host memory first."""
        srcs = []
        for slot, a in arrays.items():
            a = np.ascontiguousarray(a)
            if pinned:
                keep, a = pinned_like(a)
                self._keep.append(keep)
            else:
                self._keep.append(a)
            srcs.append((slot, tb.dtype_code(a), tb.host_ptr(a)))
        tb.tidal_materialize(self.h, srcs, self.copy_stream, self.compute_stream)
        if sync:
            self.sync()

    def sync(self):
        tb.tidal_template_sync(self.h)
        torch.cuda.synchronize()
        self._keep.clear()

    def slot(self, i: int) -> np.ndarray:
        """Slot contents as bf16 bit patterns (uint16), shape (rows, cols)."""
        ptr, nbytes = tb.tidal_template_slot_ptr(self.h, i)
        off = ptr - self.arena.data_ptr()
        raw = self.arena[off: off + nbytes].cpu().numpy()
        return raw.view(np.uint16).reshape(self.shapes[i])

    def slot_area(self) -> np.ndarray:
        last = len(self.shapes) - 1
        ptr, nbytes = tb.tidal_template_slot_ptr(self.h, last)
        end = ptr - self.arena.data_ptr() + nbytes
        return self.arena[:end].cpu().numpy()

    # -- LoRA -----------------------------------------------------------------------------
    def _targets(self, items):
        items = [(s, al, np.ascontiguousarray(A), np.ascontiguousarray(B)) for s, al, A, B in items]
        self._keep.append(items)
        return tb.targets_from_arrays(items)

    def attach(self, items, sync=True):
        tb.tidal_lora_attach(self.h, self._targets(items), self.compute_stream)
        if sync:
            self.sync()

    def swap(self, items, sync=True):
        tb.tidal_lora_swap(self.h, self._targets(items), self.compute_stream)
        if sync:
            self.sync()

    def detach(self, sync=True):
        tb.tidal_lora_detach(self.h, self.compute_stream)
        if sync:
            self.sync()

    def upload_adapter(self, items):
        tg = self._targets(items)
        need = tb.tidal_adapter_required_bytes(self.h, tg)
        assert need > 0
        mem = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        a = tb.tidal_adapter_upload(self.h, tg, mem, need, self.compute_stream)
        self._adapters.append(a)
        self._keep_adapter_mem = getattr(self, "_keep_adapter_mem", []) + [mem]
        self.sync()
        return a

    def attach_adapter(self, a, sync=True):
        tb.tidal_lora_attach_adapter(self.h, a, self.compute_stream)
        if sync:
            self.sync()

    def swap_adapter(self, a, sync=True):
        tb.tidal_lora_swap_adapter(self.h, a, self.compute_stream)
        if sync:
            self.sync()
