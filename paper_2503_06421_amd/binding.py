"""ctypes binding of libtidal.so: same names as the C ABI (include/tidal.h), argument
marshalling only.  Every step of the path runs in the library's HIP kernels; there is no
fallback of any kind: if the library is not built, or no GPU is present, calls raise.

PyTorch appears only as plumbing: `device_ptr` / `stream_ptr` accept torch tensors and streams,
and `lib()` imports torch (when installed) before loading the library so that both share one
HIP runtime.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, byref, c_char_p, c_double, c_float, c_int32, c_int64, c_size_t,
                    c_uint64, c_void_p)

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtidal.so")

TIDAL_F32, TIDAL_F16, TIDAL_BF16 = 0, 1, 2
TIDAL_OK, TIDAL_E_INVAL, TIDAL_E_NOMEM, TIDAL_E_STATE, TIDAL_E_HIP = 0, -1, -2, -3, -4
TIDAL_FLAG_ORDERED_ACCUM, TIDAL_FLAG_TWO_PASS_SWAP, TIDAL_FLAG_SLOT_EVENTS, TIDAL_FLAG_KERNEL_TIMING = 1, 2, 4, 8
TIDAL_FLAG_ASYNC_ENQUEUE = 16
TIDAL_FLAG_NO_COPY_MERGE = 32
TIDAL_FLAG_PIPELINED_UPLOAD = 64
TIDAL_FLAG_SERIAL_UPLOAD = 128

EXPORTS = [
    "tidal_config_default", "tidal_template_required_bytes", "tidal_template_create", "tidal_materialize",
    "tidal_materialize_plan", "tidal_materialize_attach", "tidal_lora_attach", "tidal_lora_swap", "tidal_lora_detach",
    "tidal_adapter_required_bytes", "tidal_adapter_upload", "tidal_adapter_destroy",
    "tidal_lora_attach_adapter", "tidal_lora_swap_adapter", "tidal_lora_apply_workspace_bytes", "tidal_lora_apply", "tidal_lora_apply_multi",
    "tidal_lora_apply_static", "tidal_lora_apply_static_max_tokens", "tidal_lora_launch_info", "tidal_lora_upload_plan",
    "tidal_fork_required_bytes", "tidal_fork_create",
    "tidal_fork_apply", "tidal_fork_slot_ptr", "tidal_fork_destroy", "tidal_template_slot_ptr",
    "tidal_template_slot_wait", "tidal_prefetch_bytes", "tidal_template_resident_prefix", "tidal_slot_checksum",
    "tidal_convert_device", "tidal_h2d_peak", "tidal_hbm_rmw_peak", "tidal_hbm_probe", "tidal_get_stats",
    "tidal_reset_stats", "tidal_template_sync", "tidal_template_destroy", "tidal_last_error",
]


class tidal_slot_desc(Structure):
    _fields_ = [("rows", c_int64), ("cols", c_int64)]


class tidal_src(Structure):
    _fields_ = [("slot", c_int32), ("dtype", c_int32), ("host", c_void_p)]


class tidal_lora_target(Structure):
    _fields_ = [("slot", c_int32), ("r", c_int32), ("alpha", c_float), ("dtype", c_int32),
                ("A", c_void_p), ("B", c_void_p)]


class tidal_lora_segment(Structure):
    _fields_ = [("adapter", c_int32), ("token_begin", c_int32), ("token_end", c_int32)]


class tidal_config(Structure):
    _fields_ = [("chunk_bytes", c_size_t), ("max_rank", c_int32), ("max_adapter_bytes", c_size_t),
                ("flags", c_int32), ("coalesce_bytes", c_size_t), ("gather_threads", c_int32),
                ("chunks_ahead", c_int32)]


class tidal_copy_piece(Structure):
    _fields_ = [("chunk", c_int32), ("slot", c_int32), ("elem_offset", c_int64), ("elems", c_int64),
                ("src_bytes", c_int64), ("staging_offset", c_int64), ("gathered", c_int32),
                ("reserved", c_int32)]


class tidal_lora_launch(Structure):
    _fields_ = [("kernel", ctypes.c_char * 64), ("launches", c_int32), ("targets_per_launch", c_int32),
                ("rank_padded_old", c_int32), ("rank_padded_new", c_int32), ("blocks_per_walk", c_int32),
                ("waves_per_simd", c_int32), ("workgroups", c_int64)]


class tidal_stats(Structure):
    _fields_ = [("h2d_bytes", c_uint64), ("h2d_copies", c_uint64), ("chunks", c_uint64),
                ("converted_elems", c_uint64), ("gathered_bytes", c_uint64), ("rmw_elems", c_uint64),
                ("lora_launches", c_uint64), ("lora_kernel_ms", c_double), ("convert_kernel_ms", c_double)]


class TidalError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("tidal error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Load libtidal.so.  Raises if it has not been built (python -m paper_2503_06421_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2503_06421_amd.build` "
            "(there is no fallback path)" % LIB_PATH)
    # One HIP runtime per process: the caller's device memory and streams come from PyTorch,
    # whose wheel bundles its own libamdhip64 under the same soname as the system one.  Loading
    # torch first makes libtidal bind to that copy; loading libtidal first would bring in a
    # second runtime that does not see torch's device state.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(LIB_PATH)
    vp = c_void_p
    L.tidal_config_default.argtypes = [POINTER(tidal_config)]
    L.tidal_template_required_bytes.restype = c_size_t
    L.tidal_template_required_bytes.argtypes = [POINTER(tidal_slot_desc), c_int32, POINTER(tidal_config)]
    L.tidal_template_create.argtypes = [POINTER(tidal_slot_desc), c_int32, vp, c_size_t, POINTER(tidal_config),
                                        POINTER(vp)]
    L.tidal_materialize.argtypes = [vp, POINTER(tidal_src), c_int32, vp, vp]
    L.tidal_materialize_attach.argtypes = [vp, POINTER(tidal_src), c_int32, POINTER(tidal_lora_target), c_int32, vp, vp]
    L.tidal_materialize_plan.restype = c_int32
    L.tidal_materialize_plan.argtypes = [vp, POINTER(tidal_src), c_int32, c_int32, POINTER(tidal_copy_piece), c_int32]
    for name in ("tidal_lora_attach", "tidal_lora_swap"):
        getattr(L, name).argtypes = [vp, POINTER(tidal_lora_target), c_int32, vp]
    L.tidal_lora_detach.argtypes = [vp, vp]
    L.tidal_lora_upload_plan.argtypes = [vp, POINTER(tidal_lora_target), c_int32, c_int32, POINTER(c_int32), c_int32]
    L.tidal_lora_upload_plan.restype = c_int32
    L.tidal_lora_launch_info.argtypes = [vp, c_int64, c_int64, c_int32, c_int32, c_int32, c_int32, POINTER(tidal_lora_launch)]
    L.tidal_adapter_required_bytes.restype = c_size_t
    L.tidal_adapter_required_bytes.argtypes = [vp, POINTER(tidal_lora_target), c_int32]
    L.tidal_adapter_upload.argtypes = [vp, POINTER(tidal_lora_target), c_int32, vp, c_size_t, vp, POINTER(vp)]
    L.tidal_adapter_destroy.argtypes = [vp]
    L.tidal_lora_attach_adapter.argtypes = [vp, vp, vp]
    L.tidal_lora_swap_adapter.argtypes = [vp, vp, vp]
    L.tidal_lora_apply_workspace_bytes.restype = c_size_t
    L.tidal_lora_apply_workspace_bytes.argtypes = [c_int32]
    L.tidal_lora_apply.argtypes = [vp, c_int32, POINTER(vp), c_int32, POINTER(tidal_lora_segment), c_int32, vp, vp,
                                   c_int32, vp, c_size_t, vp]
    L.tidal_lora_apply_multi.argtypes = [vp, POINTER(c_int32), c_int32, POINTER(vp), c_int32, POINTER(tidal_lora_segment),
                                         c_int32, vp, POINTER(vp), c_int32, vp, c_size_t, vp]
    L.tidal_lora_apply_static_max_tokens.restype = c_int32
    L.tidal_lora_apply_static_max_tokens.argtypes = []
    L.tidal_lora_apply_static.argtypes = [vp, c_int32, POINTER(vp), c_int32, POINTER(tidal_lora_segment), c_int32, vp, vp,
                                          c_int32, vp]
    L.tidal_fork_required_bytes.restype = c_size_t
    L.tidal_fork_required_bytes.argtypes = [vp, POINTER(c_int32), c_int32]
    L.tidal_fork_create.argtypes = [vp, POINTER(c_int32), c_int32, vp, c_size_t, POINTER(vp)]
    L.tidal_fork_apply.argtypes = [vp, vp, vp]
    L.tidal_fork_slot_ptr.argtypes = [vp, c_int32, POINTER(vp), POINTER(c_size_t)]
    L.tidal_fork_destroy.argtypes = [vp]
    L.tidal_template_slot_ptr.argtypes = [vp, c_int32, POINTER(vp), POINTER(c_size_t)]
    L.tidal_template_slot_wait.argtypes = [vp, c_int32, vp]
    L.tidal_prefetch_bytes.restype = c_size_t
    L.tidal_prefetch_bytes.argtypes = [c_size_t, c_double, c_double]
    L.tidal_template_resident_prefix.argtypes = [vp, c_size_t, POINTER(c_int32), POINTER(c_size_t)]
    L.tidal_slot_checksum.argtypes = [vp, c_int32, c_int32, vp, vp]
    L.tidal_convert_device.argtypes = [vp, vp, c_int32, c_int64, vp]
    L.tidal_h2d_peak.argtypes = [vp, c_size_t, c_int32, vp, POINTER(c_double)]
    L.tidal_hbm_rmw_peak.argtypes = [vp, c_int64, c_int64, c_int64, c_int32, c_int32, vp, POINTER(c_double)]
    L.tidal_hbm_probe.argtypes = [vp, c_int64, c_int64, c_int64, c_int32, c_int32, c_int32, vp, POINTER(c_double)]
    L.tidal_get_stats.argtypes = [vp, POINTER(tidal_stats)]
    L.tidal_reset_stats.argtypes = [vp]
    L.tidal_template_sync.argtypes = [vp]
    L.tidal_template_destroy.argtypes = [vp]
    L.tidal_last_error.restype = c_char_p
    L.tidal_last_error.argtypes = []
    _lib = L
    return L


def _check(rc: int) -> int:
    if rc < 0:
        raise TidalError(rc, lib().tidal_last_error().decode())
    return rc


def tidal_last_error() -> str:
    return lib().tidal_last_error().decode()


# ---- marshalling helpers ------------------------------------------------------------------

_NP_DTYPE_CODE = {np.dtype(np.float32): TIDAL_F32, np.dtype(np.float16): TIDAL_F16, np.dtype(np.uint16): TIDAL_BF16}


def dtype_code(arr) -> int:
    """float32 / float16 numpy arrays carry their dtype; uint16 arrays are bf16 bit patterns."""
    try:
        return _NP_DTYPE_CODE[np.dtype(arr.dtype)]
    except KeyError:
        raise TypeError("host tensors must be float32, float16 or uint16 (bf16 bits), got %s" % arr.dtype)


def host_ptr(arr) -> int:
    """Address of a C-contiguous numpy array, or of a CPU torch tensor (e.g. pinned)."""
    if isinstance(arr, np.ndarray):
        if not arr.flags.c_contiguous:
            raise ValueError("host tensor must be C-contiguous")
        return arr.ctypes.data
    if not arr.is_contiguous():
        raise ValueError("host tensor must be contiguous")
    return arr.data_ptr()


def device_ptr(x) -> int:
    """int passes through; a torch CUDA tensor gives its data_ptr()."""
    return x if isinstance(x, int) else x.data_ptr()


def stream_ptr(s) -> int:
    """None / 0 = null stream; int passes through; torch.cuda.Stream gives its hipStream_t."""
    if s is None:
        return 0
    return s if isinstance(s, int) else s.cuda_stream


def _slot_array(shapes):
    arr = (tidal_slot_desc * max(1, len(shapes)))()
    for i, (r, c) in enumerate(shapes):
        arr[i].rows, arr[i].cols = int(r), int(c)
    return arr


def _src_array(srcs):
    """srcs: iterable of (slot, dtype_code, host_address)."""
    srcs = list(srcs)
    arr = (tidal_src * max(1, len(srcs)))()
    for i, (slot, dt, ptr) in enumerate(srcs):
        arr[i].slot, arr[i].dtype, arr[i].host = int(slot), int(dt), ptr
    return arr, len(srcs)


def _target_array(targets):
    """targets: iterable of (slot, r, alpha, dtype_code, A_address, B_address)."""
    targets = list(targets)
    arr = (tidal_lora_target * max(1, len(targets)))()
    for i, (slot, r, alpha, dt, a, b) in enumerate(targets):
        arr[i].slot, arr[i].r, arr[i].alpha, arr[i].dtype = int(slot), int(r), float(alpha), int(dt)
        arr[i].A, arr[i].B = a, b
    return arr, len(targets)


def make_config(chunk_bytes=0, max_rank=0, max_adapter_bytes=0, flags=0, coalesce_bytes=0, gather_threads=0,
                chunks_ahead=0) -> tidal_config:
    return tidal_config(chunk_bytes, max_rank, max_adapter_bytes, flags, coalesce_bytes, gather_threads, chunks_ahead)


def sources_from_arrays(arrays: dict):
    """{slot: host array} -> [(slot, dtype, address)] in dict order (the load order)."""
    return [(slot, dtype_code(a), host_ptr(a)) for slot, a in arrays.items()]


def targets_from_arrays(items):
    """[(slot, alpha, A, B)] with A (r, in) and B (out, r) host arrays -> target tuples."""
    out = []
    for slot, alpha, A, B in items:
        r = int(A.shape[0])
        if r:
            out.append((slot, r, alpha, dtype_code(A), host_ptr(A), host_ptr(B)))
        else:
            out.append((slot, 0, alpha, TIDAL_F32, None, None))
    return out


# ---- the calls, one per C entry point --------------------------------------------------------

def tidal_config_default() -> tidal_config:
    c = tidal_config()
    _check(lib().tidal_config_default(byref(c)))
    return c


def tidal_template_required_bytes(shapes, cfg: tidal_config | None = None) -> int:
    arr = _slot_array(shapes)
    return lib().tidal_template_required_bytes(arr, len(shapes), byref(cfg) if cfg is not None else None)


def tidal_template_create(shapes, dev_arena, arena_bytes: int, cfg: tidal_config | None = None) -> int:
    arr = _slot_array(shapes)
    out = c_void_p()
    _check(lib().tidal_template_create(arr, len(shapes), device_ptr(dev_arena), arena_bytes,
                                       byref(cfg) if cfg is not None else None, byref(out)))
    return out.value


def tidal_materialize(t, srcs, copy_stream=None, compute_stream=None) -> None:
    arr, n = _src_array(srcs)
    _check(lib().tidal_materialize(t, arr, n, stream_ptr(copy_stream), stream_ptr(compute_stream)))


def tidal_materialize_attach(t, srcs, targets, copy_stream=None, compute_stream=None) -> None:
    arr, n = _src_array(srcs)
    tarr, tn = _target_array(targets)
    _check(lib().tidal_materialize_attach(t, arr, n, tarr, tn, stream_ptr(copy_stream), stream_ptr(compute_stream)))


def tidal_materialize_plan(t, srcs, assume_pinned: int = 1):
    arr, n = _src_array(srcs)
    need = _check(lib().tidal_materialize_plan(t, arr, n, assume_pinned, None, 0))
    out = (tidal_copy_piece * max(1, need))()
    got = _check(lib().tidal_materialize_plan(t, arr, n, assume_pinned, out, need))
    return [out[i] for i in range(got)]


def tidal_lora_attach(t, targets, stream=None) -> None:
    arr, n = _target_array(targets)
    _check(lib().tidal_lora_attach(t, arr, n, stream_ptr(stream)))


def tidal_lora_swap(t, targets, stream=None) -> None:
    arr, n = _target_array(targets)
    _check(lib().tidal_lora_swap(t, arr, n, stream_ptr(stream)))


def tidal_lora_detach(t, stream=None) -> None:
    _check(lib().tidal_lora_detach(t, stream_ptr(stream)))


def tidal_lora_launch_info(t, out: int, inn: int, n_targets: int, r_old: int, r_new: int, fork: bool = False) -> dict:
    info = tidal_lora_launch()
    _check(lib().tidal_lora_launch_info(t, out, inn, n_targets, r_old, r_new, int(fork), byref(info)))
    d = {k: getattr(info, k) for k, _ in tidal_lora_launch._fields_}
    d["kernel"] = d["kernel"].decode()
    return d


def tidal_lora_upload_plan(t, targets, swap: bool = False) -> list:
    """Targets per group, in order, as tidal_lora_attach / _swap would upload and merge them."""
    arr, n = _target_array(targets)
    out = (c_int32 * 64)()
    g = lib().tidal_lora_upload_plan(t, arr, n, int(swap), out, 64)
    if g < 0:
        _check(g)
    return [out[i] for i in range(min(g, 64))]


def tidal_adapter_required_bytes(t, targets) -> int:
    arr, n = _target_array(targets)
    return lib().tidal_adapter_required_bytes(t, arr, n)


def tidal_adapter_upload(t, targets, dev_mem, dev_bytes: int, stream=None) -> int:
    arr, n = _target_array(targets)
    out = c_void_p()
    _check(lib().tidal_adapter_upload(t, arr, n, device_ptr(dev_mem), dev_bytes, stream_ptr(stream), byref(out)))
    return out.value


def tidal_adapter_destroy(a) -> None:
    _check(lib().tidal_adapter_destroy(a))


def tidal_lora_attach_adapter(t, a, stream=None) -> None:
    _check(lib().tidal_lora_attach_adapter(t, a, stream_ptr(stream)))


def tidal_lora_swap_adapter(t, a, stream=None) -> None:
    _check(lib().tidal_lora_swap_adapter(t, a, stream_ptr(stream)))


def tidal_lora_apply_workspace_bytes(n_tokens: int) -> int:
    return lib().tidal_lora_apply_workspace_bytes(n_tokens)


def lora_apply_arrays(adapters, segments):
    """ctypes arrays for tidal_lora_apply, for callers that reuse one batch layout many times."""
    adapters = list(adapters)
    segments = list(segments)
    aarr = (c_void_p * max(1, len(adapters)))(*adapters)
    sarr = (tidal_lora_segment * max(1, len(segments)))(*[tidal_lora_segment(a, b, e) for a, b, e in segments])
    return (aarr, len(adapters)), (sarr, len(segments))


def tidal_lora_apply(t, slot: int, adapters, segments, x, y, n_tokens: int, workspace, workspace_bytes: int,
                     stream=None) -> None:
    """segments: iterable of (adapter index, token_begin, token_end); or pass the two values of
    lora_apply_arrays() as adapters and segments."""
    if not (isinstance(adapters, tuple) and isinstance(segments, tuple) and len(segments) == 2
            and isinstance(segments[0], ctypes.Array)):
        adapters, segments = lora_apply_arrays(adapters, segments)
    _check(lib().tidal_lora_apply(t, slot, adapters[0], adapters[1], segments[0], segments[1], device_ptr(x),
                                  device_ptr(y), n_tokens, device_ptr(workspace), workspace_bytes, stream_ptr(stream)))


def tidal_lora_apply_static_max_tokens() -> int:
    return lib().tidal_lora_apply_static_max_tokens()


def tidal_lora_apply_static(t, slot: int, adapters, segments, x, y, n_tokens: int, stream=None) -> None:
    """tidal_lora_apply without a workspace: the library's fixed scratch array is used."""
    if not (isinstance(adapters, tuple) and isinstance(segments, tuple) and len(segments) == 2
            and isinstance(segments[0], ctypes.Array)):
        adapters, segments = lora_apply_arrays(adapters, segments)
    _check(lib().tidal_lora_apply_static(t, slot, adapters[0], adapters[1], segments[0], segments[1], device_ptr(x),
                                         device_ptr(y), n_tokens, stream_ptr(stream)))


def tidal_lora_apply_multi(t, slots, adapters, segments, x, ys, n_tokens: int, workspace, workspace_bytes: int,
                           stream=None) -> None:
    """Several target slots reading the same x; ys: one output per slot."""
    if not (isinstance(adapters, tuple) and isinstance(segments, tuple) and len(segments) == 2
            and isinstance(segments[0], ctypes.Array)):
        adapters, segments = lora_apply_arrays(adapters, segments)
    slots = list(slots)
    sl = (c_int32 * max(1, len(slots)))(*slots)
    yarr = (c_void_p * max(1, len(slots)))(*[device_ptr(y) for y in ys])
    _check(lib().tidal_lora_apply_multi(t, sl, len(slots), adapters[0], adapters[1], segments[0], segments[1],
                                        device_ptr(x), yarr, n_tokens, device_ptr(workspace), workspace_bytes,
                                        stream_ptr(stream)))


def _slot_list(slots):
    slots = list(slots)
    arr = (c_int32 * max(1, len(slots)))(*slots)
    return arr, len(slots)


def tidal_fork_required_bytes(t, slots) -> int:
    arr, n = _slot_list(slots)
    return lib().tidal_fork_required_bytes(t, arr, n)


def tidal_fork_create(t, slots, dev_mem, dev_bytes: int) -> int:
    arr, n = _slot_list(slots)
    out = c_void_p()
    _check(lib().tidal_fork_create(t, arr, n, device_ptr(dev_mem), dev_bytes, byref(out)))
    return out.value


def tidal_fork_apply(f, a=None, stream=None) -> None:
    _check(lib().tidal_fork_apply(f, a, stream_ptr(stream)))


def tidal_fork_slot_ptr(f, slot: int):
    p, n = c_void_p(), c_size_t()
    _check(lib().tidal_fork_slot_ptr(f, slot, byref(p), byref(n)))
    return (p.value or 0), n.value


def tidal_fork_destroy(f) -> None:
    _check(lib().tidal_fork_destroy(f))


def tidal_template_slot_ptr(t, slot: int):
    p, n = c_void_p(), c_size_t()
    _check(lib().tidal_template_slot_ptr(t, slot, byref(p), byref(n)))
    return (p.value or 0), n.value


def tidal_template_slot_wait(t, slot: int, stream=None) -> None:
    _check(lib().tidal_template_slot_wait(t, slot, stream_ptr(stream)))


def tidal_prefetch_bytes(model_bytes: int, ttft_seconds: float, link_bytes_per_second: float) -> int:
    return lib().tidal_prefetch_bytes(model_bytes, ttft_seconds, link_bytes_per_second)


def tidal_template_resident_prefix(t, prefetch_bytes: int):
    n, b = c_int32(), c_size_t()
    _check(lib().tidal_template_resident_prefix(t, prefetch_bytes, byref(n), byref(b)))
    return n.value, b.value


def tidal_slot_checksum(t, slot: int, passes: int, stream, dev_sum) -> None:
    _check(lib().tidal_slot_checksum(t, slot, passes, stream_ptr(stream), device_ptr(dev_sum)))


def tidal_convert_device(dst, src, dtype: int, n: int, stream=None) -> None:
    _check(lib().tidal_convert_device(device_ptr(dst), device_ptr(src), dtype, n, stream_ptr(stream)))


def tidal_h2d_peak(dev, nbytes: int, reps: int = 5, stream=None) -> float:
    out = c_double()
    _check(lib().tidal_h2d_peak(device_ptr(dev), nbytes, reps, stream_ptr(stream), byref(out)))
    return out.value


TIDAL_PROBE_RMW, TIDAL_PROBE_READ, TIDAL_PROBE_WRITE = 0, 1, 2


def tidal_hbm_probe(dev, rows: int, cols: int, n: int, blocks_per_walk: int = 4, mode: int = TIDAL_PROBE_RMW, reps: int = 4,
                    stream=None) -> float:
    out = c_double(0.0)
    _check(lib().tidal_hbm_probe(device_ptr(dev), rows, cols, n, blocks_per_walk, mode, reps, stream_ptr(stream), byref(out)))
    return out.value


def tidal_hbm_rmw_peak(dev, rows: int, cols: int, n: int, blocks_per_walk: int = 4, reps: int = 4, stream=None) -> float:
    out = c_double()
    _check(lib().tidal_hbm_rmw_peak(device_ptr(dev), rows, cols, n, blocks_per_walk, reps, stream_ptr(stream), byref(out)))
    return out.value


def tidal_get_stats(t) -> dict:
    s = tidal_stats()
    _check(lib().tidal_get_stats(t, byref(s)))
    return {k: (int if ty is c_uint64 else float)(getattr(s, k)) for k, ty in tidal_stats._fields_}


def tidal_reset_stats(t) -> None:
    _check(lib().tidal_reset_stats(t))


def tidal_template_sync(t) -> None:
    _check(lib().tidal_template_sync(t))


def tidal_template_destroy(t) -> None:
    _check(lib().tidal_template_destroy(t))
