"""ctypes loader for the CPU oracle (oracle/tidal_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; the product package never does.
All arithmetic lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tidal_oracle.c")
_LIB = os.path.join(_HERE, "libtidal_oracle.so")

F32, F16, BF16 = 0, 1, 2

GCC_FLAGS = ["-std=c99", "-O2", "-mfma", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (about a second)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *GCC_FLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, i32, f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_float
        vp = ctypes.c_void_p
        L.orc_f16_bits_to_f32_bits.restype = ctypes.c_uint32
        L.orc_f16_bits_to_f32_bits.argtypes = [ctypes.c_uint16]
        L.orc_f32_bits_to_bf16_bits.restype = ctypes.c_uint16
        L.orc_f32_bits_to_bf16_bits.argtypes = [ctypes.c_uint32]
        L.orc_convert_to_bf16.restype = None
        L.orc_convert_to_bf16.argtypes = [vp, ctypes.c_int, i64, vp]
        L.orc_layout.restype = i64
        L.orc_layout.argtypes = [vp, vp, i32, vp]
        L.orc_materialize_slot.restype = None
        L.orc_materialize_slot.argtypes = [vp, i64, vp, ctypes.c_int, i64, i64]
        L.orc_lora_merge_bf16.restype = None
        L.orc_lora_merge_bf16.argtypes = [vp, i64, i64, vp, vp, i32, f32, ctypes.c_int, ctypes.c_int]
        L.orc_lora_merge_f32.restype = None
        L.orc_lora_merge_f32.argtypes = [vp, i64, i64, vp, vp, i32, f32, ctypes.c_int, ctypes.c_int]
        L.orc_lora_swap_bf16.restype = None
        L.orc_lora_swap_bf16.argtypes = [vp, i64, i64, vp, vp, i32, f32, vp, vp, i32, f32]
        L.orc_prefetch_bytes.restype = ctypes.c_uint64
        L.orc_prefetch_bytes.argtypes = [ctypes.c_uint64, ctypes.c_double, ctypes.c_double]
        L.orc_resident_prefix.restype = i32
        L.orc_resident_prefix.argtypes = [vp, vp, i32, ctypes.c_uint64]
        L.orc_slot_checksum.restype = ctypes.c_uint64
        L.orc_slot_checksum.argtypes = [vp, i64, i32]
        L.orc_materialize_merge_slot.restype = None
        L.orc_materialize_merge_slot.argtypes = [vp, ctypes.c_int, i64, i64, vp, vp, i32, f32, vp]
        L.orc_lora_apply.restype = None
        L.orc_lora_apply.argtypes = [vp, vp, i64, i64, vp, vp, i32, f32, i64, i64]
        _lib = L
    return _lib


_NP_OF = {F32: np.float32, F16: np.float16, BF16: np.uint16}


def dtype_code(arr: np.ndarray) -> int:
    """fp32 / fp16 arrays carry their dtype; uint16 arrays are bf16 bit patterns."""
    if arr.dtype == np.float32:
        return F32
    if arr.dtype == np.float16:
        return F16
    if arr.dtype == np.uint16:
        return BF16
    raise TypeError("oracle accepts float32, float16 or uint16 (bf16 bits), got %s" % arr.dtype)


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def f16_bits_to_f32_bits(h: int) -> int:
    return lib().orc_f16_bits_to_f32_bits(h)


def f32_bits_to_bf16_bits(u: int) -> int:
    return lib().orc_f32_bits_to_bf16_bits(u)


def convert_to_bf16(src: np.ndarray) -> np.ndarray:
    """Element-wise narrowing to bf16 bit patterns (uint16), same shape."""
    src = np.ascontiguousarray(src)
    dst = np.empty(src.shape, dtype=np.uint16)
    lib().orc_convert_to_bf16(_ptr(src), dtype_code(src), src.size, _ptr(dst))
    return dst


def layout(shapes) -> np.ndarray:
    """Slot byte offsets (n+1 entries, last = total) for [(rows, cols), ...]."""
    n = len(shapes)
    rows = np.array([s[0] for s in shapes], dtype=np.int64)
    cols = np.array([s[1] for s in shapes], dtype=np.int64)
    off = np.zeros(n + 1, dtype=np.int64)
    lib().orc_layout(_ptr(rows), _ptr(cols), n, _ptr(off))
    return off


def materialize(shapes, sources) -> tuple[np.ndarray, np.ndarray]:
    """Build the whole slot area on the host: returns (arena bytes, offsets).

    ``sources`` maps slot index -> host array (fp32, fp16 or uint16 bf16 bits);
    slots without a source stay zero.
    """
    off = layout(shapes)
    arena = np.zeros(int(off[-1]), dtype=np.uint8)
    for slot, src in sources.items():
        src = np.ascontiguousarray(src)
        rows, cols = shapes[slot]
        assert src.size == rows * cols
        lib().orc_materialize_slot(_ptr(arena), int(off[slot]), _ptr(src), dtype_code(src), rows, cols)
    return arena, off


def slot_view(arena: np.ndarray, off: np.ndarray, shapes, slot: int) -> np.ndarray:
    rows, cols = shapes[slot]
    return arena[int(off[slot]): int(off[slot]) + 2 * rows * cols].view(np.uint16).reshape(rows, cols)


def _check_adapter(W, A, B, r):
    out, inn = W.shape
    assert A.dtype == np.uint16 and B.dtype == np.uint16
    assert A.shape == (r, inn), (A.shape, r, inn)
    assert B.shape == (out, r), (B.shape, out, r)
    assert A.flags.c_contiguous and B.flags.c_contiguous and W.flags.c_contiguous


def lora_merge(W: np.ndarray, A: np.ndarray, B: np.ndarray, alpha: float, sign: int = +1,
               short_circuit: bool = True) -> None:
    """In-place merge (sign=+1) / unmerge (sign=-1).  W: uint16 bf16 bits or float32 (out, in);
    A: (r, in), B: (out, r) as bf16 bit patterns."""
    r = A.shape[0]
    _check_adapter(W, A, B, r)
    out, inn = W.shape
    if W.dtype == np.uint16:
        fn = lib().orc_lora_merge_bf16
    elif W.dtype == np.float32:
        fn = lib().orc_lora_merge_f32
    else:
        raise TypeError(W.dtype)
    fn(_ptr(W), out, inn, _ptr(A), _ptr(B), r, float(alpha), int(sign), int(short_circuit))


def lora_swap(W: np.ndarray, A_old, B_old, alpha_old, A_new, B_new, alpha_new) -> None:
    assert W.dtype == np.uint16
    r0, r1 = A_old.shape[0], A_new.shape[0]
    _check_adapter(W, A_old, B_old, r0)
    _check_adapter(W, A_new, B_new, r1)
    out, inn = W.shape
    lib().orc_lora_swap_bf16(_ptr(W), out, inn, _ptr(A_old), _ptr(B_old), r0, float(alpha_old),
                             _ptr(A_new), _ptr(B_new), r1, float(alpha_new))


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32 values (a reinterpretation, no arithmetic)."""
    return (b.astype(np.uint32) << 16).view(np.float32)


def prefetch_bytes(model_bytes: int, ttft_seconds: float, link_bytes_per_second: float) -> int:
    return lib().orc_prefetch_bytes(model_bytes, ttft_seconds, link_bytes_per_second)


def resident_prefix(shapes, prefetch: int) -> int:
    rows = np.array([s[0] for s in shapes], dtype=np.int64)
    cols = np.array([s[1] for s in shapes], dtype=np.int64)
    return lib().orc_resident_prefix(_ptr(rows), _ptr(cols), len(shapes), prefetch)


def slot_checksum(bits: np.ndarray, passes: int = 1) -> int:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return lib().orc_slot_checksum(_ptr(bits), bits.size, passes)


def lora_apply(X: np.ndarray, Y: np.ndarray, A: np.ndarray, B: np.ndarray, alpha: float, t0: int, t1: int) -> None:
    """Y[t0:t1] += (alpha/r) * B (A x) for the tokens of one segment, in place.  All arrays are bf16
    bit patterns: X (T, in), Y (T, out), A (r, in), B (out, r)."""
    r = A.shape[0]
    assert r <= 64
    for a in (X, Y, A, B):
        assert a.dtype == np.uint16 and a.flags.c_contiguous
    assert A.shape == (r, X.shape[1]) and B.shape == (Y.shape[1], r) and X.shape[0] == Y.shape[0]
    assert 0 <= t0 <= t1 <= X.shape[0]
    lib().orc_lora_apply(_ptr(X), _ptr(Y), X.shape[1], Y.shape[1], _ptr(A), _ptr(B), r, float(alpha), t0, t1)


def materialize_merge(src: np.ndarray, A: np.ndarray, B: np.ndarray, alpha: float) -> np.ndarray:
    """bf16( f32(src) + (alpha/r) B A ) with one rounding; src (out, in) fp32 / fp16 / uint16 bf16 bits."""
    src = np.ascontiguousarray(src)
    r = A.shape[0]
    out, inn = src.shape
    assert A.dtype == np.uint16 and B.dtype == np.uint16 and A.shape == (r, inn) and B.shape == (out, r)
    assert A.flags.c_contiguous and B.flags.c_contiguous
    slot = np.empty((out, inn), np.uint16)
    lib().orc_materialize_merge_slot(_ptr(src), dtype_code(src), out, inn, _ptr(A), _ptr(B), r, float(alpha), _ptr(slot))
    return slot
