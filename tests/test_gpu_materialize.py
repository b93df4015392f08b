"""GPU parity, materialisation: conversion and slot placement must be bit-exact against the
CPU oracle.  Everything goes through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402
from paper_2503_06421_amd import workloads as wl_mod      # noqa: E402


@pytest.fixture(scope="module")
def G():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from tests import gpu_util
    return gpu_util


def _oracle_slots(orc, shapes, arrays):
    arena, off = orc.materialize(shapes, arrays)
    return arena, off


def _compare_all_slots(orc, T, shapes, arrays):
    arena, off = _oracle_slots(orc, shapes, arrays)
    for i in range(len(shapes)):
        want = orc.slot_view(arena, off, shapes, i)
        got = T.slot(i)
        assert np.array_equal(got, want), "slot %d differs" % i


@pytest.mark.parametrize("dtype", [wl_mod.F32, wl_mod.F16, wl_mod.BF16])
@pytest.mark.parametrize("pinned", [True, False])
def test_tiny_stack_bit_exact(orc, G, dtype, pinned):
    """Several chunks (64 KiB each), ragged tails, tiny norm vectors gathered by the CPU."""
    w = wl_mod.tiny_stack(host_dtype=dtype, with_norms=True, hidden=200, ffn=536, vocab=1003)
    arrays = {i: wl_mod.draw_tensor(w, i) for i in range(len(w.tensors))}
    with G.Template(w.shapes, chunk_bytes=64 << 10, coalesce_bytes=4096) as T:
        T.materialize(arrays, pinned=pinned)
        _compare_all_slots(orc, T, w.shapes, arrays)
        st = tb.tidal_get_stats(T.h)
        assert st["h2d_bytes"] == w.source_bytes
        if dtype != wl_mod.BF16:
            assert st["converted_elems"] == sum(t.numel for t in w.tensors)
            assert st["chunks"] >= w.source_bytes // (64 << 10)
        if pinned:
            assert 0 < st["gathered_bytes"] < w.source_bytes // 10       # only the norm vectors
        else:
            assert st["gathered_bytes"] == w.source_bytes


def test_load_order_is_the_order_given(orc, G):
    """Sources given in reverse still land in their own slots."""
    w = wl_mod.tiny_stack(host_dtype=wl_mod.F16)
    arrays = {i: wl_mod.draw_tensor(w, i) for i in reversed(range(len(w.tensors)))}
    with G.Template(w.shapes, chunk_bytes=128 << 10) as T:
        T.materialize(arrays)
        _compare_all_slots(orc, T, w.shapes, arrays)


def test_all_fp16_patterns(orc, G):
    h = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16).view(np.float16).reshape(256, 256)
    with G.Template([(256, 256)]) as T:
        T.materialize({0: h})
        assert np.array_equal(T.slot(0), orc.convert_to_bf16(h))


def test_fp32_every_upper_half_times_tie_neighbourhood(orc, G):
    lows = np.array([0, 1, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x1234, 0xC000], dtype=np.uint32)
    u = ((np.arange(1 << 16, dtype=np.uint32) << 16)[None, :] | lows[:, None]).reshape(8 * 256, 256)
    x = u.view(np.float32)
    with G.Template([x.shape]) as T:
        T.materialize({0: x})
        assert np.array_equal(T.slot(0), orc.convert_to_bf16(x))


def test_fp32_random_bit_patterns_multi_chunk(orc, G):
    rng = np.random.default_rng(5)
    u = rng.integers(0, 1 << 32, size=(1531, 1023), dtype=np.uint64).astype(np.uint32)
    x = u.view(np.float32)
    with G.Template([x.shape], chunk_bytes=1 << 20) as T:
        T.materialize({0: x})
        assert np.array_equal(T.slot(0), orc.convert_to_bf16(x))


@pytest.mark.parametrize("threads", [1, 3, 16])
def test_large_pageable_sources_split_among_gather_threads(orc, G, threads):
    """Pageable sources go through the pinned bounce buffer; pieces of 8 MiB or more are copied
    there by several host threads.  Odd sizes so that the parts are ragged."""
    rng = np.random.default_rng(6)
    a = rng.normal(0, 1, (2999, 3001)).astype(np.float32)                    # 36 MB, pageable
    b = rng.normal(0, 1, (1777, 4099)).astype(np.float16)                    # 14.6 MB
    with G.Template([a.shape, b.shape, (3, 5)], chunk_bytes=24 << 20, gather_threads=threads) as T:
        T.materialize({0: a, 1: b, 2: np.ones((3, 5), np.float32)}, pinned=False)
        assert np.array_equal(T.slot(0), orc.convert_to_bf16(a))
        assert np.array_equal(T.slot(1), orc.convert_to_bf16(b))
        assert tb.tidal_get_stats(T.h)["gathered_bytes"] == a.nbytes + b.nbytes + 60


def test_empty_and_degenerate(orc, G):
    shapes = [(0, 5), (1, 1), (3, 0), (1, 7)]
    arrays = {1: np.array([[1.5]], np.float32), 3: np.arange(7, dtype=np.float16).reshape(1, 7),
              0: np.zeros((0, 5), np.float32)}
    with G.Template(shapes) as T:
        tb.tidal_materialize(T.h, [], T.copy_stream, T.compute_stream)       # nothing to do
        T.materialize(arrays)
        assert np.array_equal(T.slot(1), orc.convert_to_bf16(arrays[1]))
        assert np.array_equal(T.slot(3), orc.convert_to_bf16(arrays[3]))


def test_single_linear_full_size(orc, G):
    """Configuration 1: 4096 x 4096 fp32 U[-0.02, 0.02] -> bf16."""
    w = wl_mod.single_linear()
    x = wl_mod.draw_tensor(w, 0)
    with G.Template(w.shapes) as T:
        T.materialize({0: x})
        assert np.array_equal(T.slot(0), orc.convert_to_bf16(x))
        assert tb.tidal_get_stats(T.h)["chunks"] == 1


def test_slot_events(orc, G):
    w = wl_mod.tiny_stack(host_dtype=wl_mod.F32)
    arrays = {i: wl_mod.draw_tensor(w, i) for i in range(len(w.tensors))}
    with G.Template(w.shapes, chunk_bytes=64 << 10, flags=tb.TIDAL_FLAG_SLOT_EVENTS) as T:
        with pytest.raises(tb.TidalError):
            tb.tidal_template_slot_wait(T.h, 0, None)
        T.materialize(arrays, sync=False)
        side = torch.cuda.Stream()
        for i in range(len(w.shapes)):
            tb.tidal_template_slot_wait(T.h, i, side)
        side.synchronize()
        # the side stream waited for every slot, so without any other sync the data is there
        arena, off = orc.materialize(w.shapes, arrays)
        for i in range(len(w.shapes)):
            assert np.array_equal(T.slot(i), orc.slot_view(arena, off, w.shapes, i))
        T.sync()


def test_convert_device_standalone(orc, G):
    rng = np.random.default_rng(2)
    for dt, n in [(np.float32, 100003), (np.float16, 65536 + 5), (np.float32, 7), (np.float16, 8)]:
        x = rng.normal(0, 1, n).astype(dt)
        src = torch.from_numpy(x.view(np.uint8).copy()).cuda()
        dst = torch.zeros(n, dtype=torch.int16, device="cuda")
        tb.tidal_convert_device(dst, src, tb.dtype_code(x), n, None)
        torch.cuda.synchronize()
        got = dst.cpu().numpy().view(np.uint16)
        assert np.array_equal(got, orc.convert_to_bf16(x))


def test_rematerialise_twice_and_stats(orc, G):
    w = wl_mod.tiny_stack(host_dtype=wl_mod.F16)
    a1 = {i: wl_mod.draw_tensor(w, i) for i in range(len(w.tensors))}
    with G.Template(w.shapes, chunk_bytes=64 << 10) as T:
        T.materialize(a1)
        a2 = {i: (a1[i] * np.float16(0.5)) for i in a1}
        T.materialize(a2)
        _compare_all_slots(orc, T, w.shapes, a2)


def test_fp32_all_2_to_32_patterns_device_resident(orc, G):
    """Every binary32 bit pattern through the convert kernel (device-resident source), against the
    oracle, 2^26 patterns at a time."""
    n = 1 << 26
    dst = torch.empty(n, dtype=torch.int16, device="cuda")
    base = torch.arange(n, dtype=torch.int64, device="cuda")
    for hi in range(64):
        src = (base + (hi << 26)).to(torch.int32) if hi < 32 else (base + (hi << 26) - (1 << 32)).to(torch.int32)
        tb.tidal_convert_device(dst, src, tb.TIDAL_F32, n, None)
        torch.cuda.synchronize()
        got = dst.cpu().numpy().view(np.uint16)
        u = (np.arange(n, dtype=np.uint64) + (hi << 26)).astype(np.uint32)
        want = orc.convert_to_bf16(u.view(np.float32))
        assert np.array_equal(got, want), "block %d" % hi


def test_one_stream_for_everything_and_null_stream(orc, G):
    """copy_stream == compute_stream, and the null stream, are legal."""
    w = wl_mod.tiny_stack(host_dtype=wl_mod.F16, with_norms=True)
    arrays = {i: wl_mod.draw_tensor(w, i) for i in range(len(w.tensors))}
    for use_null in (False, True):
        with G.Template(w.shapes, chunk_bytes=64 << 10) as T:
            s = None if use_null else T.compute_stream
            keep = [G.pinned_like(np.ascontiguousarray(a)) for a in arrays.values()]
            srcs = [(i, tb.dtype_code(v), tb.host_ptr(v)) for i, (_, v) in zip(arrays.keys(), keep)]
            tb.tidal_materialize(T.h, srcs, s, s)
            T.sync()
            _compare_all_slots(orc, T, w.shapes, arrays)


def test_lora_on_another_stream_waits_for_the_materialisation(orc, G):
    """attach issued on a third stream right after an asynchronous materialisation, no host sync in
    between: the library orders the two on the GPU."""
    rng = np.random.default_rng(3)
    shapes = [(512, 1024)] * 6
    arrays = {i: rng.normal(0, 0.02, shapes[i]).astype(np.float16) for i in range(6)}
    A = rng.normal(0, 0.05, (8, 1024)).astype(np.float16)
    B = rng.normal(0, 0.05, (512, 8)).astype(np.float16)
    with G.Template(shapes, chunk_bytes=64 << 10, max_adapter_bytes=1 << 20,
                    flags=tb.TIDAL_FLAG_ORDERED_ACCUM | tb.TIDAL_FLAG_ASYNC_ENQUEUE) as T:
        T.arena.fill_(0x77)
        keep = [G.pinned_like(a) for a in arrays.values()]
        srcs = [(i, tb.TIDAL_F16, tb.host_ptr(v)) for i, (_, v) in enumerate(keep)]
        other = torch.cuda.Stream()
        tb.tidal_materialize(T.h, srcs, T.copy_stream, T.compute_stream)
        tb.tidal_lora_attach(T.h, tb.targets_from_arrays([(i, 16.0, A, B) for i in range(6)]), other)
        other.synchronize()
        T.sync()
        merged = []
        for i in range(6):
            want = orc.convert_to_bf16(arrays[i])
            orc.lora_merge(want, orc.convert_to_bf16(A), orc.convert_to_bf16(B), 16.0, +1)
            assert np.array_equal(T.slot(i), want), i
            merged.append(want)
        # the other direction: a materialisation right behind a LoRA call on another stream
        tb.tidal_lora_detach(T.h, other)
        tb.tidal_materialize(T.h, srcs[:3], T.copy_stream, T.compute_stream)
        other.synchronize()
        T.sync()
        for i in range(6):
            if i < 3:
                want = orc.convert_to_bf16(arrays[i])
            else:
                want = merged[i].copy()
                orc.lora_merge(want, orc.convert_to_bf16(A), orc.convert_to_bf16(B), 16.0, -1)
            assert np.array_equal(T.slot(i), want), i


@pytest.mark.parametrize("ahead", [1, 3, 7, 4096])
def test_every_pacing_depth_gives_the_same_slots(orc, G, ahead):
    """A load of a few dozen chunks with the host two chunks ahead for all of it, for part of it, and
    enqueued in one burst: same bits as the oracle's conversion every time (twice in a row, so the
    second load's copies meet the first one's staging events)."""
    rng = np.random.default_rng(50 + ahead)
    shapes = [(96, 1024), (33, 517), (256, 1024), (1, 7), (128, 2048)]
    with G.Template(shapes, chunk_bytes=64 << 10, chunks_ahead=ahead) as T:
        for rep in range(2):
            arrays = {i: rng.normal(0, 1.0, s).astype(np.float32 if i % 2 else np.float16) for i, s in enumerate(shapes)}
            T.arena.fill_(0x5A)
            T.materialize(arrays, sync=False)
            T.sync()
            assert tb.tidal_get_stats(T.h)["chunks"] >= 20 * (rep + 1)
            _compare_all_slots(orc, T, shapes, arrays)


def test_a_load_within_the_burst_budget_returns_before_it_is_done(G):
    """1.5 GiB of pinned fp16 in 128 MiB chunks (12 chunks, default budget 160): the call only
    enqueues, so it is back long before the ~27 ms the link needs."""
    import time
    n = 3
    shapes = [(8192, 32768)] * n
    with G.Template(shapes) as T:
        keep = [torch.zeros(shapes[0], dtype=torch.float16).pin_memory() for _ in range(n)]
        srcs = [(i, tb.TIDAL_F16, k.data_ptr()) for i, k in enumerate(keep)]
        tb.tidal_materialize(T.h, srcs, T.copy_stream, T.compute_stream)      # first call: buffers, events
        T.sync()
        t0 = time.perf_counter()
        tb.tidal_materialize(T.h, srcs, T.copy_stream, T.compute_stream)
        t1 = time.perf_counter()
        T.sync()
        t2 = time.perf_counter()
        assert (t1 - t0) < 0.5 * (t2 - t0), "call %.2f ms of %.2f ms" % ((t1 - t0) * 1e3, (t2 - t0) * 1e3)
