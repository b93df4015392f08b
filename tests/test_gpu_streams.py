"""Calls of one template on different streams: completion and ordering cover every stream used,
not only the one used last.

A resident adapter is uploaded on a side stream that is still busy with earlier work (so the upload
starts late) into memory pre-filled with NaN patterns; a swap, an unmerged apply or a fork apply on
another stream must wait for that upload, and tidal_template_sync must wait for it even when a later
call used a different stream.  Anything that ran ahead would read the NaN patterns (or, for the host
side, return while the caller's factors are still being read).
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402
from tests.gpu_util import Template                       # noqa: E402

OUT, INN = 1024, 1536


def f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def occupy(stream, n=60):
    """Tens of milliseconds of ordinary work on `stream` (a chain of fp32 matrix products)."""
    with torch.cuda.stream(stream):
        a = torch.ones((4096, 4096), device="cuda:0") * 1e-4
        b = a
        for _ in range(n):
            b = a @ b
    return b


def factors(seed, r):
    g = np.random.default_rng(seed)
    return g.normal(0, 0.02, (r, INN)).astype(np.float16), g.normal(0, 0.02, (OUT, r)).astype(np.float16)


def upload_late(T, items, stream):
    """Upload on `stream` behind the work already queued there; the device memory starts as NaN patterns."""
    tg = tb.targets_from_arrays(items)
    nb = tb.tidal_adapter_required_bytes(T.h, tg)
    mem = torch.full((nb,), 0xFF, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    keep = occupy(stream)
    a = tb.tidal_adapter_upload(T.h, tg, mem, nb, stream)
    T._adapters.append(a)
    return a, mem, keep


def check(got, want):
    g, w = f32(got), f32(want)
    assert np.all(np.isfinite(g)), "NaN patterns reached the result: a kernel ran ahead of the upload"
    assert np.max(np.abs(g - w)) <= 2.0 ** -7 * np.max(np.abs(w))
    assert np.mean(got != want) < 5e-3


def test_swap_on_another_stream_waits_for_the_upload(orc):
    assert torch.cuda.is_available()
    rng = np.random.default_rng(1)
    W = rng.normal(0, 0.02, (OUT, INN)).astype(np.float16)
    with Template([(OUT, INN)]) as T:
        T.materialize({0: W})
        A0, B0 = factors(2, 16)
        A1, B1 = factors(3, 64)
        y = T.upload_adapter([(0, 32.0, A0, B0)])
        T.attach_adapter(y)
        before = T.slot(0)
        side, serve = torch.cuda.Stream(), T.compute_stream
        x, mem, keep = upload_late(T, [(0, 128.0, A1, B1)], side)
        tb.tidal_lora_swap_adapter(T.h, x, serve)                 # enqueued at once, on another stream
        tb.tidal_template_sync(T.h)
        want = before.copy()
        orc.lora_swap(want, orc.convert_to_bf16(A0), orc.convert_to_bf16(B0), 32.0,
                      orc.convert_to_bf16(A1), orc.convert_to_bf16(B1), 128.0)
        check(T.slot(0), want)
        T.detach()


def test_sync_covers_every_stream_used(orc):
    assert torch.cuda.is_available()
    rng = np.random.default_rng(4)
    W = rng.normal(0, 0.02, (OUT, INN)).astype(np.float16)
    with Template([(OUT, INN)]) as T:
        T.materialize({0: W})
        A0, B0 = factors(5, 8)
        y = T.upload_adapter([(0, 16.0, A0, B0)])
        T.attach_adapter(y)
        side = torch.cuda.Stream()
        A1, B1 = factors(6, 32)
        x, mem, keep = upload_late(T, [(0, 64.0, A1, B1)], side)
        tb.tidal_lora_detach(T.h, T.compute_stream)              # the last call uses another stream than the upload
        tb.tidal_template_sync(T.h)                                # ... and the sync still waits for the upload
        raw = mem.cpu().numpy().view(np.uint16)                    # default stream: no implicit wait for `side`
        assert np.mean(raw == 0xFFFF) < 0.01, "tidal_template_sync returned before the upload on the side stream was done"
        # and what was packed are the converted factors: A (transposed, some order of 16-byte groups) comes first
        want = np.sort(orc.convert_to_bf16(A1).reshape(-1))
        assert np.array_equal(np.sort(raw[: INN * 32]), want)
        torch.cuda.synchronize()
        # an attach with it gives the oracle's merge
        before = T.slot(0)
        T.attach_adapter(x)
        merged = before.copy()
        orc.lora_merge(merged, orc.convert_to_bf16(A1), orc.convert_to_bf16(B1), 64.0, +1)
        check(T.slot(0), merged)
        T.detach()


def test_apply_and_fork_wait_for_the_upload(orc):
    assert torch.cuda.is_available()
    rng = np.random.default_rng(7)
    W = rng.normal(0, 0.02, (OUT, INN)).astype(np.float16)
    with Template([(OUT, INN)]) as T:
        T.materialize({0: W})
        base = T.slot(0)
        A1, B1 = factors(8, 16)
        n = 96
        X = (rng.normal(0, 1.0, (n, INN)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
        Y = (rng.normal(0, 1.0, (n, OUT)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
        xd = torch.from_numpy(X.view(np.int16)).to("cuda:0")
        yd = torch.from_numpy(Y.view(np.int16).copy()).to("cuda:0")
        nb = tb.tidal_lora_apply_workspace_bytes(n)
        ws = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
        need = tb.tidal_fork_required_bytes(T.h, [0])
        fmem = torch.zeros(need, dtype=torch.uint8, device="cuda:0")
        F = tb.tidal_fork_create(T.h, [0], fmem, need)
        side, s_apply, s_fork = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        try:
            x, mem, keep = upload_late(T, [(0, 32.0, A1, B1)], side)
            tb.tidal_lora_apply(T.h, 0, [x], [(0, 0, n)], xd, yd, n, ws, nb, s_apply)
            tb.tidal_fork_apply(F, x, s_fork)
            torch.cuda.synchronize()
            Ab, Bb = orc.convert_to_bf16(A1), orc.convert_to_bf16(B1)
            got = yd.cpu().numpy().view(np.uint16)
            want = Y.copy()
            orc.lora_apply(X, want, Ab, Bb, 32.0, 0, n)
            assert np.all(np.isfinite(f32(got))), "the apply ran ahead of the upload"
            assert np.mean(got == want) > 0.99
            p, nbytes = tb.tidal_fork_slot_ptr(F, 0)
            o = p - fmem.data_ptr()
            fgot = fmem[o:o + nbytes].cpu().numpy().view(np.uint16).reshape(OUT, INN)
            fwant = base.copy()
            orc.lora_merge(fwant, Ab, Bb, 32.0, +1)
            check(fgot, fwant)
            assert np.array_equal(T.slot(0), base)
        finally:
            tb.tidal_fork_destroy(F)


def test_two_threads_each_with_a_template_of_its_own(orc):
    """One thread at a time per template, but templates are independent: two host threads load,
    attach, swap and detach on their own templates at the same time (ordered accumulation: every
    state is compared with the oracle bit for bit)."""
    import threading
    assert torch.cuda.is_available()
    errors = []

    def worker(seed):
        try:
            rng = np.random.default_rng(seed)
            shapes = [(256, 384), (96, 520)]
            with Template(shapes, flags=tb.TIDAL_FLAG_ORDERED_ACCUM, max_adapter_bytes=1 << 20) as T:
                for rep in range(4):
                    Ws = {i: rng.normal(0, 0.02, sh).astype(np.float16) for i, sh in enumerate(shapes)}
                    T.materialize(Ws)
                    want = {i: orc.convert_to_bf16(w) for i, w in Ws.items()}
                    ads = []
                    for r in (8, 24):
                        ads.append([(i, 2.0 * r, rng.normal(0, 0.05, (r, sh[1])).astype(np.float16),
                                     rng.normal(0, 0.05, (sh[0], r)).astype(np.float16)) for i, sh in enumerate(shapes)])
                    T.attach(ads[0])
                    for i, al, A, B in ads[0]:
                        orc.lora_merge(want[i], orc.convert_to_bf16(A), orc.convert_to_bf16(B), al, +1)
                        assert np.array_equal(T.slot(i), want[i]), (seed, rep, "attach", i)
                    T.swap(ads[1])
                    for (i, al0, A0, B0), (_, al1, A1, B1) in zip(ads[0], ads[1]):
                        orc.lora_swap(want[i], orc.convert_to_bf16(A0), orc.convert_to_bf16(B0), al0,
                                      orc.convert_to_bf16(A1), orc.convert_to_bf16(B1), al1)
                        assert np.array_equal(T.slot(i), want[i]), (seed, rep, "swap", i)
                    T.detach()
                    for i, al, A, B in ads[1]:
                        orc.lora_merge(want[i], orc.convert_to_bf16(A), orc.convert_to_bf16(B), al, -1)
                        assert np.array_equal(T.slot(i), want[i]), (seed, rep, "detach", i)
        except Exception as exc:                                  # noqa: BLE001 -- reported by the main thread
            errors.append(repr(exc))

    threads = [threading.Thread(target=worker, args=(s,)) for s in (11, 12)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not any(th.is_alive() for th in threads), "a worker did not finish"
    assert not errors, errors
