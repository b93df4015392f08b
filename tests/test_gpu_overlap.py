"""GPU tests of event-gated consumption (Sec. 5.2: data must be on the GPU before the kernel that
reads it runs; loading overlaps with inference; part of the template may be resident already).

The stand-in consumer adds up a slot's bf16 bit patterns as integers, so its result is exact and is
compared with the oracle's sum.  The arena is poisoned first: a consumer that ran before its slot
arrived would add up poison and fail."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402
from paper_2503_06421_amd import harness as hz            # noqa: E402
from paper_2503_06421_amd import workloads as wl_mod      # noqa: E402


def expected_sums(orc, wl, views, passes):
    return [orc.slot_checksum(orc.convert_to_bf16(v), passes) for v in views]


@pytest.mark.parametrize("order", ["access", "reverse"])
@pytest.mark.parametrize("resident_fraction", [0.0, 0.4])
def test_consumer_waits_for_each_slot(orc, order, resident_fraction):
    wl = wl_mod.tiny_stack(host_dtype=wl_mod.F16, layers=3, hidden=256, ffn=688, vocab=2000, with_norms=True)
    pool = hz.HostPool(wl)
    T = hz.DeviceTemplate(wl.shapes, chunk_bytes=128 << 10, flags=tb.TIDAL_FLAG_SLOT_EVENTS)
    try:
        T.arena.fill_(0xA5)                                           # poison
        n = len(wl.shapes)
        srcs = pool.sources()
        n_res, res_bytes = tb.tidal_template_resident_prefix(T.h, int(resident_fraction * wl.source_bytes))
        if n_res:
            tb.tidal_materialize(T.h, srcs[:n_res], T.copy_stream, T.compute_stream)
            T.sync()
        rest = srcs[n_res:]
        if order == "reverse":
            rest = rest[::-1]
        sums = torch.zeros(n, dtype=torch.int64, device="cuda:0")
        consumer = torch.cuda.Stream()
        passes = 3
        # nothing is synchronised between the load and the consumer except the per-slot events
        with pytest.raises(tb.TidalError):
            tb.tidal_slot_checksum(T.h, n - 1, passes, consumer, sums[n - 1:])   # not materialised yet
        tb.tidal_materialize(T.h, rest, T.copy_stream, T.compute_stream)
        for i in range(n):
            tb.tidal_slot_checksum(T.h, i, passes, consumer, sums[i:])
        consumer.synchronize()
        got = [int(x) & 0xFFFFFFFFFFFFFFFF for x in sums.cpu().numpy()]
        assert got == expected_sums(orc, wl, pool.views, passes)
        T.sync()
    finally:
        T.close()


def test_checksum_ragged_and_argument_checks(orc):
    shapes = [(1, 5), (3, 7), (33, 129), (0, 4)]
    rng = np.random.default_rng(0)
    arrays = [rng.normal(0, 1, s).astype(np.float32) for s in shapes]
    T = hz.DeviceTemplate(shapes)
    try:
        keep = [torch.from_numpy(a).pin_memory() for a in arrays]
        tb.tidal_materialize(T.h, [(i, tb.TIDAL_F32, k.data_ptr()) for i, k in enumerate(keep)], T.copy_stream, T.compute_stream)
        T.sync()
        sums = torch.zeros(4, dtype=torch.int64, device="cuda:0")
        for i in range(4):
            tb.tidal_slot_checksum(T.h, i, 2, T.compute_stream, sums[i:])
        T.sync()
        got = [int(x) & 0xFFFFFFFFFFFFFFFF for x in sums.cpu().numpy()]
        assert got == [orc.slot_checksum(orc.convert_to_bf16(a), 2) for a in arrays]
        for bad in [lambda: tb.tidal_slot_checksum(T.h, 9, 1, None, sums), lambda: tb.tidal_slot_checksum(T.h, 0, 0, None, sums)]:
            with pytest.raises(tb.TidalError):
                bad()
    finally:
        T.close()
