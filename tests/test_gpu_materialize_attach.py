"""GPU parity of the cold start with the adapter folded into the load (tidal_materialize_attach):
targeted slots are written once as bf16(f32(src) + (alpha/r) B A), one rounding from the fp32 / fp16
source.  Bit-exact against the oracle with ordered accumulation, within the merge tolerance with
the matrix-core kernel; everything else must be a plain conversion, bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402
from tests.gpu_util import Template, pinned_like          # noqa: E402
from tests.test_gpu_lora import check_against_oracle, f32  # noqa: E402

ORDERED = tb.TIDAL_FLAG_ORDERED_ACCUM


def draw(rng, shape, dtype, scale):
    x = rng.normal(0, scale, shape).astype(np.float32)
    if dtype == "bf16":
        return (x.view(np.uint32) >> 16).astype(np.uint16)
    return x.astype(dtype)


def run_case(orc, flags, dtype, shapes, targets, chunk_bytes, seed, one_stream=False):
    """targets: {slot: (r, alpha)}"""
    rng = np.random.default_rng(seed)
    src = {i: draw(rng, s, dtype, 0.05) for i, s in enumerate(shapes)}
    ad = {}
    adt = np.float32 if dtype == "bf16" else dtype
    for s, (r, al) in targets.items():
        out, inn = shapes[s]
        ad[s] = (al, draw(rng, (r, inn), adt, 0.05), draw(rng, (out, r), adt, 0.05))
    with Template(shapes, chunk_bytes=chunk_bytes, flags=flags, max_adapter_bytes=1 << 20) as T:
        keep, srcs = [], []
        for i, a in src.items():
            k, v = pinned_like(a)
            keep.append(k)
            srcs.append((i, tb.dtype_code(v), tb.host_ptr(v)))
        items = [(s, al, A, B) for s, (al, A, B) in ad.items()]
        tg = T._targets(items)
        tb.tidal_materialize_attach(T.h, srcs, tg, T.compute_stream if one_stream else T.copy_stream, T.compute_stream)
        T.sync()
        exact = bool(flags & ORDERED)
        merged = {}
        for i in range(len(shapes)):
            got = T.slot(i)
            merged[i] = got
            if i in ad and ad[i][1].shape[0] > 0 and ad[i][0] != 0.0:
                al, A, B = ad[i]
                want = orc.materialize_merge(src[i], orc.convert_to_bf16(A), orc.convert_to_bf16(B), al)
                check_against_oracle(got, want, exact, "slot %d" % i)
                assert np.mean(got != orc.convert_to_bf16(src[i])) > 0.3          # the delta is in
            else:
                assert np.array_equal(got, orc.convert_to_bf16(src[i])), i
        # the adapter counts as attached: detach brings every slot back to (about) its plain conversion
        tb.tidal_lora_detach(T.h, T.compute_stream)
        T.sync()
        for i in ad:
            al, A, B = ad[i]
            got = T.slot(i)
            if A.shape[0] > 0 and al != 0.0:
                # the oracle's unmerge of what the GPU held after the fused load
                want = merged[i].copy()
                orc.lora_merge(want, orc.convert_to_bf16(A), orc.convert_to_bf16(B), al, -1)
                check_against_oracle(got, want, exact, "slot %d after detach" % i)
            else:
                assert np.array_equal(got, merged[i]), i
            base = orc.convert_to_bf16(src[i])
            g, b = f32(got).astype(np.float64), f32(base).astype(np.float64)
            assert np.max(np.abs(g - b)) <= 2.0 ** -6 * max(np.max(np.abs(b)), 1e-30), i
        return T.slot(0)


SHAPES = [(300, 200), (33, 130), (256, 520), (5, 7), (64, 96)]
TARGETS = {0: (8, 16.0), 1: (3, 6.0), 2: (64, 128.0), 3: (1, 2.0)}


@pytest.mark.parametrize("flags", [ORDERED, 0], ids=["ordered", "mfma"])
@pytest.mark.parametrize("dtype", [np.float32, np.float16, "bf16"], ids=["f32", "f16", "bf16"])
def test_fused_cold_start_matches_oracle(orc, flags, dtype):
    # 160 KiB chunks: the larger slots are cut into pieces that start and end inside rows
    run_case(orc, flags, dtype, SHAPES, TARGETS, 160 << 10, seed=31)


def test_fused_cold_start_one_chunk_and_ragged_widths(orc):
    # widths that are not multiples of 4 take the element-wise path; one big chunk holds everything
    shapes = [(40, 37), (17, 129), (64, 64)]
    run_case(orc, ORDERED, np.float16, shapes, {0: (5, 10.0), 1: (16, 32.0)}, 1 << 20, seed=32)
    run_case(orc, 0, np.float32, shapes, {0: (5, 10.0), 1: (16, 32.0), 2: (0, 4.0)}, 1 << 20, seed=33)
    # copies and kernels on one stream
    run_case(orc, ORDERED, np.float32, SHAPES, TARGETS, 160 << 10, seed=36, one_stream=True)


def test_one_rounding_beats_two(orc):
    """On fp32 sources the fused result is the correctly rounded sum more often than
    convert-then-attach, whose first rounding throws away the source's low bits."""
    rng = np.random.default_rng(34)
    shape = (96, 256)
    W = rng.normal(0, 0.05, shape).astype(np.float32)
    A = rng.normal(0, 0.05, (8, 256)).astype(np.float32)
    B = rng.normal(0, 0.05, (96, 8)).astype(np.float32)
    Ab, Bb = orc.convert_to_bf16(A), orc.convert_to_bf16(B)
    exact = W.astype(np.float64) + 2.0 * (f32(Bb).astype(np.float64) @ f32(Ab).astype(np.float64))
    errs = {}
    for mode in ("fused", "two_step"):
        with Template([shape], flags=ORDERED, max_adapter_bytes=1 << 20) as T:
            k, v = pinned_like(W)
            srcs = [(0, tb.dtype_code(v), tb.host_ptr(v))]
            tg = T._targets([(0, 16.0, A, B)])
            if mode == "fused":
                tb.tidal_materialize_attach(T.h, srcs, tg, T.copy_stream, T.compute_stream)
            else:
                tb.tidal_materialize(T.h, srcs, T.copy_stream, T.compute_stream)
                tb.tidal_lora_attach(T.h, tg, T.compute_stream)
            T.sync()
            errs[mode] = np.abs(f32(T.slot(0)).astype(np.float64) - exact)
            tb.tidal_lora_detach(T.h, T.compute_stream)
            T.sync()
    half_ulp = 2.0 ** (np.floor(np.log2(np.abs(exact))) - 8)
    assert np.all(errs["fused"] <= half_ulp * 1.001 + 1e-9)                # correctly rounded (up to the fp32 chain)
    assert np.mean(errs["two_step"] > half_ulp * 1.001 + 1e-9) > 0.05      # two roundings miss it regularly
    assert errs["fused"].mean() < errs["two_step"].mean()


def test_fused_cold_start_rejects_bad_calls():
    rng = np.random.default_rng(35)
    shapes = [(32, 64), (32, 64)]
    with Template(shapes, max_adapter_bytes=1 << 20) as T:
        W = [rng.normal(0, 0.05, s).astype(np.float32) for s in shapes]
        keep = [pinned_like(w) for w in W]
        srcs = [(i, tb.dtype_code(v), tb.host_ptr(v)) for i, (_, v) in enumerate(keep)]
        A = rng.normal(0, 0.05, (4, 64)).astype(np.float32)
        B = rng.normal(0, 0.05, (32, 4)).astype(np.float32)
        tg1 = T._targets([(1, 8.0, A, B)])
        with pytest.raises(tb.TidalError) as e:
            tb.tidal_materialize_attach(T.h, srcs[:1], tg1, T.copy_stream, T.compute_stream)   # target not loaded
        assert e.value.code == tb.TIDAL_E_INVAL
        tb.tidal_materialize_attach(T.h, srcs, tg1, T.copy_stream, T.compute_stream)
        T.sync()
        with pytest.raises(tb.TidalError) as e:
            tb.tidal_materialize_attach(T.h, srcs[:1], T._targets([(0, 8.0, A, B)]), T.copy_stream, T.compute_stream)
        assert e.value.code == tb.TIDAL_E_STATE                                                # slot 1 stays merged
        # re-materialising the merged slot with another adapter is a fresh cold start
        tb.tidal_materialize_attach(T.h, srcs, T._targets([(0, 8.0, A, B)]), T.copy_stream, T.compute_stream)
        T.sync()
        tb.tidal_lora_detach(T.h, T.compute_stream)
        T.sync()
