"""GPU parity tests of the unmerged adapter apply  y += (alpha/r) B bf16(A x)  on mixed batches:
requests with different resident adapters share one batch of token rows."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402
from tests.gpu_util import Template                       # noqa: E402


def f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bf16_bits(rng, shape, scale):
    return (rng.normal(0, scale, shape).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)


def dev(bits):
    return torch.from_numpy(bits.view(np.int16).copy()).to("cuda:0")


def host(t):
    return t.cpu().numpy().view(np.uint16)


def ulp(v):
    e = np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -126)))
    return 2.0 ** (e - 7)


def make_adapters(T, rng, slot, ranks, alphas, dtype=np.float32):
    out, inn = T.shapes[slot]
    items, handles = [], []
    for r, al in zip(ranks, alphas):
        A = rng.normal(0, 0.05, (r, inn)).astype(dtype)
        B = rng.normal(0, 0.05, (out, r)).astype(dtype)
        items.append((A, B, al))
        handles.append(T.upload_adapter([(slot, al, A, B)]))
    return items, handles


def run_apply(T, slot, handles, segs, X, Y, ws_extra=0):
    n = X.shape[0]
    xd, yd = dev(X), dev(Y)
    nb = tb.tidal_lora_apply_workspace_bytes(n)
    ws = torch.full((nb + ws_extra,), 0x7F, dtype=torch.uint8, device="cuda:0")
    tb.tidal_lora_apply(T.h, slot, handles, segs, xd, yd, n, ws, nb, T.compute_stream)
    T.sync()
    return host(yd).reshape(Y.shape)


ORDERED = tb.TIDAL_FLAG_ORDERED_ACCUM
MODES = pytest.mark.parametrize("flags", [ORDERED, 0], ids=["ordered", "fast"])


def check(orc, items, segs, X, Y, got, exact_bits=False):
    want = Y.copy()
    touched = np.zeros(X.shape[0], bool)
    bound = np.zeros(Y.shape)
    for a, t0, t1 in segs:
        if a < 0 or t1 == t0:
            continue
        A, B, al = items[a]
        Ab, Bb = orc.convert_to_bf16(A), orc.convert_to_bf16(B)
        orc.lora_apply(X, want, Ab, Bb, al, t0, t1)
        if A.shape[0] and al != 0.0:
            touched[t0:t1] = True
            u = f32(X[t0:t1]) @ f32(Ab).T                                   # (tokens, r)
            # u may land on the neighbouring bf16 (2^-8 relative) when the fp32 sums differ in order
            bound[t0:t1] = 2.0 ** -8 * (al / A.shape[0]) * (np.abs(u) @ np.abs(f32(Bb)).T)
    assert np.array_equal(got[~touched], Y[~touched])                       # other rows: bit-identical
    if exact_bits:                                                          # ordered accumulation: the oracle's own order
        assert np.array_equal(got, want), "%d elements differ" % int(np.sum(got != want))
        assert np.mean(got[touched] != Y[touched]) > 0.5
        return 1.0
    g, w = f32(got[touched]), f32(want[touched])
    err = np.abs(g - w)
    assert np.all(err <= ulp(np.maximum(np.abs(g), np.abs(w))) + bound[touched] + 1e-30), float(err.max())
    exact = np.mean(got[touched] == want[touched])
    assert exact > 0.99, exact                                              # nearly all elements agree bit for bit (measured >= 0.999)
    changed = np.mean(got[touched] != Y[touched])
    assert changed > 0.5, changed
    print("apply parity: %d rows, %.4f of elements bit-exact, max err %.3g" % (int(touched.sum()), exact, float(err.max())), flush=True)
    return exact


@MODES
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_mixed_batch_matches_oracle(orc, dtype, flags):
    rng = np.random.default_rng(11)
    shapes = [(64, 64), (384, 520)]                      # in: ragged last 64-column group; out: 1.5 strips
    with Template(shapes, flags=flags) as T:
        ranks = [4, 16, 24, 64, 33, 8]
        alphas = [8.0, 32.0, 48.0, 96.0, 66.0, 0.0]       # the last adapter is switched off by alpha
        items, handles = make_adapters(T, rng, 1, ranks, alphas, dtype)
        # tokens: 1 | 3 | gap 2 | 32 | 33 | 70 | empty | no-adapter 4 | alpha-0 5 | tail 7
        lens = [(0, 1), (1, 3), (-2, 2), (2, 32), (3, 33), (4, 70), (0, 0), (-1, 4), (5, 5), (1, 7)]
        segs, t = [], 0
        for a, n in lens:
            if a != -2:
                segs.append((a, t, t + n))
            t += n
        X = bf16_bits(rng, (t, 520), 1.0)
        Y = bf16_bits(rng, (t, 384), 1.0)
        got = run_apply(T, 1, handles, segs, X, Y)
        check(orc, items, segs, X, Y, got, bool(flags))
        # segments given in another order, same result
        got2 = run_apply(T, 1, handles, segs[::-1], X, Y)
        assert np.array_equal(got, got2)


def test_many_single_token_requests_span_several_launches(orc):
    rng = np.random.default_rng(12)
    with Template([(512, 256)]) as T:
        items, handles = make_adapters(T, rng, 0, [8, 16, 32, 64], [16.0, 32.0, 64.0, 128.0])
        n = 300                                          # more segments than one launch carries
        segs = [(i % 4, i, i + 1) for i in range(n)]
        X = bf16_bits(rng, (n, 256), 1.0)
        Y = bf16_bits(rng, (n, 512), 0.5)
        got = run_apply(T, 0, handles, segs, X, Y)
        check(orc, items, segs, X, Y, got)


@MODES
def test_segment_lengths_around_the_kernel_boundaries(orc, flags):
    """4 | 5 tokens: vector and matrix-core expand; 128 | 129: one and two chunks of four tiles;
    more than 80 longer segments: several launches of the matrix-core kernels."""
    rng = np.random.default_rng(15)
    with Template([(320, 192)], flags=flags) as T:
        items, handles = make_adapters(T, rng, 0, [16, 40, 1], [32.0, 80.0, 2.0])
        lens = [4, 5, 128, 129, 31, 32, 2, 8, 9] + [5] * 90
        segs, t = [], 0
        for i, n in enumerate(lens):
            segs.append((i % 3, t, t + n))
            t += n + (i % 2)                              # every other segment is followed by a free token
        X = bf16_bits(rng, (t, 192), 1.0)
        Y = bf16_bits(rng, (t, 320), 1.0)
        got = run_apply(T, 0, handles, segs, X, Y)
        check(orc, items, segs, X, Y, got, bool(flags))


def test_batch_of_more_than_256_tiles_takes_32_token_tiles(orc):
    """Prompt batches of 8192 tokens or more run one workgroup per 32 token rows (smaller ones per 16):
    three ranks, a ragged last tile per segment, 1.03 strips of outputs, a ragged last 64-column group."""
    rng = np.random.default_rng(16)
    with Template([(264, 200)]) as T:
        items, handles = make_adapters(T, rng, 0, [16, 64, 20], [32.0, 64.0, 40.0])
        lens = [4999, 2500, 777, 33]
        segs, t = [], 0
        for i, n in enumerate(lens):
            segs.append((i % 3, t, t + n))
            t += n + 1
        X = bf16_bits(rng, (t, 200), 1.0)
        Y = bf16_bits(rng, (t, 264), 1.0)
        got = run_apply(T, 0, handles, segs, X, Y)
        check(orc, items, segs, X, Y, got)


def test_long_prompt_one_adapter_and_merged_weights_untouched(orc):
    rng = np.random.default_rng(13)
    with Template([(256, 1024)]) as T:
        W = rng.normal(0, 0.02, (256, 1024)).astype(np.float32)
        T.materialize({0: W})
        items, handles = make_adapters(T, rng, 0, [16, 64], [32.0, 64.0])
        tb.tidal_lora_attach_adapter(T.h, handles[0], T.compute_stream)     # apply may run while merged
        T.sync()
        before = T.slot(0).copy()
        n = 300
        segs = [(1, 0, 200), (0, 200, 300)]
        X = bf16_bits(rng, (n, 1024), 1.0)
        Y = bf16_bits(rng, (n, 256), 2.0)
        got = run_apply(T, 0, handles, segs, X, Y)
        check(orc, items, segs, X, Y, got)
        assert np.array_equal(T.slot(0), before)
        tb.tidal_lora_detach(T.h, T.compute_stream)
        T.sync()


def test_apply_rejects_bad_arguments():
    rng = np.random.default_rng(14)
    with Template([(64, 64), (64, 64), (8, 12)]) as T:
        items, handles = make_adapters(T, rng, 0, [8], [16.0])
        X = dev(bf16_bits(rng, (8, 64), 1.0))
        Y = dev(bf16_bits(rng, (8, 64), 1.0))
        y0 = host(Y).copy()
        nb = tb.tidal_lora_apply_workspace_bytes(8)
        ws = torch.zeros(nb, dtype=torch.uint8, device="cuda:0")

        def bad(code, *a):
            with pytest.raises(tb.TidalError) as e:
                tb.tidal_lora_apply(*a)
            assert e.value.code == code

        bad(tb.TIDAL_E_INVAL, T.h, 0, handles, [(0, 0, 5), (0, 4, 8)], X, Y, 8, ws, nb)        # overlap
        bad(tb.TIDAL_E_INVAL, T.h, 0, handles, [(0, 0, 9)], X, Y, 8, ws, nb)                   # past the end
        bad(tb.TIDAL_E_INVAL, T.h, 0, handles, [(1, 0, 4)], X, Y, 8, ws, nb)                   # no such adapter
        bad(tb.TIDAL_E_INVAL, T.h, 1, handles, [(0, 0, 4)], X, Y, 8, ws, nb)                   # adapter lacks slot 1
        bad(tb.TIDAL_E_INVAL, T.h, 2, [], [(-1, 0, 4)], X, Y, 8, ws, nb)                       # 12 columns: not 8k
        bad(tb.TIDAL_E_NOMEM, T.h, 0, handles, [(0, 0, 4)], X, Y, 8, ws, nb - 1)               # workspace
        torch.cuda.synchronize()
        assert np.array_equal(host(Y), y0)                                                     # nothing ran


@MODES
@pytest.mark.parametrize("seed", [101, 102, 103])
def test_random_batches(orc, seed, flags):
    """Seeded random mixes of prompts and decode steps, ranks and gaps."""
    rng = np.random.default_rng(seed)
    out, inn = int(rng.choice([136, 264, 512])), int(rng.choice([72, 200, 448]))
    with Template([(out, inn)], flags=flags) as T:
        ranks = [int(r) for r in rng.choice([1, 2, 7, 8, 16, 17, 32, 48, 64], size=5)]
        items, handles = make_adapters(T, rng, 0, ranks, [2.0 * r for r in ranks])
        segs, t = [], 0
        for _ in range(int(rng.integers(20, 120))):
            n = int(rng.choice([1, 1, 1, 2, 3, 4, 5, 6, 31, 32, 33, 64, 100, 130]))
            if rng.random() < 0.15:
                t += int(rng.integers(1, 4))              # tokens without an adapter
            segs.append((int(rng.integers(-1, 5)), t, t + n))
            t += n
        order = rng.permutation(len(segs))
        X = bf16_bits(rng, (t, inn), 1.0)
        Y = bf16_bits(rng, (t, out), 1.0)
        got = run_apply(T, 0, handles, [segs[i] for i in order], X, Y)
        check(orc, items, segs, X, Y, got, bool(flags))


@MODES
def test_multi_target_call_equals_one_call_per_slot(orc, flags):
    """Query, key and value projections read the same x: one call for the three targets must give
    exactly what three calls give (and therefore what the oracle gives)."""
    rng = np.random.default_rng(16)
    shapes = [(320, 192), (136, 192), (136, 192), (64, 64)]
    with Template(shapes, flags=flags) as T:
        # the third adapter has another rank on every slot and none at all on the last one
        ranks, alphas = [(8, 8, 8), (64, 64, 64), (20, 64, 0)], [16.0, 128.0, 40.0]
        per_slot, handles = {0: [], 1: [], 2: []}, []
        for rs, al in zip(ranks, alphas):
            items = []
            for s in (0, 1, 2):
                r = rs[s]
                out, inn = shapes[s]
                A = rng.normal(0, 0.05, (r, inn)).astype(np.float32)
                B = rng.normal(0, 0.05, (out, r)).astype(np.float32)
                per_slot[s].append((A, B, al))
                items.append((s, al, A, B))
            handles.append(T.upload_adapter(items))
        lens = [(0, 1), (1, 40), (2, 3), (-1, 2), (0, 200), (1, 4), (2, 5)]
        segs, t = [], 0
        for a, n in lens:
            segs.append((a, t, t + n))
            t += n
        X = bf16_bits(rng, (t, 192), 1.0)
        Ys = [bf16_bits(rng, (t, shapes[s][0]), 1.0) for s in (0, 1, 2)]
        single = [run_apply(T, s, handles, segs, X, Ys[s]) for s in (0, 1, 2)]
        for s in (0, 1, 2):
            check(orc, per_slot[s], segs, X, Ys[s], single[s], bool(flags))
        xd = dev(X)
        yd = [dev(y) for y in Ys]
        nb = tb.tidal_lora_apply_workspace_bytes(3 * t)
        ws = torch.full((nb,), 0x7F, dtype=torch.uint8, device="cuda:0")
        tb.tidal_lora_apply_multi(T.h, [0, 1, 2], handles, segs, xd, yd, t, ws, nb, T.compute_stream)
        T.sync()
        for s in (0, 1, 2):
            assert np.array_equal(host(yd[s]).reshape(Ys[s].shape), single[s]), s
        # slots with different input widths cannot share a call; the workspace scales with the slots
        with pytest.raises(tb.TidalError) as e:
            tb.tidal_lora_apply_multi(T.h, [0, 3], handles, segs, xd, yd[:2], t, ws, nb, T.compute_stream)
        assert e.value.code == tb.TIDAL_E_INVAL
        with pytest.raises(tb.TidalError) as e:
            tb.tidal_lora_apply_multi(T.h, [0, 1, 2], handles, segs, xd, yd, t, ws,
                                      tb.tidal_lora_apply_workspace_bytes(2 * t), T.compute_stream)
        assert e.value.code == tb.TIDAL_E_NOMEM


def test_more_adapters_than_one_launch_carries(orc):
    """40 adapters on three slots are 120 (adapter, slot) pairs: the factor table of a decode launch
    holds 96, so the batch is cut where the table is full."""
    rng = np.random.default_rng(17)
    shapes = [(64, 64), (72, 64), (64, 64)]
    with Template(shapes) as T:
        per_slot, handles = {0: [], 1: [], 2: []}, []
        for a in range(40):
            r, al = 1 + a % 5, 2.0 + a
            items = []
            for s in (0, 1, 2):
                A = rng.normal(0, 0.2, (r, 64)).astype(np.float32)
                B = rng.normal(0, 0.2, (shapes[s][0], r)).astype(np.float32)
                per_slot[s].append((A, B, al))
                items.append((s, al, A, B))
            handles.append(T.upload_adapter(items))
        segs, t = [], 0
        for i in range(130):
            n = 1 + i % 3
            segs.append(((i * 7) % 40, t, t + n))
            t += n
        X = bf16_bits(rng, (t, 64), 1.0)
        Ys = [bf16_bits(rng, (t, shapes[s][0]), 1.0) for s in (0, 1, 2)]
        xd, yd = dev(X), [dev(y) for y in Ys]
        nb = tb.tidal_lora_apply_workspace_bytes(3 * t)
        ws = torch.zeros(nb, dtype=torch.uint8, device="cuda:0")
        tb.tidal_lora_apply_multi(T.h, [0, 1, 2], handles, segs, xd, yd, t, ws, nb, T.compute_stream)
        T.sync()
        for s in (0, 1, 2):
            check(orc, per_slot[s], segs, X, Ys[s], host(yd[s]).reshape(Ys[s].shape))
