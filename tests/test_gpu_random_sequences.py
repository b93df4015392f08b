"""GPU parity on seeded random sequences of calls: ragged stacks with mixed host dtypes, pinned and
pageable sources, small chunks (so tensors split and coalesce), then a run of attach / swap /
detach / re-materialise / materialise-with-adapter calls with adapters given by host pointers or
resident, ranks 0..64, mixed factor dtypes.  After every call every slot is compared with the CPU
oracle, which replays the same sequence: bit for bit with ordered accumulation; with the
matrix-core kernels the oracle restarts from the GPU's state before each call, so that one-ulp
differences (allowed by the merge tolerance) do not compound."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2503_06421_amd import binding as tb            # noqa: E402
from tests.gpu_util import Template, pinned_like          # noqa: E402
from tests.test_gpu_lora import TOL, check_against_oracle, f32      # noqa: E402

ORDERED = tb.TIDAL_FLAG_ORDERED_ACCUM
DTYPES = ["f32", "f16", "bf16"]


def draw(rng, shape, dtype, scale):
    x = rng.normal(0, scale, shape).astype(np.float32)
    if dtype == "bf16":
        return (x.view(np.uint32) >> 16).astype(np.uint16)
    return x.astype(np.float16 if dtype == "f16" else np.float32)


def random_adapter(rng, shapes, lora_slots):
    """{slot: (alpha, A, B)} on a random non-empty subset of lora_slots; ranks 0..64, alpha sometimes 0."""
    k = int(rng.integers(1, len(lora_slots) + 1))
    chosen = sorted(rng.choice(lora_slots, size=k, replace=False).tolist())
    dt = DTYPES[int(rng.integers(0, 3))]
    ad = {}
    for s in chosen:
        out, inn = shapes[s]
        r = int(rng.choice([0, 1, 3, 8, 16, 17, 32, 40, 64]))
        alpha = 0.0 if rng.random() < 0.1 else float(rng.choice([1.0, 2.0 * max(r, 1), 7.5]))
        ad[s] = (alpha, draw(rng, (r, inn), dt, 0.05), draw(rng, (out, r), dt, 0.05))
    return ad


OTHER = tb.TIDAL_FLAG_TWO_PASS_SWAP | tb.TIDAL_FLAG_NO_COPY_MERGE | tb.TIDAL_FLAG_SLOT_EVENTS | tb.TIDAL_FLAG_ASYNC_ENQUEUE
CASES = [(ORDERED, s) for s in range(11, 23)] + [(0, s) for s in range(11, 23)] + \
        [(ORDERED | OTHER, s) for s in range(31, 35)] + [(OTHER, s) for s in range(31, 35)]


@pytest.mark.parametrize("flags,seed", CASES, ids=["%s-%d" % ("ordered" if f & ORDERED else "mfma", s) +
                                                   ("-otherflags" if f & OTHER else "") for f, s in CASES])
def test_random_call_sequences(orc, flags, seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(5, 10))
    shapes = []
    for _ in range(n):
        kind = rng.random()
        if kind < 0.15:
            shapes.append((1, int(rng.integers(1, 600))))                       # a vector
        elif kind < 0.25:
            shapes.append((int(rng.integers(0, 3)), int(rng.integers(0, 3))))   # tiny or empty
        else:
            shapes.append((int(rng.integers(1, 300)), int(rng.integers(1, 700))))
    src_dtype = [DTYPES[int(rng.integers(0, 3))] for _ in range(n)]
    src = [draw(rng, shapes[i], src_dtype[i], 0.05) for i in range(n)]
    pinned = [bool(rng.random() < 0.6) for _ in range(n)]
    lora_slots = [i for i, s in enumerate(shapes) if s[0] * s[1] > 0]
    chunk = int(rng.choice([192 << 10, 256 << 10, 1 << 20]))        # a factor (<= 179 KB here) must fit a chunk
    exact = bool(flags & ORDERED)

    with Template(shapes, chunk_bytes=chunk, flags=flags, max_adapter_bytes=4 << 20,
                  coalesce_bytes=int(rng.choice([0, 512, 4096]))) as T:
        keep = []

        def sources(slots):
            out = []
            for i in slots:
                a = np.ascontiguousarray(src[i])
                if pinned[i]:
                    k, a = pinned_like(a)
                    keep.append(k)
                else:
                    keep.append(a)
                out.append((i, tb.dtype_code(a), tb.host_ptr(a)))
            return out

        def items(ad):
            return [(s, al, A, B) for s, (al, A, B) in ad.items()]

        def bf(ad):
            return {s: (al, orc.convert_to_bf16(A), orc.convert_to_bf16(B)) for s, (al, A, B) in ad.items()}

        def gpu_state():
            return [T.slot(i).copy() for i in range(n)]

        def compare(state, what, mid=None):
            """mid: {slot: oracle value between the unmerge and the merge of a swap}.  With the matrix-core
            kernels that intermediate may land on the neighbouring bf16, and the difference then
            travels into the result at the intermediate's magnitude, not the result's (the old and the
            new delta may cancel): still within 2^-7 * max|W| per tensor, the stated tolerance, but
            more than one ulp of a small element."""
            for i in range(n):
                if shapes[i][0] * shapes[i][1] == 0:
                    continue
                tag = "seed %d, %s, slot %d %s" % (seed, what, i, shapes[i])
                if exact:
                    check_against_oracle(T.slot(i), state[i], True, tag)
                    continue
                got = T.slot(i)
                g, w = f32(got).astype(np.float64), f32(state[i]).astype(np.float64)
                m = np.abs(f32(mid[i]).astype(np.float64)) if mid and i in mid else 0.0
                assert np.max(np.abs(g - w)) <= TOL * np.max(np.abs(w)), tag                       # the stated tolerance
                assert np.sum(got != state[i]) <= max(3, 4e-3 * got.size), tag                     # nearly all identical
                assert np.all(np.abs(g - w) <= 2.0 ** -7 * np.maximum(np.abs(w), m) + 2.0 ** -20 * np.max(np.abs(w))), tag

        tb.tidal_materialize(T.h, sources(range(n)), T.copy_stream, T.compute_stream)
        T.sync()
        state = [orc.convert_to_bf16(src[i]) for i in range(n)]
        for i in range(n):
            assert np.array_equal(T.slot(i), state[i]), "materialise: slot %d" % i

        attached = None            # the adapter merged into the template ({slot: (alpha, A_bf16, B_bf16)})
        for step in range(10):
            if not exact:
                state = gpu_state()
            ops = ["detach", "swap", "swap_resident", "rematerialise"] if attached is not None else \
                  ["attach", "attach_resident", "materialize_attach"]
            op = ops[int(rng.integers(0, len(ops)))]
            what = "step %d %s" % (step, op)
            if op in ("attach", "attach_resident", "swap", "swap_resident"):
                ad = random_adapter(rng, shapes, lora_slots)
                new = bf(ad)
                mid = {}
                for s in sorted(set(new) | set(attached or {})):
                    old_s = (attached or {}).get(s)
                    new_s = new.get(s)
                    if old_s is not None:
                        orc.lora_merge(state[s], old_s[1], old_s[2], old_s[0], -1)
                        if new_s is not None:
                            mid[s] = state[s].copy()
                    if new_s is not None:
                        orc.lora_merge(state[s], new_s[1], new_s[2], new_s[0], +1)
                if op == "attach":
                    T.attach(items(ad))
                elif op == "swap":
                    T.swap(items(ad))
                else:
                    h = T.upload_adapter(items(ad))
                    (T.attach_adapter if op == "attach_resident" else T.swap_adapter)(h)
                attached = new
            elif op == "detach":
                for s, (al, A, B) in attached.items():
                    orc.lora_merge(state[s], A, B, al, -1)
                T.detach()
                attached = None
            elif op == "rematerialise":
                # every slot the adapter is merged into comes back from its source: nothing attached afterwards
                tb.tidal_materialize(T.h, sources(sorted(attached)), T.copy_stream, T.compute_stream)
                T.sync()
                for s in attached:
                    state[s] = orc.convert_to_bf16(src[s])
                attached = None
            else:                  # materialize_attach: the adapter folded into the load of its slots
                ad = random_adapter(rng, shapes, lora_slots)
                new = bf(ad)
                tb.tidal_materialize_attach(T.h, sources(sorted(ad)), T._targets(items(ad)), T.copy_stream,
                                            T.compute_stream)
                T.sync()
                for s, (al, A, B) in new.items():
                    if A.shape[0] > 0 and al != 0.0:
                        state[s] = orc.materialize_merge(src[s], A, B, al)
                    else:
                        state[s] = orc.convert_to_bf16(src[s])
                attached = new
            compare(state, what, mid if op in ("swap", "swap_resident") else None)
            keep.clear()
