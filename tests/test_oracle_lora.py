"""Pins for the oracle's LoRA merge / unmerge / swap and slot placement (not GPU).

None of the expected values below comes from the oracle itself: they are float64 brute
force, closed forms, identities and bounds that the definition
W' = W + (alpha/r) * B * A  (fp32 accumulation, bf16 or fp32 storage) implies.
"""
import os

import numpy as np
import pytest

from paper_2503_06421_amd import workloads as wl_mod


def bf16_trunc(x):
    """A bf16-representable float32 near x (truncation: used only to *make inputs*)."""
    x = np.asarray(x, dtype=np.float32)
    return (x.view(np.uint32) & 0xFFFF0000).view(np.float32)


def to_bits(x):
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & 0xFFFF), "input is not bf16-representable"
    return (u >> 16).astype(np.uint16)


def from_bits(b):
    return (b.astype(np.uint32) << 16).view(np.float32)


def ulp_bf16(x):
    """Spacing of bfloat16 at |x| (normal range)."""
    x = np.abs(np.asarray(x, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(x, 2.0 ** -126)))
    return 2.0 ** (e - 7)


def make_case(rng, out, inn, r, wscale=0.02, ascale=0.01):
    W = bf16_trunc(rng.uniform(-wscale, wscale, (out, inn)))
    A = bf16_trunc(rng.normal(0, ascale, (r, inn)))
    B = bf16_trunc(rng.normal(0, ascale, (out, r)))
    return W, A, B


def brute_delta(A, B):
    """sum_k B[i,k] * A[k,j] in float64, written as the triple loop of the definition."""
    out, r = B.shape
    inn = A.shape[1]
    d = np.zeros((out, inn), dtype=np.float64)
    for i in range(out):
        for j in range(inn):
            acc = 0.0
            for k in range(r):
                acc += float(B[i, k]) * float(A[k, j])
            d[i, j] = acc
    return d


@pytest.mark.parametrize("out,inn,r,alpha", [(5, 7, 1, 2.0), (5, 7, 3, 5.0), (7, 5, 3, 5.0),
                                             (4, 9, 8, 16.0), (3, 3, 16, 7.0), (6, 11, 64, 128.0)])
@pytest.mark.parametrize("sign", [+1, -1])
def test_merge_matches_float64_brute_force(orc, out, inn, r, alpha, sign):
    rng = np.random.default_rng(100 * out + 10 * inn + r)
    # adapters large enough that the update moves W by many ulps
    W, A, B = make_case(rng, out, inn, r, wscale=0.5, ascale=0.5)
    Wb = to_bits(W)
    orc.lora_merge(Wb, to_bits(A), to_bits(B), alpha, sign)
    got = from_bits(Wb).astype(np.float64)
    d = brute_delta(A, B)
    ref = W.astype(np.float64) + sign * (alpha / r) * d
    # one rounding to bf16 (half an ulp) plus fp32 accumulation slack
    slack = (r + 2) * 2.0 ** -24 * (np.abs(W) + (alpha / r) * np.abs(B).astype(np.float64) @ np.abs(A).astype(np.float64))
    assert np.all(np.abs(got - ref) <= 0.5 * ulp_bf16(ref) * (1 + 2.0 ** -6) + slack)
    # and the update really happened: far from the un-merged W in most places
    assert np.mean(np.abs(got - W) > 4 * ulp_bf16(W)) > 0.5


def test_merge_distinguishes_operand_layout(orc):
    """A transposed A or B, or swapped roles, cannot pass: out, in and r are pairwise different
    and the expected value is the brute-force definition."""
    rng = np.random.default_rng(5)
    out, inn, r = 6, 10, 4
    W, A, B = make_case(rng, out, inn, r, wscale=0.5, ascale=0.5)
    Wb = to_bits(W)
    orc.lora_merge(Wb, to_bits(A), to_bits(B), 4.0, +1)
    got = from_bits(Wb).astype(np.float64)
    ref = W + 1.0 * brute_delta(A, B)
    assert np.max(np.abs(got - ref)) <= np.max(ulp_bf16(ref))
    # the same data read with B's rows and columns exchanged gives something else entirely
    B_wrong = np.ascontiguousarray(B.reshape(r, out).T)
    wrong = W + 1.0 * brute_delta(A, B_wrong)
    assert np.max(np.abs(got - wrong)) > 100 * np.max(ulp_bf16(ref))


def test_rank1_closed_form_exact(orc):
    """r = 1: W' = bf16( fl32( s*b_i*a_j + W ) ).  With s a power of two and operands of similar
    magnitude the float64 evaluation of s*b*a + w is exact, so float64 -> float32 is the single
    fp32 rounding of the fused multiply-add, and the nearest-even bf16 of that is the result."""
    from tests.test_oracle_convert import _nearest_even_bf16_by_value
    rng = np.random.default_rng(21)
    out, inn = 33, 65
    W = bf16_trunc(rng.uniform(0.25, 1.0, (out, inn)) * rng.choice([-1, 1], (out, inn)))
    a = bf16_trunc(rng.uniform(0.5, 1.0, (1, inn)))
    b = bf16_trunc(rng.uniform(0.5, 1.0, (out, 1)) * rng.choice([-1, 1], (out, 1)))
    for alpha, sign in [(2.0, +1), (0.5, -1)]:
        Wb = to_bits(W)
        orc.lora_merge(Wb, to_bits(a), to_bits(b), alpha, sign)
        exact = sign * alpha * (b.astype(np.float64) * a.astype(np.float64)) + W.astype(np.float64)
        f32 = exact.astype(np.float32)
        want = _nearest_even_bf16_by_value(f32.view(np.uint32).reshape(-1)).reshape(out, inn)
        assert np.array_equal(Wb.astype(np.uint32), want)


def test_accumulation_is_fp32_in_ascending_k(orc):
    """2^24 + 1 - 2^24 evaluated left to right in fp32 loses the 1 (2^24+1 ties to 2^24);
    right to left, or exactly, it is 1.  The definition fixes ascending k in fp32."""
    B = np.array([[4096.0, 1.0, -4096.0]], dtype=np.float32)
    A = np.array([[4096.0], [1.0], [4096.0]], dtype=np.float32)
    W = np.array([[0.5]], dtype=np.float32)
    Wb = to_bits(W)
    orc.lora_merge(Wb, to_bits(A), to_bits(B), 3.0, +1)           # s = 1
    assert from_bits(Wb)[0, 0] == 0.5
    Wb = to_bits(W)
    orc.lora_merge(Wb, to_bits(A[::-1].copy()), to_bits(B[:, ::-1].copy()), 3.0, +1)
    assert from_bits(Wb)[0, 0] == 1.5                              # -2^24 + 1 is exact, + 2^24 = 1


def test_scale_is_alpha_over_r(orc):
    rng = np.random.default_rng(8)
    W, A, B = make_case(rng, 4, 6, 4, wscale=0.5, ascale=0.5)
    Wf = W.copy()
    orc.lora_merge(Wf, to_bits(A), to_bits(B), 6.0, +1)           # fp32 storage, s = 1.5
    ref = W + 1.5 * brute_delta(A, B)
    assert np.allclose(Wf, ref, rtol=1e-6, atol=1e-7)
    assert not np.allclose(Wf, W + 6.0 * brute_delta(A, B), rtol=1e-3)


def test_zero_operands_and_identities(orc):
    rng = np.random.default_rng(9)
    W, A, B = make_case(rng, 9, 12, 8)
    Wb0 = to_bits(W)
    for A_, B_ in [(np.zeros_like(A), B), (A, np.zeros_like(B))]:
        Wb = Wb0.copy()
        orc.lora_merge(Wb, to_bits(A_), to_bits(B_), 16.0, +1)
        assert np.array_equal(from_bits(Wb), from_bits(Wb0))       # value-equal
    # alpha = 0 and r = 0: untouched bit for bit, even -0, inf and NaN payloads
    odd = Wb0.copy()
    odd[0, :4] = [0x8000, 0x7F80, 0x7FA1, 0xFF80]
    for alpha, r in [(0.0, 8), (16.0, 0)]:
        Wb = odd.copy()
        orc.lora_merge(Wb, to_bits(A[:r]), to_bits(B[:, :r]), alpha, +1)
        assert np.array_equal(Wb, odd)
    # the general loop with alpha = 0 on finite data gives equal values (-0 may become +0)
    Wb = Wb0.copy()
    orc.lora_merge(Wb, to_bits(A), to_bits(B), 0.0, +1, short_circuit=False)
    assert np.array_equal(from_bits(Wb), from_bits(Wb0))


@pytest.mark.parametrize("r,alpha", [(8, 16.0), (16, 32.0), (64, 128.0)])
def test_merge_then_unmerge_restores_within_bound(orc, r, alpha):
    """bf16 storage rounds twice, so restoration holds to 2^-7 of the magnitudes involved;
    fp32 storage restores to fp32 rounding."""
    rng = np.random.default_rng(r)
    W, A, B = make_case(rng, 64, 96, r)
    Ab, Bb = to_bits(A), to_bits(B)
    W0 = to_bits(W)
    W1 = W0.copy()
    orc.lora_merge(W1, Ab, Bb, alpha, +1)
    W2 = W1.copy()
    orc.lora_merge(W2, Ab, Bb, alpha, -1)
    w0, w1, w2 = (from_bits(x).astype(np.float64) for x in (W0, W1, W2))
    assert np.any(W1 != W0)
    assert np.all(np.abs(w2 - w0) <= 2.0 ** -7 * np.maximum(np.abs(w0), np.maximum(np.abs(w1), np.abs(w2))))
    assert np.max(np.abs(w2 - w0)) <= 2.0 ** -7 * max(np.max(np.abs(w0)), np.max(np.abs(w1)))
    assert np.mean(W2 == W0) > 0.5                                  # most elements come back exactly
    F0 = W.copy()
    F1 = F0.copy()
    orc.lora_merge(F1, Ab, Bb, alpha, +1)
    F2 = F1.copy()
    orc.lora_merge(F2, Ab, Bb, alpha, -1)
    assert np.all(np.abs(F2 - F0) <= 2.0 ** -23 * np.maximum(np.abs(F0), np.maximum(np.abs(F1), np.abs(F2))))


def test_swap_is_unmerge_then_merge(orc):
    rng = np.random.default_rng(31)
    W, A0, B0 = make_case(rng, 40, 56, 8)
    _, A1, B1 = make_case(rng, 40, 56, 32)
    Wb = to_bits(W)
    orc.lora_merge(Wb, to_bits(A0), to_bits(B0), 16.0, +1)
    two = Wb.copy()
    orc.lora_merge(two, to_bits(A0), to_bits(B0), 16.0, -1)
    orc.lora_merge(two, to_bits(A1), to_bits(B1), 64.0, +1)
    one = Wb.copy()
    orc.lora_swap(one, to_bits(A0), to_bits(B0), 16.0, to_bits(A1), to_bits(B1), 64.0)
    assert np.array_equal(one, two)
    # and it lands near W + delta_new (float64), within the two roundings
    ref = W.astype(np.float64) + 2.0 * (B1.astype(np.float64) @ A1.astype(np.float64))
    assert np.max(np.abs(from_bits(one) - ref)) <= 2.0 ** -7 * np.max(np.abs(ref))


def test_layout_closed_form_and_alignment(orc):
    shapes = [(3, 5), (1, 128), (7, 1), (128, 128), (1, 1)]
    off = orc.layout(shapes)
    want = [0]
    for r, c in shapes:
        want.append(-(-(want[-1] + 2 * r * c) // 256) * 256)
    assert list(off) == want
    assert all(o % 256 == 0 for o in off)
    for (r, c), a, b in zip(shapes, off[:-1], off[1:]):
        assert b - a >= 2 * r * c and b - a < 2 * r * c + 256


def test_materialize_places_every_slot(orc):
    w = wl_mod.tiny_stack(with_norms=True)
    srcs = {i: wl_mod.draw_tensor(w, i) for i in range(len(w.tensors))}
    arena, off = orc.materialize(w.shapes, srcs)
    for i, t in enumerate(w.tensors):
        got = orc.slot_view(arena, off, w.shapes, i)
        assert np.array_equal(got, orc.convert_to_bf16(srcs[i]))
        pad = arena[int(off[i]) + 2 * t.numel: int(off[i + 1])]
        assert not pad.any()


def test_13b_stack_matches_paper_footprint(orc):
    """The paper's model-size table prints 24.3G for the 13B Llama weights (fp16)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_model_sizes.txt")
    printed = None
    with open(path) as f:
        for line in f:
            parts = line.split("#")[0].split()
            if parts and parts[0] == "llama2_13b":
                printed = float(parts[1])
    w = wl_mod.llama2_13b()
    assert len(w.tensors) == 282 and len(w.lora_slots) == 280
    assert w.source_bytes == 26_030_899_200
    off = orc.layout(w.shapes)
    assert int(off[-1]) == w.source_bytes                          # every slot is a multiple of 256 B
    assert abs(w.source_bytes / 2 ** 30 - printed) <= 0.1


def test_workload_shapes():
    w2 = wl_mod.llama2_7b()
    assert len(w2.tensors) == 226 and len(w2.lora_slots) == 64
    assert w2.source_bytes == 13_476_298_752 and 4 * w2.lora_w_elements == 4_294_967_296
    w5 = wl_mod.llama3_70b()
    assert len(w5.tensors) == 562 and len(w5.lora_slots) == 560
    assert w5.source_bytes == 141_104_775_168 and 4 * w5.lora_w_elements == 273_804_165_120
    w3 = wl_mod.llama2_13b()
    assert 4 * w3.lora_w_elements == 50_751_078_400
    ch = wl_mod.adapter_churn()
    assert len(ch.base.lora_slots) == 128 and 4 * ch.base.lora_w_elements == 8_589_934_592
    assert len(ch.schedule) == 200 and set(ch.ranks) <= {8, 16, 32, 64}
    assert wl_mod.adapter_churn().schedule == ch.schedule          # seeded


def test_prefetch_rule_eq1(orc):
    """Eq. 1 of the paper's Sec. 5.2: M_prefetch = max(M_model - T_TTFT * B_PCIe, 0).  Worked by
    hand: a 24.3 GB model, 0.4 s of inference and a 32 GB/s link leave 24.3 - 12.8 = 11.5 GB to
    prefetch; a long inference hides everything."""
    assert orc.prefetch_bytes(24_300_000_000, 0.4, 32e9) == 11_500_000_000
    assert orc.prefetch_bytes(24_300_000_000, 1.0, 32e9) == 0
    assert orc.prefetch_bytes(24_300_000_000, 0.0, 32e9) == 24_300_000_000
    assert orc.prefetch_bytes(1000, 1e-9, 1e9) == 999
    assert orc.prefetch_bytes(1000, 0.5e-9, 1e9) == 1000          # 999.5 rounds up to a whole byte
    shapes = [(4, 8), (2, 2), (16, 16), (1, 1)]                   # 64, 8, 512, 2 bytes
    assert [orc.resident_prefix(shapes, b) for b in (0, 1, 64, 65, 72, 73, 584, 585, 10 ** 6)] == [0, 1, 1, 2, 2, 3, 3, 4, 4]


def test_slot_checksum_closed_form(orc):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    assert orc.slot_checksum(bits) == 65535 * 65536 // 2
    assert orc.slot_checksum(bits, 7) == 7 * (65535 * 65536 // 2)
    assert orc.slot_checksum(np.full(3, 0xFFFF, np.uint16), 2) == 6 * 0xFFFF
    big = np.full(1 << 20, 0xFFFF, np.uint16)
    assert orc.slot_checksum(big, 1 << 20) == ((1 << 20) * 0xFFFF * (1 << 20)) % (1 << 64)


# ---- materialise with the adapter folded in: one rounding from the host-precision source --------------

@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_materialize_merge_is_the_fp32_merge_rounded_once(orc, dtype):
    """Composition of two pinned pieces: the fp32-storage merge (float64 brute force above) and
    the RNE narrowing (exhaustive pins): slot == bf16(merge_f32(widen(src)))."""
    rng = np.random.default_rng(21)
    out, inn, r, alpha = 9, 14, 5, 10.0
    src = rng.normal(0, 0.5, (out, inn)).astype(dtype)
    A = bf16_trunc(rng.normal(0, 0.3, (r, inn)))
    B = bf16_trunc(rng.normal(0, 0.3, (out, r)))
    got = orc.materialize_merge(src, to_bits(A), to_bits(B), alpha)
    W = src.astype(np.float32)                       # fp16 -> fp32 is exact
    orc.lora_merge(W, to_bits(A), to_bits(B), alpha, +1)
    assert np.array_equal(got, orc.convert_to_bf16(W))
    # and against float64: a single rounding of the exact value, up to the fp32 chain's error
    exact = src.astype(np.float64) + (alpha / r) * (B.astype(np.float64) @ A.astype(np.float64))
    mag = np.abs(src.astype(np.float64)) + (alpha / r) * (np.abs(B).astype(np.float64) @ np.abs(A).astype(np.float64))
    assert np.all(np.abs(from_bits(got).astype(np.float64) - exact) <= 0.5 * ulp_bf16(exact) * 1.001 + 2e-6 * mag)


def test_materialize_merge_rounds_once_where_two_roundings_differ(orc):
    """src = 1 + 2^-9 + 2^-14 (fp32): converting first gives bf16(1.0 + ...) = 1.0 and loses the
    tail; adding delta = 2^-9 afterwards gives 1 + 2^-9, below half an ulp -> 1.0.  The single rounding sees
    1 + 2^-8 + 2^-14 and must round UP to 1 + 2^-7."""
    src = np.array([[1.0 + 2.0 ** -9 + 2.0 ** -14]], np.float32)
    A = to_bits(np.array([[2.0 ** -9]], np.float32))
    B = to_bits(np.array([[1.0]], np.float32))
    fused = orc.materialize_merge(src, A, B, 1.0)
    assert from_bits(fused)[0, 0] == np.float32(1.0 + 2.0 ** -7)
    two_step = orc.convert_to_bf16(src)
    orc.lora_merge(two_step, A, B, 1.0, +1)
    assert from_bits(two_step)[0, 0] == np.float32(1.0)
    # short circuits are plain conversions
    assert np.array_equal(orc.materialize_merge(src, A, B, 0.0), orc.convert_to_bf16(src))
    assert np.array_equal(orc.materialize_merge(src, A[:0], B[:, :0], 4.0), orc.convert_to_bf16(src))
    # bf16 source: identical to the in-place merge
    sb = to_bits(bf16_trunc(np.array([[0.75, -3.0]], np.float32)))
    A2 = to_bits(bf16_trunc(np.array([[0.5, 0.25]], np.float32)))
    B2 = to_bits(np.array([[1.5]], np.float32))
    w = sb.copy()
    orc.lora_merge(w, A2, B2, 2.0, +1)
    assert np.array_equal(orc.materialize_merge(sb, A2, B2, 2.0), w)
