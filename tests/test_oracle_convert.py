"""Pins for the oracle's number-format conversions (not GPU).

The oracle narrows with an add-and-shift on the bit pattern; the pins below never
reuse that trick.  They check it against (1) hand-derived special cases stored under
tests/golden, (2) a value-based search for the nearest bfloat16 in float64 with ties
to even, and (3) library conversions (numpy's float16, torch's bfloat16).
"""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _table(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) >= 2:
                rows.append((int(line[0], 16), int(line[1], 16)))
    assert rows
    return rows


def test_golden_bf16_special_cases(orc):
    for u, want in _table("bf16_rounding_cases.txt"):
        assert orc.f32_bits_to_bf16_bits(u) == want, hex(u)


def test_golden_fp16_special_cases(orc):
    for h, want in _table("fp16_widening_cases.txt"):
        assert orc.f16_bits_to_f32_bits(h) == want, hex(h)


def _fp16_value(h: int) -> float:
    """Value of a binary16 pattern straight from the format definition, in Python floats."""
    s = -1.0 if h >> 15 else 1.0
    e = (h >> 10) & 0x1F
    f = h & 0x3FF
    if e == 0:
        return s * f * 2.0 ** -24
    return s * (1.0 + f / 1024.0) * 2.0 ** (e - 15)


def test_fp16_widening_exhaustive_by_value(orc):
    for h in range(1 << 16):
        u = orc.f16_bits_to_f32_bits(h)
        e = (h >> 10) & 0x1F
        if e == 0x1F:
            assert (u & 0x7F800000) == 0x7F800000 and (u >> 31) == (h >> 15)
            assert ((u & 0x007FFFFF) == 0) == ((h & 0x3FF) == 0)      # inf stays inf, NaN stays NaN
            continue
        got = float(np.array([u], dtype=np.uint32).view(np.float32)[0])
        assert got == _fp16_value(h), hex(h)
        assert (u >> 31) == (h >> 15)                                  # sign of zero too


def test_fp16_widening_exhaustive_vs_numpy(orc):
    h = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    want = h.view(np.float16).astype(np.float32).view(np.uint32)
    got = np.array([orc.f16_bits_to_f32_bits(int(x)) for x in h], dtype=np.uint32)
    nan = (h & 0x7C00 == 0x7C00) & (h & 0x03FF != 0)
    assert np.array_equal(got[~nan], want[~nan])
    # a library may quiet a signalling NaN while widening; class and sign must agree
    assert np.all(np.isnan(got[nan].view(np.float32)))
    assert np.array_equal(got[nan] >> 31, want[nan] >> 31)


def _nearest_even_bf16_by_value(u: np.ndarray) -> np.ndarray:
    """Independent definition: among the two bfloat16 neighbours of |x| choose the nearer one
    by comparing exact float64 distances, the even one on a tie; 2**128 stands in for the
    neighbour above the largest finite value, as IEEE rounding prescribes.  Finite inputs only."""
    sign = (u >> 16) & 0x8000
    m = u & 0x7FFFFFFF
    lo = m & 0xFFFF0000
    hi = lo + 0x10000

    def val(bits):
        v = bits.astype(np.uint32).view(np.float32).astype(np.float64)
        return np.where(bits >= 0x7F800000, 2.0 ** 128, v)

    x = val(m)
    d_lo = x - val(lo)
    d_hi = val(hi) - x
    lo_even = ((lo >> 16) & 1) == 0
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & ~lo_even)
    return (np.where(pick_hi, hi, lo) >> 16).astype(np.uint32) | sign


def _low_halves():
    rng = np.random.default_rng(7)
    fixed = [0, 1, 2, 0x7FFE, 0x7FFF, 0x8000, 0x8001, 0x8002, 0xFFFE, 0xFFFF, 0x4000, 0xC000]
    return np.unique(np.concatenate([np.array(fixed), rng.integers(0, 1 << 16, 244)])).astype(np.uint32)


def test_bf16_rounding_by_value_all_upper_halves(orc):
    """Every upper half (all signs, exponents, kept fractions) x 250-odd lower halves
    including both sides of the tie."""
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    for low in _low_halves():
        u = hi | low
        finite = (u & 0x7F800000) != 0x7F800000
        got = orc.convert_to_bf16(u.view(np.float32)).astype(np.uint32)
        want = _nearest_even_bf16_by_value(u[finite])
        assert np.array_equal(got[finite], want), hex(int(low))
        isnan = ~finite & ((u & 0x007FFFFF) != 0)
        assert np.array_equal(got[isnan], (u[isnan] >> 16) | 0x40)
        isinf = ~finite & ~isnan
        assert np.array_equal(got[isinf], u[isinf] >> 16)


def test_bf16_rounding_vs_torch_random_and_dense(orc):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11)
    u = np.concatenate([
        rng.integers(0, 1 << 32, 1 << 22, dtype=np.uint64).astype(np.uint32),
        np.arange(0x3F7F0000, 0x3F830000, dtype=np.uint32),       # dense sweep across 1.0
        np.arange(0x00000000, 0x00030000, dtype=np.uint32),       # subnormals
        np.arange(0x7F7E0000, 0x7F800001, dtype=np.uint32),       # up to overflow
    ])
    x = u.view(np.float32)
    got = orc.convert_to_bf16(x)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x7F) != 0)


def test_bf16_idempotent_and_monotone(orc):
    b = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    wide = (b.astype(np.uint32) << 16).view(np.float32)
    again = orc.convert_to_bf16(wide)
    nan = np.isnan(wide)
    assert np.array_equal(again[~nan], b[~nan])                      # bf16 values are fixed points
    x = np.sort(np.random.default_rng(3).normal(0, 1, 100000).astype(np.float32))
    y = orc.bf16_bits_to_f32(orc.convert_to_bf16(x))
    assert np.all(np.diff(y) >= 0)                                   # rounding is monotone
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)            # half an ulp of 8 significant bits


def test_convert_dispatch_fp16_and_bf16_passthrough(orc):
    h = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    got = orc.convert_to_bf16(h.view(np.float16))
    via = np.array([orc.f32_bits_to_bf16_bits(orc.f16_bits_to_f32_bits(int(x))) for x in h], dtype=np.uint16)
    assert np.array_equal(got, via)
    # fp16 has 10 fraction bits, bf16 keeps 7: normal fp16 values round on the low 3 bits
    assert orc.convert_to_bf16(np.array([0x3C04], np.uint16).view(np.float16))[0] == 0x3F80  # 1+4/1024 tie -> even
    assert orc.convert_to_bf16(np.array([0x3C0C], np.uint16).view(np.float16))[0] == 0x3F82  # 1+12/1024 tie -> even (up)
    assert orc.convert_to_bf16(np.array([0x3C05], np.uint16).view(np.float16))[0] == 0x3F81
    assert np.array_equal(orc.convert_to_bf16(h), h)                 # uint16 = bf16 bits: copied


def test_bf16_rounding_all_2_to_32_patterns_vs_torch(orc):
    """Every binary32 pattern against an independent library conversion (torch CPU), 2^26 at a
    time.  NaN inputs: the library may canonicalise the payload, so only NaN-ness is compared there
    (the payload rule is pinned by the golden table and the by-value test above)."""
    torch = pytest.importorskip("torch")
    n = 1 << 26
    base = np.arange(n, dtype=np.uint32)
    for hi in range(64):
        u = base + np.uint32(hi << 26)
        x = u.view(np.float32)
        got = orc.convert_to_bf16(x)
        want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        nan = (u & 0x7FFFFFFF) > 0x7F800000
        if nan.any():
            assert np.array_equal(got[~nan], want[~nan]), hi
            assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x007F) != 0)
            assert np.array_equal(got[nan], ((u[nan] >> 16) | 0x40).astype(np.uint16))
        else:
            assert np.array_equal(got, want), hi
