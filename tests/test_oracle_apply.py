"""Pins for the oracle's unmerged adapter apply  Y += (alpha/r) * B (A x)  (not GPU)."""
import numpy as np
import pytest

from tests.test_oracle_lora import bf16_trunc, from_bits, to_bits, ulp_bf16


def case(rng, T, inn, out, r, xs=1.0, ws=0.05):
    X = bf16_trunc(rng.normal(0, xs, (T, inn)))
    Y = bf16_trunc(rng.normal(0, xs, (T, out)))
    A = bf16_trunc(rng.normal(0, ws, (r, inn)))
    B = bf16_trunc(rng.normal(0, ws, (out, r)))
    return X, Y, A, B


@pytest.mark.parametrize("T,inn,out,r,alpha", [(3, 7, 5, 1, 2.0), (4, 33, 9, 3, 5.0), (2, 64, 17, 16, 32.0), (5, 40, 6, 64, 96.0)])
def test_apply_matches_float64_brute_force(orc, T, inn, out, r, alpha):
    rng = np.random.default_rng(T * 100 + inn)
    X, Y, A, B = case(rng, T, inn, out, r, ws=0.3)
    Yb = to_bits(Y)
    orc.lora_apply(to_bits(X), Yb, to_bits(A), to_bits(B), alpha, 1, T)       # token 0 is not in the segment
    got = from_bits(Yb).astype(np.float64)
    s = alpha / r
    ref = Y.astype(np.float64).copy()
    u_all = np.zeros((T, r))
    for t in range(1, T):
        for k in range(r):
            u_all[t, k] = sum(float(A[k, j]) * float(X[t, j]) for j in range(inn))
        for i in range(out):
            ref[t, i] += s * sum(float(B[i, k]) * u_all[t, k] for k in range(r))
    assert np.array_equal(got[0], Y[0].astype(np.float64))                    # untouched
    # error budget: u is rounded to bf16 (2^-9 relative each), then one bf16 rounding of Y
    mag = s * (np.abs(B).astype(np.float64) @ np.abs(u_all[1:]).T).T
    bound = 0.5 * ulp_bf16(ref[1:]) * 1.02 + 2.0 ** -8 * mag + 1e-6 * (np.abs(ref[1:]) + mag)
    assert np.all(np.abs(got[1:] - ref[1:]) <= bound)
    assert np.mean(np.abs(got[1:] - Y[1:]) > 2 * ulp_bf16(Y[1:])) > 0.5        # it did something


def test_apply_agrees_with_merged_weights(orc):
    """(W + s B A) x  ==  W x + s B (A x) up to rounding: applying the adapter to activations must
    match running the merged weight, which ties this path to the merge oracle."""
    rng = np.random.default_rng(4)
    T, inn, out, r, alpha = 6, 48, 20, 8, 16.0
    X, _, A, B = case(rng, T, inn, out, r, ws=0.2)
    W = bf16_trunc(rng.normal(0, 0.2, (out, inn)))
    y_base = bf16_trunc(X.astype(np.float64) @ W.T.astype(np.float64))        # some base output, bf16
    Yb = to_bits(y_base)
    orc.lora_apply(to_bits(X), Yb, to_bits(A), to_bits(B), alpha, 0, T)
    unmerged = from_bits(Yb).astype(np.float64)
    Wm = W.copy()                                                             # merge in fp32 storage: no W rounding
    orc.lora_merge(Wm, to_bits(A), to_bits(B), alpha, +1)
    merged = X.astype(np.float64) @ Wm.T.astype(np.float64)
    scale = np.max(np.abs(merged))
    assert np.max(np.abs(unmerged - merged)) <= 2.0 ** -6 * scale             # a few bf16 roundings apart
    assert np.max(np.abs(y_base - merged)) > 2.0 ** -3 * scale                # and far from the base alone


def test_apply_identities_and_layout(orc):
    rng = np.random.default_rng(5)
    X, Y, A, B = case(rng, 4, 24, 10, 4, ws=0.3)
    Y0 = to_bits(Y)
    for A_, B_, alpha in [(np.zeros_like(A), B, 8.0), (A, np.zeros_like(B), 8.0)]:
        Yb = Y0.copy()
        orc.lora_apply(to_bits(X), Yb, to_bits(A_), to_bits(B_), alpha, 0, 4)
        assert np.array_equal(from_bits(Yb), from_bits(Y0))
    odd = Y0.copy()
    odd[0, :3] = [0x8000, 0x7F80, 0x7FA1]
    for alpha, rr in [(0.0, 4), (8.0, 0)]:
        Yb = odd.copy()
        orc.lora_apply(to_bits(X), Yb, to_bits(A[:rr]), to_bits(B[:, :rr]), alpha, 0, 4)
        assert np.array_equal(Yb, odd)                                        # bit-identical short circuit
    # empty segment
    Yb = Y0.copy()
    orc.lora_apply(to_bits(X), Yb, to_bits(A), to_bits(B), 8.0, 2, 2)
    assert np.array_equal(Yb, Y0)
    # rank-1, power-of-two scale: exact closed form  y + s * b_i * bf16(a . x)
    a = bf16_trunc(rng.uniform(0.5, 1, (1, 24)))
    b = bf16_trunc(rng.uniform(0.5, 1, (10, 1)))
    x = np.zeros((1, 24), np.float32)
    x[0, 3] = 0.75                                                            # a . x is a single exact product
    y = bf16_trunc(rng.uniform(0.25, 1, (1, 10)))
    Yb = to_bits(y)
    orc.lora_apply(to_bits(x), Yb, to_bits(a), to_bits(b), 2.0, 0, 1)
    from tests.test_oracle_convert import _nearest_even_bf16_by_value
    u = np.float32(a[0, 3] * np.float32(0.75))
    ub = from_bits(_nearest_even_bf16_by_value(np.array([u]).view(np.uint32)).astype(np.uint16))[0]
    exact = (y.astype(np.float64) + 2.0 * b[:, 0].astype(np.float64) * float(ub)).astype(np.float32)
    want = _nearest_even_bf16_by_value(exact.view(np.uint32).reshape(-1))
    assert np.array_equal(Yb.reshape(-1).astype(np.uint32), want)
