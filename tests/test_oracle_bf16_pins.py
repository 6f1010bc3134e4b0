"""Pins for the bfloat16 rounding the reduced-precision mode is defined with (no GPU).

bfloat16 is the upper half of an FP32 bit pattern (1 sign, 8 exponent, 7 fraction bits); the mode
rounds operands to it (nearest, ties to even) and multiplies the rounded values exactly.  The rounding
is pinned by tabulated ties and their neighbours, by the library's own conversion, by idempotence,
monotonicity and the half-ulp bound; the split x = hi + lo by the exactness of x - hi and the size
of what is left; the reduced-precision layer by lattice inputs (unchanged by the rounding) and by its
distance from the full-precision layer.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_05753_amd import inputs


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def test_tabulated_values():
    e = 2.0 ** -8            # half of the spacing of bfloat16 numbers in [1, 2)
    cases = [
        (1.0, 1.0), (-1.0, -1.0), (0.0, 0.0), (0.5, 0.5), (3.0, 3.0), (1.0 + 2 * e, 1.0 + 2 * e),
        (1.0 + e, 1.0),                       # tie: 1 (even fraction) wins over 1 + 2^-7
        (1.0 + 3 * e, 1.0 + 4 * e),           # tie: 1 + 2^-6 (even) wins over 1 + 2^-7
        (1.0 + e + 2.0 ** -23, 1.0 + 2 * e),  # just above the tie
        (1.0 + e - 2.0 ** -23, 1.0),          # just below
        (-(1.0 + e), -1.0), (-(1.0 + 3 * e), -(1.0 + 4 * e)),
        (2.0 - 2.0 ** -23, 2.0),              # carries into the exponent
        (256.0 + 1.0, 256.0), (256.0 + 3.0, 256.0 + 4.0), (0.1, 0.10009765625),
    ]
    x = np.array([c[0] for c in cases], dtype=np.float32)
    want = np.array([c[1] for c in cases], dtype=np.float32)
    assert np.array_equal(oracle.round_bf16(x), want)
    # specials: signed zero and infinities pass, NaN stays NaN, the largest FP32 values round to infinity
    sp = np.array([-0.0, np.inf, -np.inf, np.nan, 3.4e38], dtype=np.float32)
    got = oracle.round_bf16(sp)
    assert np.signbit(got[0]) and got[0] == 0 and got[1] == np.inf and got[2] == -np.inf
    assert np.isnan(got[3]) and got[4] == np.inf


def test_low_half_is_cleared_and_rounding_is_idempotent():
    x = inputs.matrix(301, 64, 64, "R") * np.float32(37.0)
    r = oracle.round_bf16(x)
    assert np.all(bits(r) & 0xFFFF == 0)
    assert np.array_equal(oracle.round_bf16(r), r)


def test_matches_the_library_conversion():
    x = np.concatenate([inputs.matrix(302, 200, 50, "R").ravel() * np.float32(s) for s in (1e-30, 1e-3, 1.0, 1e5, 1e30)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.round_bf16(x), want)
    # every tie in a binade, both parities
    base = np.arange(0x3F80, 0x4000, dtype=np.uint32) << 16
    ties = (base | 0x8000).view(np.float32)
    want = torch.from_numpy(ties.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.round_bf16(ties), want)


def test_half_ulp_bound_and_monotonicity():
    x = np.sort(inputs.matrix(303, 1, 20000, "R")[0] * np.float32(5.0))
    r = oracle.round_bf16(x)
    assert np.all(np.abs(r.astype(np.float64) - x) <= 2.0 ** -8 * np.abs(x))
    assert np.all(np.diff(r) >= 0)
    # nearest: no other bfloat16 value is closer
    up = (bits(r) + 0x10000).view(np.float32).astype(np.float64)
    dn = (bits(r) - 0x10000).view(np.float32).astype(np.float64)
    d = np.abs(r.astype(np.float64) - x)
    assert np.all(d <= np.abs(up - x)) and np.all(d <= np.abs(dn - x))


def test_split_remainder():
    x = inputs.matrix(304, 100, 100, "R") * np.float32(3.0)
    hi, lo = oracle.split_bf16(x)
    # x - hi is exact in FP32: the same number in double
    assert np.array_equal((x - hi).astype(np.float64), x.astype(np.float64) - hi.astype(np.float64))
    rest = np.abs(x.astype(np.float64) - hi - lo)
    assert np.all(rest <= 2.0 ** -16 * np.abs(x))
    assert np.all(np.abs(lo) <= 2.0 ** -8 * np.abs(x))
    assert np.array_equal(oracle.round_bf16(hi), hi) and np.array_equal(oracle.round_bf16(lo), lo)


@pytest.mark.parametrize("terms", [1, 3])
def test_lattice_inputs_are_not_changed_by_the_mode(terms):
    X, W, b = inputs.layer_inputs(305, 12, 40, 14, "L", bias=True)
    assert np.array_equal(oracle.round_bf16(X), X) and np.array_equal(oracle.round_bf16(W), W)
    assert np.array_equal(oracle.linear_reduced(X, W, b, terms), oracle.linear(X, W, b))


def test_distance_from_the_full_precision_layer():
    M, K, N = 20, 300, 24
    X, W, b = inputs.layer_inputs(306, M, K, N, "R", bias=True)
    Y = oracle.linear(X, W, b)
    S = oracle.magnitude(X, W, b)
    e1 = np.abs(oracle.linear_reduced(X, W, b, 1) - Y) / S
    e3 = np.abs(oracle.linear_reduced(X, W, b, 3) - Y) / S
    assert e1.max() <= 2.0 ** -7 and e1.max() > 2.0 ** -14       # rounded operands: visibly coarser than FP32
    assert e3.max() <= 2.0 ** -15                                  # split operands: close to it
    assert e3.max() < e1.max() / 100
    # the magnitude variant bounds the value
    assert np.all(np.abs(oracle.linear_reduced(X, W, b, 3)) <= oracle.linear_reduced(X, W, b, 3, absolute=True))
    with pytest.raises(RuntimeError):
        oracle.linear_reduced(X, W, b, 2)


def test_split_products_by_hand():
    # one product, all three terms written out
    x, w = np.float32(1.2345678), np.float32(-0.87654321)
    xh, xl = oracle.split_bf16(np.array([x]))
    wh, wl = oracle.split_bf16(np.array([w]))
    want = float(xh[0]) * float(wh[0]) + float(xh[0]) * float(wl[0]) + float(xl[0]) * float(wh[0])
    got = oracle.linear_reduced(np.array([[x]]), np.array([[w]]), None, 3)[0, 0]
    assert abs(got - want) <= 1e-16
    assert abs(got - float(x) * float(w)) <= 2.0 ** -15 * abs(float(x) * float(w))
