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


# ---------------------------------------------------------------------------------------------
# the mixing MLP and the channel-mixing block in mixed precision
# ---------------------------------------------------------------------------------------------
def small_int_mlp(seed, M, C, Hd):
    """Operands for which every step of the MLP is exact: X in {0, 1, 2}, W1 in {0, 1}, b1 = 10 (so that the
    pre-activation is an integer in [10, 10 + 2 C], where gelu(x) = x Phi(x) rounds to x in double), W2 in
    {-1, 0, 1}, b2 small integers."""
    rng = np.random.default_rng(seed)
    X = rng.integers(0, 3, (M, C)).astype(np.float32)
    W1 = rng.integers(0, 2, (Hd, C)).astype(np.float32)
    b1 = np.full(Hd, 10.0, dtype=np.float32)
    W2 = rng.integers(-1, 2, (C, Hd)).astype(np.float32)
    b2 = rng.integers(-3, 4, C).astype(np.float32)
    return X, W1, b1, W2, b2


@pytest.mark.parametrize("terms", [1, 3])
def test_mixed_mlp_in_closed_form(terms):
    M, C, Hd = 5, 8, 6
    X, W1, b1, W2, b2 = small_int_mlp(320, M, C, Hd)
    Xi, W1i, W2i = X.astype(np.int64), W1.astype(np.int64), W2.astype(np.int64)
    H = Xi @ W1i.T + 10                       # integers up to 26: exact in bfloat16, and gelu leaves them alone
    Y = Xi + H @ W2i.T + b2.astype(np.int64)
    r = oracle.mlp_reduced(X, W1, b1, W2, b2, terms)
    assert np.array_equal(r["H"], H.astype(np.float64))
    assert np.array_equal(r["Y"], Y.astype(np.float64))
    assert np.array_equal(oracle.mlp_reduced(X, W1, b1, W2, b2, terms, residual=False)["Y"], (Y - Xi).astype(np.float64))
    # a transposed W2 or a dropped bias would give another matrix
    assert not np.array_equal(Y, Xi + H @ W2i[:, ::-1].T + b2.astype(np.int64))
    # magnitudes: sums of absolute values
    assert np.array_equal(r["S1"], (Xi @ W1i.T + 10).astype(np.float64))
    assert np.array_equal(r["SY"], (np.abs(Xi) + H @ np.abs(W2i).T + np.abs(b2.astype(np.int64))).astype(np.float64))


@pytest.mark.parametrize("terms", [1, 3])
def test_mixed_mlp_is_the_pinned_pieces_in_sequence(terms):
    M, C, Hd = 6, 16, 24
    X, W1, b1 = inputs.layer_inputs(321, M, C, Hd, "R")
    W2 = inputs.matrix(322, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(323, 1, C, "R")[0]
    r = oracle.mlp_reduced(X, W1, b1, W2, b2, terms)
    H = oracle.gelu(oracle.linear_reduced(X, W1, b1, terms))
    assert np.array_equal(r["H"], H)
    Y = X.astype(np.float64) + oracle.linear_reduced(H.astype(np.float32), W2, b2, terms)
    assert np.array_equal(r["Y"], Y)
    # H is rounded again where the second product reads it: with the unrounded H the result differs, by no more
    # than the rounding allows (2^-8 of |H| |W2| for one term, 2^-16 for the split)
    full = oracle.mlp(X, W1, b1, W2, b2)
    assert not np.array_equal(r["Y"], full["Y"])
    loose = (2.0 ** -7 if terms == 1 else 2.0 ** -14) * (full["SY"] + full["PY"])
    assert np.all(np.abs(r["Y"] - full["Y"]) <= loose)
    if terms == 3:      # and the split is far closer to full precision than the single rounding
        one = oracle.mlp_reduced(X, W1, b1, W2, b2, 1)
        assert np.abs(r["Y"] - full["Y"]).max() < 0.02 * np.abs(one["Y"] - full["Y"]).max()


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_mixed_block_norms_first_and_skips_in_full_precision(ways):
    M, C, Hd = 6, 16, 24
    X, W1, b1 = inputs.layer_inputs(324, M, C, Hd, "R")
    X = (X + np.float32(0.3)).astype(np.float32)
    W2 = inputs.matrix(325, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(326, 1, C, "R")[0]
    gamma = (inputs.matrix(327, 1, C, "R")[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(328, 1, C, "R")[0]
    r = oracle.mixing_block_reduced(ways, X, gamma, beta, W1, b1, W2, b2, 1)
    Xn = oracle.layernorm(X, gamma, beta, oracle.ln_groups(ways))
    assert np.array_equal(r["Xn"], Xn)
    inner = oracle.mlp_reduced(Xn.astype(np.float32), W1, b1, W2, b2, 1, residual=False)
    assert np.array_equal(r["H"], inner["H"])
    assert np.array_equal(r["Y"], inner["Y"] + X.astype(np.float64))          # X itself, not its rounding
    assert not np.array_equal(r["Y"], inner["Y"] + oracle.round_bf16(X).astype(np.float64))
    # zero second layer: the block is the identity plus b2
    z = oracle.mixing_block_reduced(ways, X, gamma, beta, W1, b1, np.zeros_like(W2), b2, 1)
    assert np.array_equal(z["Y"], X.astype(np.float64) + b2)


@pytest.mark.parametrize("terms", [1, 3])
def test_transposed_layer_in_reduced_precision(terms):
    """linear_xtw_reduced: the rounding acts on the elements, the product is the transposed layer's."""
    T, C, D = 24, 6, 10
    X = inputs.matrix(61, T, C, "R") * np.float32(3.0)
    W = inputs.matrix(62, T, D, "R", inputs.W_SCALE_EXP)
    b = inputs.matrix(63, 1, D, "R")[0]
    got = oracle.linear_xtw_reduced(X, W, b, terms)
    if terms == 1:
        want = oracle.linear_xtw(oracle.round_bf16(X), oracle.round_bf16(W), b)     # exact products of rounded operands
        assert np.array_equal(got, want)
        assert np.abs(got - oracle.linear_xtw(X, W, b)).max() > 1e-4               # and the rounding is there
    else:
        (xh, xl), (wh, wl) = oracle.split_bf16(X), oracle.split_bf16(W)
        want = (oracle.linear_xtw(xh, wh) + oracle.linear_xtw(xh, wl) + oracle.linear_xtw(xl, wh)) + b.astype(np.float64)
        S = oracle.linear_xtw_reduced(X, W, b, terms, absolute=True)
        assert np.all(np.abs(got - want) <= 1e-14 * S)
        assert np.all(np.abs(got - oracle.linear_xtw(X, W, b)) <= 2.0 ** -15 * oracle.magnitude_xtw(X, W, b))
    # X^T W, not X W^T or W^T X: shapes tell them apart
    assert got.shape == (C, D)
    # lattice values are not changed by the mode
    XL, WL = inputs.matrix(64, T, C, "L"), inputs.matrix(65, T, D, "L")
    assert np.array_equal(oracle.linear_xtw_reduced(XL, WL, None, terms), oracle.linear_xtw(XL, WL))


@pytest.mark.parametrize("terms", [1, 3])
def test_mixed_token_mixing_block_is_the_pinned_pieces_in_sequence(terms):
    T, C, D = 16, 6, 10
    X = (inputs.matrix(71, T, C, "R") + np.float32(0.25)).astype(np.float32)
    gamma = (inputs.matrix(72, 1, C, "R")[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(73, 1, C, "R")[0]
    W1, W2 = inputs.matrix(74, T, D, "R", inputs.W_SCALE_EXP), inputs.matrix(75, T, D, "R", inputs.W_SCALE_EXP)
    b1, b2 = inputs.matrix(76, 1, D, "R")[0], inputs.matrix(77, 1, T, "R")[0]
    r = oracle.token_mixing_block_reduced(1, X, gamma, beta, W1, b1, W2, b2, terms)
    Xn32 = oracle.layernorm(X, gamma, beta, 1).astype(np.float32)
    assert np.array_equal(r["Xn"].astype(np.float32), Xn32)                       # the norm is not rounded to bfloat16
    H = oracle.gelu(oracle.linear_xtw_reduced(Xn32, W1, b1, terms))
    assert np.array_equal(r["H"], H)
    Y = X.astype(np.float64) + oracle.linear_reduced(W2, H.astype(np.float32), None, terms) + b2.astype(np.float64)[:, None]
    assert np.array_equal(r["Y"], Y)
    # against the full-precision block: the split mode is close, the one-term mode visibly rounded
    full = oracle.token_mixing_block(1, X, gamma, beta, W1, b1, W2, b2)
    d = np.abs(r["Y"] - full["Y"]).max()
    assert (d < 1e-4) if terms == 3 else (1e-5 < d < 5e-2)
    # the skip connection and the per-token bias are added in full precision: shifting b2 shifts Y by exactly that
    r2 = oracle.token_mixing_block_reduced(1, X, gamma, beta, W1, b1, W2, b2 + np.float32(0.5), terms)
    assert np.all(np.abs((r2["Y"] - r["Y"]) - 0.5) < 1e-12)


@pytest.mark.parametrize("terms", [1, 3])
def test_backward_in_reduced_precision(terms):
    M, K, N = 12, 10, 6
    X = inputs.matrix(81, M, K, "R") * np.float32(3.0)
    W = inputs.matrix(82, N, K, "R", inputs.W_SCALE_EXP)
    G = inputs.matrix(83, M, N, "R")
    dX, dW = oracle.backward_reduced(X, W, G, terms)
    assert dX.shape == (M, K) and dW.shape == (N, K)
    if terms == 1:      # exact products of the rounded operands: the full-precision backward of the rounded matrices
        wX, wW = oracle.backward(oracle.round_bf16(X), oracle.round_bf16(W), oracle.round_bf16(G))
        assert np.array_equal(dX, wX) and np.array_equal(dW, wW)
        fX, _ = oracle.backward(X, W, G)
        assert np.abs(dX - fX).max() > 1e-5
    else:               # hi hi + hi lo + lo hi of the split operands
        (gh, gl), (wh, wl), (xh, xl) = oracle.split_bf16(G), oracle.split_bf16(W), oracle.split_bf16(X)
        z = np.zeros_like
        wX = oracle.backward(z(X), wh, gh)[0] + oracle.backward(z(X), wl, gh)[0] + oracle.backward(z(X), wh, gl)[0]
        wW = oracle.backward(xh, z(W), gh)[1] + oracle.backward(xl, z(W), gh)[1] + oracle.backward(xh, z(W), gl)[1]
        SX, SW = oracle.backward_reduced(X, W, G, terms, absolute=True)
        assert np.all(np.abs(dX - wX) <= 1e-14 * SX) and np.all(np.abs(dW - wW) <= 1e-14 * SW)
        fX, fW = oracle.backward(X, W, G)
        mX, mW = oracle.backward_magnitude(X, W, G)
        assert np.all(np.abs(dX - fX) <= 2.0 ** -15 * mX) and np.all(np.abs(dW - fW) <= 2.0 ** -15 * mW)
    # lattice values are not changed by the mode, and the adjoint identity holds exactly on them
    XL, WL, GL = inputs.matrix(84, M, K, "L"), inputs.matrix(85, N, K, "L"), inputs.matrix(86, M, N, "L")
    lX, lW = oracle.backward_reduced(XL, WL, GL, terms)
    eX, eW = oracle.backward(XL, WL, GL)
    assert np.array_equal(lX, eX) and np.array_equal(lW, eW)
    assert np.sum(GL.astype(np.float64) * oracle.linear(XL, WL)) == np.sum(lX * XL) == np.sum(lW * WL)


@pytest.mark.parametrize("terms", [1, 3])
def test_mixed_mlp_backward_is_the_pinned_pieces_in_sequence(terms):
    M, C, Hd = 10, 8, 12
    X = inputs.matrix(91, M, C, "R")
    W1, W2 = inputs.matrix(92, Hd, C, "R", inputs.W_SCALE_EXP), inputs.matrix(93, C, Hd, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(94, 1, Hd, "R")[0]
    dY = inputs.matrix(95, M, C, "R")
    r = oracle.mlp_backward_reduced(X, W1, b1, W2, dY, terms)
    A = oracle.linear_reduced(X, W1, b1, terms)
    H32 = oracle.gelu(A).astype(np.float32)
    dH, dW2 = oracle.backward_reduced(H32, W2, dY, terms)
    dA32 = (dH * oracle.gelu_grad(A)).astype(np.float32)
    dXm, dW1 = oracle.backward_reduced(X, W1, dA32, terms)
    assert np.array_equal(r["A"], A) and np.array_equal(r["dH"], dH) and np.array_equal(r["dW2"], dW2)
    assert np.array_equal(r["dX"], dXm + dY) and np.array_equal(r["dW1"], dW1)
    assert np.array_equal(r["db1"], oracle.bias_backward(dA32)) and np.array_equal(r["db2"], oracle.bias_backward(dY))
    # against the full-precision chain: the split mode is close, the one-term mode visibly rounded
    full = oracle.mlp_backward(X, W1, b1, W2, dY)
    for name in ("dX", "dW1", "dW2"):
        ref = full[name] - (dY if name == "dX" else 0.0)        # (without the skip connection, which is not rounded)
        d = (np.abs(r[name] - full[name]) / (np.abs(ref) + np.abs(ref).max())).max()
        assert (d < 1e-4) if terms == 3 else (1e-5 < d < 5e-2), (name, d)
    # and the block: the norm's part is the full-precision one applied to the mixed-precision dXn
    gamma = (inputs.matrix(96, 1, C, "R")[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(97, 1, C, "R")[0]
    rb = oracle.mixing_block_backward_reduced(1, X, gamma, beta, W1, b1, W2, dY, terms)
    Xn32 = oracle.layernorm(X, gamma, beta, 1).astype(np.float32)
    m = oracle.mlp_backward_reduced(Xn32, W1, b1, W2, dY, terms)
    dXl, dg, db = oracle.layernorm_backward(X, gamma, (m["dX"] - dY).astype(np.float32), 1)
    assert np.array_equal(rb["dX"], dY + dXl) and np.array_equal(rb["dgamma"], dg) and np.array_equal(rb["dW1"], m["dW1"])


@pytest.mark.parametrize("terms", [1, 3])
def test_backward_of_the_transposed_layer_in_reduced_precision(terms):
    T, C, D = 12, 6, 10
    X = inputs.matrix(101, T, C, "R") * np.float32(3.0)
    W = inputs.matrix(102, T, D, "R", inputs.W_SCALE_EXP)
    G = inputs.matrix(103, C, D, "R")
    dX, dW = oracle.backward_xtw_reduced(X, W, G, terms)
    assert dX.shape == (T, C) and dW.shape == (T, D)
    fX, fW = oracle.backward_xtw(X, W, G)
    if terms == 1:      # the full-precision backward of the rounded matrices, and visibly not of the unrounded ones
        wX, wW = oracle.backward_xtw(oracle.round_bf16(X), oracle.round_bf16(W), oracle.round_bf16(G))
        assert np.array_equal(dX, wX) and np.array_equal(dW, wW)
        assert np.abs(dW - fW).max() > 1e-5
    else:
        mX, mW = oracle.backward_xtw(X, W, G, absolute=True)
        assert np.all(np.abs(dX - fX) <= 2.0 ** -15 * mX) and np.all(np.abs(dW - fW) <= 2.0 ** -15 * mW)
        assert not np.array_equal(dX, fX)
    XL, WL, GL = inputs.matrix(104, T, C, "L"), inputs.matrix(105, T, D, "L"), inputs.matrix(106, C, D, "L")
    lX, lW = oracle.backward_xtw_reduced(XL, WL, GL, terms)
    eX, eW = oracle.backward_xtw(XL, WL, GL)
    assert np.array_equal(lX, eX) and np.array_equal(lW, eW)
