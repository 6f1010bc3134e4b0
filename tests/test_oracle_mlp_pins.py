"""Pins for the oracle of the mixing MLP  H = gelu(X W1^T + b1),  Y = X + H W2^T + b2  (no GPU).

gelu(x) = x * Phi(x) is pinned to tabulated values of the standard normal distribution function
(six-figure textbook tables and their well-known long forms), to the identity gelu(x) - gelu(-x) = x,
to its limits and its minimum, and to a library erf.  The MLP is pinned to the (already pinned)
forward oracle applied twice, to closed forms in which the activation drops out or is known, and to
its magnitudes' definitions; planted mistakes (tanh form, missing residual, bias inside / outside the
activation) must be told apart.
"""
import math

import numpy as np
import pytest

import oracle
from paper_2507_05753_amd import inputs

# Phi(x) for a few arguments, as printed in standard normal tables (here to 16 digits)
PHI = {0.0: 0.5, 0.5: 0.6914624612740131, 1.0: 0.8413447460685429, 1.5: 0.9331927987311419,
       2.0: 0.9772498680518208, 3.0: 0.9986501019683699}


def test_gelu_against_tabulated_normal_distribution_values():
    for x, phi in PHI.items():
        assert oracle.gelu([x])[0] == pytest.approx(x * phi, rel=1e-15, abs=1e-17)
        assert oracle.gelu([-x])[0] == pytest.approx(-x * (1.0 - phi), rel=2e-13, abs=1e-17)


def test_gelu_identities_and_limits():
    x = np.linspace(-9.0, 9.0, 3601)
    g = oracle.gelu(x)
    assert np.allclose(g - oracle.gelu(-x), x, rtol=0, atol=4e-16 * np.maximum(1.0, np.abs(x)))   # Phi(x) + Phi(-x) = 1
    assert g[x == 0.0][0] == 0.0
    assert np.all(np.abs(g[x > 8.5] - x[x > 8.5]) < 1e-15)           # identity for large arguments
    assert np.all(np.abs(g[x < -8.5]) < 1e-15)                       # zero for very negative ones
    assert np.all(g >= -0.17) and g.min() == pytest.approx(-0.169971, abs=2e-6)   # the dip near x = -0.7518
    assert x[np.argmin(g)] == pytest.approx(-0.7518, abs=5e-3)
    assert np.all(np.diff(g[x > -0.75]) > 0)                         # increasing to the right of the dip
    lib = np.array([0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0))) for t in x])
    assert np.all(np.abs(g - lib) <= 4e-16 * np.maximum(1.0, np.abs(x)))   # (1 + erf cancels for x < 0: absolute bound)
    tanh_form = 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))
    assert np.abs(g - tanh_form).max() > 1e-4                        # the approximation is a different function


def mlp_operands(seed, M, C, Hd, mode="R"):
    X = inputs.matrix(seed, M, C, mode)
    W1 = inputs.matrix(seed + 1, Hd, C, mode, inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, Hd, mode)[0]
    W2 = inputs.matrix(seed + 3, C, Hd, mode, inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 4, 1, C, mode)[0]
    return X, W1, b1, W2, b2


@pytest.mark.parametrize("M,C,Hd", [(5, 6, 8), (17, 12, 30), (40, 64, 24)])
def test_mlp_is_the_forward_oracle_applied_twice(M, C, Hd):
    X, W1, b1, W2, b2 = mlp_operands(61, M, C, Hd)
    r = oracle.mlp(X, W1, b1, W2, b2)
    H = oracle.gelu(oracle.linear(X, W1, b1))
    assert np.array_equal(r["H"], H)                                  # same sums in the same order
    assert np.array_equal(r["S1"], oracle.magnitude(X, W1, b1))
    # second layer on H in double: a library matmul with a rounding bound
    want = X.astype(np.float64) + H @ W2.astype(np.float64).T + b2.astype(np.float64)
    assert np.all(np.abs(r["Y"] - want) <= 4 * Hd * np.finfo(np.float64).eps * r["SY"])
    SY = np.abs(b2.astype(np.float64)) + np.abs(X.astype(np.float64)) + np.abs(H) @ np.abs(W2.astype(np.float64)).T
    assert np.allclose(r["SY"], SY, rtol=1e-12)
    assert np.allclose(r["PY"], r["S1"] @ np.abs(W2.astype(np.float64)).T, rtol=1e-12)
    no_res = oracle.mlp(X, W1, b1, W2, b2, residual=False)
    assert np.allclose(r["Y"] - no_res["Y"], X.astype(np.float64), rtol=0, atol=1e-12)
    assert np.array_equal(no_res["H"], r["H"])


def test_mlp_closed_forms():
    M, C, Hd = 6, 8, 8
    X, W1, b1, W2, b2 = mlp_operands(62, M, C, Hd)
    # zero first layer and zero b1: H = gelu(0) = 0, so Y = X + b2
    r = oracle.mlp(X, np.zeros_like(W1), np.zeros_like(b1), W2, b2)
    assert np.array_equal(r["H"], np.zeros((M, Hd)))
    assert np.array_equal(r["Y"], X.astype(np.float64) + b2.astype(np.float64))
    # zero first layer, b1 = 1: every H is Phi(1); Y = X + Phi(1) * rowsum(W2) + b2
    r = oracle.mlp(X, np.zeros_like(W1), np.ones_like(b1), W2, b2)
    assert np.allclose(r["H"], PHI[1.0], rtol=1e-15)
    rows = np.array([sum(float(v) for v in W2[j]) for j in range(C)])
    assert np.allclose(r["Y"], X + PHI[1.0] * rows + b2, rtol=1e-13, atol=1e-15)
    # identity weights, no bias, large positive inputs: gelu is the identity there, Y = 2 X
    I = np.eye(C, dtype=np.float32)
    Xp = (np.abs(X) + 10.0).astype(np.float32)
    r = oracle.mlp(Xp, I, None, I, None)
    assert np.allclose(r["Y"], 2.0 * Xp.astype(np.float64), rtol=1e-15)
    # ... and large negative inputs: H = 0, Y = X
    r = oracle.mlp(-Xp, I, None, I, None)
    assert np.allclose(r["Y"], -Xp.astype(np.float64), rtol=0, atol=1e-15)


def test_planted_mistakes_are_told_apart():
    X, W1, b1, W2, b2 = mlp_operands(63, 9, 10, 12)
    good = oracle.mlp(X, W1, b1, W2, b2)["Y"]
    pre = oracle.linear(X, W1, b1)
    W2d, b2d, Xd = W2.astype(np.float64), b2.astype(np.float64), X.astype(np.float64)
    tanh_h = 0.5 * pre * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (pre + 0.044715 * pre ** 3)))
    bias_outside = oracle.gelu(oracle.linear(X, W1)) + b1.astype(np.float64)
    assert np.abs(tanh_h - oracle.gelu(pre)).max() > 1e-4        # two orders above the bar H is held to
    for wrong_h, res in ((bias_outside, True), (oracle.gelu(pre), False)):
        wrong = wrong_h @ W2d.T + b2d + (Xd if res else 0.0)
        assert np.abs(wrong - good).max() > 1e-3
    relu = np.maximum(pre, 0.0) @ W2d.T + b2d + Xd
    assert np.abs(relu - good).max() > 1e-3


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_blockwise_mlp_agrees_within_the_rounding_of_h(ways):
    M, C, Hd = 24, 16, 40
    X, W1, b1, W2, b2 = mlp_operands(64, M, C, Hd)
    r = oracle.mlp(X, W1, b1, W2, b2)
    got = oracle.jigsaw_mlp(ways, X, W1, b1, W2, b2)
    # H is handed on in FP32: half an ulp of each H, carried through |W2|
    bound = 2.0 ** -24 * (np.abs(r["H"]) @ np.abs(W2.astype(np.float64)).T) + 1e-14 * r["SY"]
    assert np.all(np.abs(got - r["Y"]) <= bound)


# ---------------------------------------------------------------------------------------------
# the derivative of GELU and the MLP's backward pass
# ---------------------------------------------------------------------------------------------
def test_gelu_grad_tabulated_and_limits():
    g = oracle.gelu_grad(np.array([0.0, 1.0, -1.0, 2.0, 40.0, -40.0]))
    # Phi(1) = 0.8413447461, phi(1) = 0.2419707245, Phi(2) = 0.9772498681, phi(2) = 0.0539909665
    want = [0.5, 0.8413447461 + 0.2419707245, (1 - 0.8413447461) - 0.2419707245, 0.9772498681 + 2 * 0.0539909665, 1.0, 0.0]
    assert np.allclose(g, want, rtol=0, atol=2e-10)
    # gelu'(x) + gelu'(-x) = 1 (from gelu(x) - gelu(-x) = x)
    x = np.linspace(-6, 6, 97)
    assert np.allclose(oracle.gelu_grad(x) + oracle.gelu_grad(-x), 1.0, rtol=0, atol=1e-15)


def test_gelu_grad_is_the_slope_of_the_pinned_gelu():
    x = np.linspace(-5, 5, 201)
    h = 1e-5
    slope = (oracle.gelu(x + h) - oracle.gelu(x - h)) / (2 * h)
    assert np.allclose(oracle.gelu_grad(x), slope, rtol=0, atol=1e-9)
    # the tanh approximation's derivative is another function
    t = lambda v: 0.5 * v * (1 + np.tanh(0.7978845608 * (v + 0.044715 * v ** 3)))
    assert np.abs((t(x + h) - t(x - h)) / (2 * h) - oracle.gelu_grad(x)).max() > 1e-4


def test_mlp_backward_against_the_library_autograd_in_double():
    import torch
    M, C, Hd = 6, 8, 10
    X, W1, b1 = inputs.layer_inputs(340, M, C, Hd, "R", bias=True)
    W2 = inputs.matrix(341, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(342, 1, C, "R")[0]
    dY = inputs.matrix(343, M, C, "R")
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64)).requires_grad_(True)
    Xt, W1t, b1t, W2t, b2t = t(X), t(W1), t(b1), t(W2), t(b2)
    A = Xt @ W1t.T + b1t
    Y = Xt + torch.nn.functional.gelu(A) @ W2t.T + b2t
    Y.backward(torch.from_numpy(dY).double())
    r = oracle.mlp_backward(X, W1, b1, W2, dY)
    # H and dA are handed on in FP32 by the method: agreement to their rounding, carried through one product
    for name, ref in (("dX", Xt.grad), ("dW1", W1t.grad), ("db1", b1t.grad), ("dW2", W2t.grad), ("db2", b2t.grad)):
        ref = ref.numpy()
        assert np.all(np.abs(r[name] - ref) <= 1e-6 * (np.abs(ref) + np.abs(ref).max())), name
    assert np.allclose(r["A"], A.detach().numpy(), rtol=0, atol=1e-13)
    # the skip connection's share: without it dX would miss dY
    through = np.abs(r["dX"] - dY).max()                        # what comes back through the two layers
    assert through > 1e-5 and np.abs((r["dX"] - dY) - (Xt.grad.numpy() - dY)).max() < 1e-5 * through


def test_mlp_backward_is_the_pinned_pieces_in_sequence():
    M, C, Hd = 5, 6, 8
    X, W1, b1 = inputs.layer_inputs(344, M, C, Hd, "R", bias=True)
    W2 = inputs.matrix(345, C, Hd, "R", inputs.W_SCALE_EXP)
    dY = inputs.matrix(346, M, C, "R")
    r = oracle.mlp_backward(X, W1, b1, W2, dY)
    A = oracle.linear(X, W1, b1)
    H32 = oracle.gelu(A).astype(np.float32)
    dH, dW2 = oracle.backward(H32, W2, dY)
    assert np.array_equal(r["dH"], dH) and np.array_equal(r["dW2"], dW2)
    dA = dH * oracle.gelu_grad(A)
    assert np.array_equal(r["dA"], dA)
    dXm, dW1 = oracle.backward(X, W1, dA.astype(np.float32))
    assert np.array_equal(r["dX"], dXm + dY) and np.array_equal(r["dW1"], dW1)
    assert np.array_equal(r["db1"], oracle.bias_backward(dA.astype(np.float32)))
    assert np.array_equal(r["db2"], oracle.bias_backward(dY))
