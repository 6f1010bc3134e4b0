"""Pins for the layer-norm oracle and the pre-norm channel-mixing block built from it (no GPU).

The paper (Sec. 3; Sec. 5 "Layer norms") names the layer norm of the library it uses, over the channels
of a token; with the channels split over ranks each rank normalises over the channels it holds.  The
oracle is pinned by rows whose normalised form is known in closed form, by the moments of its output,
by its invariances, by the library routine in double, by the independence of channel blocks and tokens,
and by planted mistakes that these pins must tell apart from the right formula.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2507_05753_amd import inputs

EPS = oracle.LN_EPS


def data(seed, M, C, mode="R", shift=0.0):
    X = inputs.matrix(seed, M, C, mode) + np.float32(shift)
    gamma = inputs.matrix(seed + 1, 1, C, mode)[0] + np.float32(1.5)
    beta = inputs.matrix(seed + 2, 1, C, mode)[0]
    return X.astype(np.float32), gamma.astype(np.float32), beta.astype(np.float32)


def test_default_eps_is_the_library_default():
    assert EPS == torch.nn.LayerNorm(4).eps == 1e-5


def test_constant_rows_map_to_beta():
    # x - mean = 0 exactly, whatever the variance term is
    C = 12
    X = np.full((3, C), 2.75, dtype=np.float32)
    _, gamma, beta = data(1, 3, C)
    assert np.array_equal(oracle.layernorm(X, gamma, beta), np.tile(beta.astype(np.float64), (3, 1)))
    assert np.array_equal(oracle.layernorm(X), np.zeros((3, C)))


def test_plus_minus_one_rows():
    # mean 0, variance 1: y = x / sqrt(1 + eps) * gamma + beta
    C = 16
    X = np.tile(np.array([1.0, -1.0], dtype=np.float32), (2, C // 2))
    _, gamma, beta = data(2, 2, C)
    want = X.astype(np.float64) / math.sqrt(1.0 + EPS) * gamma + beta
    got = oracle.layernorm(X, gamma, beta)
    assert np.allclose(got, want, rtol=0, atol=4 * np.finfo(np.float64).eps * (np.abs(want).max() + 1))
    # eps = 0: exactly x * gamma + beta up to the last bit of the products
    got = oracle.layernorm(X, gamma, beta, eps=0.0)
    assert np.allclose(got, X.astype(np.float64) * gamma + beta, rtol=0, atol=1e-15)


def test_arithmetic_progression():
    # x = 0, 1, ..., C-1: mean (C-1)/2, biased variance (C^2 - 1)/12
    C = 9
    X = np.arange(C, dtype=np.float32)[None, :]
    want = (np.arange(C) - (C - 1) / 2) / math.sqrt((C * C - 1) / 12 + EPS)
    assert np.allclose(oracle.layernorm(X)[0], want, rtol=0, atol=1e-15)
    # an unbiased variance (divisor C - 1) would give another number
    wrong = (np.arange(C) - (C - 1) / 2) / math.sqrt((C * C - 1) / 12 * C / (C - 1) + EPS)
    assert np.abs(wrong - want).max() > 1e-3


def test_eps_sits_inside_the_root():
    # tiny variance: eps dominates; y = d / sqrt(var + eps), not d / (sqrt(var) + eps)
    X = np.array([[1.0, 1.0 + 2.0 ** -10]], dtype=np.float32)
    d = 2.0 ** -11
    want = np.array([-d, d]) / math.sqrt(d * d + EPS)
    assert np.allclose(oracle.layernorm(X)[0], want, rtol=1e-14, atol=0)
    outside = np.array([-d, d]) / (math.sqrt(d * d) + EPS)
    assert np.abs(outside - want).max() > 0.1


@pytest.mark.parametrize("M,C", [(4, 8), (7, 50), (3, 4320)])
def test_moments_of_the_output(M, C):
    X, _, _ = data(3, M, C, shift=0.75)
    Y = oracle.layernorm(X)
    assert np.all(np.abs(Y.mean(axis=1)) <= 1e-13)
    var = X.astype(np.float64).var(axis=1)
    assert np.allclose((Y * Y).mean(axis=1), var / (var + EPS), rtol=1e-12, atol=0)


def test_shift_and_scale_invariance():
    M, C = 5, 40
    X, gamma, beta = data(4, M, C, "L")
    base = oracle.layernorm(X, gamma, beta)
    shifted = oracle.layernorm(X + np.float32(8.0), gamma, beta)      # lattice values: the shift is exact
    assert np.allclose(shifted, base, rtol=0, atol=1e-13)
    # scaling by 4 is exact in FP32; with eps scaled by 16 the result is the same
    scaled = oracle.layernorm(X * np.float32(4.0), gamma, beta, eps=16 * EPS)
    assert np.allclose(scaled, base, rtol=0, atol=1e-13)
    # and with the same eps it is not (eps matters)
    assert np.abs(oracle.layernorm(X * np.float32(4.0), gamma, beta) - base).max() > 1e-9


@pytest.mark.parametrize("M,C", [(1, 2), (6, 10), (33, 130), (4, 4320)])
@pytest.mark.parametrize("affine", [False, True])
def test_library_routine_in_double(M, C, affine):
    X, gamma, beta = data(5, M, C, shift=0.3)
    g = torch.from_numpy(gamma).double() if affine else None
    b = torch.from_numpy(beta).double() if affine else None
    want = torch.nn.functional.layer_norm(torch.from_numpy(X).double(), (C,), g, b, EPS).numpy()
    got, S = oracle.layernorm(X, gamma if affine else None, beta if affine else None, magnitude=True)
    assert np.all(np.abs(got - want) <= 64 * np.finfo(np.float64).eps * S)


@pytest.mark.parametrize("groups", [1, 2])
def test_channel_blocks_and_tokens_are_independent(groups):
    M, C = 6, 24
    X, gamma, beta = data(6, M, C)
    Y = oracle.layernorm(X, gamma, beta, groups)
    Cg = C // groups
    for g in range(groups):
        sl = slice(g * Cg, (g + 1) * Cg)
        assert np.array_equal(Y[:, sl], oracle.layernorm(X[:, sl], gamma[sl], beta[sl]))
    # changing one token changes only that row; changing one block changes only that block
    X2 = X.copy()
    X2[2, 1] += np.float32(3.0)
    Y2 = oracle.layernorm(X2, gamma, beta, groups)
    changed = np.argwhere(Y2 != Y)
    assert set(changed[:, 0]) == {2}
    assert changed[:, 1].max() < Cg
    if groups == 2:
        assert not np.array_equal(Y, oracle.layernorm(X, gamma, beta, 1))     # statistics over the whole row differ


def test_magnitude_bounds_the_output():
    X, gamma, beta = data(7, 9, 30, shift=-2.0)
    Y, S = oracle.layernorm(X, gamma, beta, 2, magnitude=True)
    assert np.all(np.abs(Y) <= S * (1 + 1e-15))
    Xd = X.astype(np.float64)
    for g in range(2):
        sl = slice(g * 15, (g + 1) * 15)
        mu = Xd[:, sl].mean(axis=1, keepdims=True)
        rstd = 1 / np.sqrt(Xd[:, sl].var(axis=1, keepdims=True) + EPS)
        want = (np.abs(Xd[:, sl]) + np.abs(mu)) * rstd * np.abs(gamma[sl]) + np.abs(beta[sl])
        assert np.allclose(S[:, sl], want, rtol=1e-13, atol=0)


def test_argument_checks():
    X, gamma, beta = data(8, 3, 9)
    with pytest.raises(RuntimeError):
        oracle.layernorm(X, gamma, beta, 2)          # 9 channels do not split in two
    with pytest.raises(RuntimeError):
        oracle.layernorm(X, gamma, beta, 0)
    with pytest.raises(RuntimeError):
        oracle.layernorm(X, gamma, beta, eps=-1.0)
    assert oracle.layernorm(np.zeros((0, 8), np.float32)).shape == (0, 8)
    assert oracle.ln_groups(1) == 1 and oracle.ln_groups(2) == 2 and oracle.ln_groups(4) == 2
    with pytest.raises(RuntimeError):
        oracle.ln_groups(3)


# ---------------------------------------------------------------------------------------------
# the pre-norm channel-mixing block: Y = X + MLP(layernorm(X))
# ---------------------------------------------------------------------------------------------
def block_operands(seed, M, C, Hd, mode="R"):
    X, W1, b1 = inputs.layer_inputs(seed, M, C, Hd, mode)
    W2 = inputs.matrix(seed + 50, C, Hd, mode, inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 51, 1, C, mode)[0]
    _, gamma, beta = data(seed + 52, 1, C, mode)
    return X, gamma, beta, W1, b1, W2, b2


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_block_is_the_pinned_pieces_in_sequence(ways):
    M, C, Hd = 6, 8, 10
    X, gamma, beta, W1, b1, W2, b2 = block_operands(9, M, C, Hd)
    out = oracle.mixing_block(ways, X, gamma, beta, W1, b1, W2, b2)
    Xn = oracle.layernorm(X, gamma, beta, oracle.ln_groups(ways))
    assert np.array_equal(out["Xn"], Xn)
    H = oracle.gelu(oracle.linear(Xn.astype(np.float32), W1, b1))
    assert np.array_equal(out["H"], H)
    # second layer from H in double, by a library product
    want = X.astype(np.float64) + H @ W2.astype(np.float64).T + b2
    assert np.allclose(out["Y"], want, rtol=0, atol=1e-12 * np.abs(out["SY"]).max())


def test_block_with_zero_second_layer_is_the_identity_plus_bias():
    M, C, Hd = 4, 6, 8
    X, gamma, beta, W1, b1, W2, b2 = block_operands(10, M, C, Hd)
    out = oracle.mixing_block(2, X, gamma, beta, W1, b1, np.zeros_like(W2), b2)
    assert np.array_equal(out["Y"], X.astype(np.float64) + b2)


def test_block_sees_the_norm():
    # constant rows: layernorm gives beta for every token, so Y - X is the same row for all tokens
    M, C, Hd = 5, 6, 8
    X, gamma, beta, W1, b1, W2, b2 = block_operands(11, M, C, Hd)
    X = np.tile(np.arange(M, dtype=np.float32)[:, None], (1, C))
    out = oracle.mixing_block(1, X, gamma, beta, W1, b1, W2, b2)
    D = out["Y"] - X
    assert np.allclose(D, np.tile(D[0], (M, 1)), rtol=0, atol=1e-13)
    # without the norm the rows would differ
    plain = oracle.mlp(X, W1, b1, W2, b2)["Y"] - X
    assert np.abs(plain - plain[0]).max() > 1e-3


# ---------------------------------------------------------------------------------------------
# the token-mixing half of a mixing block: per channel, y_c = x_c + W2 gelu(W1^T xn_c + b1) + b2
# ---------------------------------------------------------------------------------------------
def token_operands(seed, T, C, D, mode="R"):
    X = (inputs.matrix(seed, T, C, mode) + np.float32(0.25)).astype(np.float32)
    W1 = inputs.matrix(seed + 60, T, D, mode, inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 61, 1, D, mode)[0]
    W2 = inputs.matrix(seed + 62, T, D, mode, inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 63, 1, T, mode)[0]
    _, gamma, beta = data(seed + 64, 1, C, mode)
    return X, gamma, beta, W1, b1, W2, b2


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_token_mixing_channel_by_channel(ways):
    """The definition, one channel at a time, with library products in double."""
    T, C, D = 10, 8, 6
    X, gamma, beta, W1, b1, W2, b2 = token_operands(12, T, C, D)
    out = oracle.token_mixing_block(ways, X, gamma, beta, W1, b1, W2, b2)
    Xn = oracle.layernorm(X, gamma, beta, oracle.ln_groups(ways))
    assert np.array_equal(out["Xn"], Xn)
    Xn32 = Xn.astype(np.float32).astype(np.float64)
    W1d, W2d = W1.astype(np.float64), W2.astype(np.float64)
    for c in range(C):
        h = oracle.gelu(W1d.T @ Xn32[:, c] + b1)                     # [D]
        assert np.allclose(out["H"][c], h, rtol=0, atol=1e-13)
        h32 = out["H"][c].astype(np.float32).astype(np.float64)       # handed on in FP32
        y = X[:, c].astype(np.float64) + W2d @ h32 + b2
        assert np.allclose(out["Y"][:, c], y, rtol=0, atol=1e-12 * np.abs(out["SY"][:, c]).max())


def test_token_mixing_in_closed_form():
    """All-integer operands with gamma = 1, beta = 0 replaced by a norm that is known: constant channels.  With every
    token's channels equal the layer norm gives beta for every entry, so H and Y follow from small integers."""
    T, C, D = 6, 4, 5
    X = np.tile(np.arange(1, T + 1, dtype=np.float32)[:, None], (1, C))      # token t holds t + 1 in every channel
    gamma = np.ones(C, dtype=np.float32)
    beta = np.full(C, 2.0, dtype=np.float32)                                   # Xn = 2 everywhere, exactly
    rng = np.random.default_rng(5)
    W1 = rng.integers(0, 2, (T, D)).astype(np.float32)
    b1 = np.full(D, 10.0, dtype=np.float32)                                    # pre-activation >= 10: gelu(x) = x in double
    W2 = rng.integers(-1, 2, (T, D)).astype(np.float32)
    b2 = rng.integers(-3, 4, T).astype(np.float32)
    out = oracle.token_mixing_block(1, X, gamma, beta, W1, b1, W2, b2)
    h = 2 * W1.astype(np.int64).sum(axis=0) + 10                               # the same for every channel
    assert np.array_equal(out["H"], np.tile(h.astype(np.float64), (C, 1)))
    y = X.astype(np.int64) + (W2.astype(np.int64) @ h)[:, None] + b2.astype(np.int64)[:, None]
    assert np.array_equal(out["Y"], y.astype(np.float64))
    # the bias of the second layer goes with the token (row), not with the channel
    assert not np.array_equal(y, X.astype(np.int64) + (W2.astype(np.int64) @ h)[:, None] + b2.astype(np.int64)[None, :C].repeat(T, 0)) \
        or np.all(b2 == b2[0])


def test_token_mixing_mixes_tokens_not_channels():
    T, C, D = 8, 6, 5
    X, gamma, beta, W1, b1, W2, b2 = token_operands(13, T, C, D)
    base = oracle.token_mixing_block(1, X, gamma, beta, W1, b1, W2, b2)
    # changing one weight row (one token's weights) changes every channel; channels do not mix apart from the norm:
    # with the norm switched to a fixed input (gamma = 0) a change in one channel of X moves only that channel of Y
    g0 = np.zeros_like(gamma)
    a = oracle.token_mixing_block(1, X, g0, beta, W1, b1, W2, b2)
    X2 = X.copy()
    X2[3, 2] += np.float32(1.0)
    b = oracle.token_mixing_block(1, X2, g0, beta, W1, b1, W2, b2)
    changed = np.argwhere(a["Y"] != b["Y"])
    assert set(changed[:, 1]) == {2} and set(changed[:, 0]) == {3}             # only through the skip connection
    # with the norm in place the same change reaches all tokens of all channels of that token's norm group
    c2 = oracle.token_mixing_block(1, X2, gamma, beta, W1, b1, W2, b2)
    assert len(np.argwhere(c2["Y"] != base["Y"])) > T
    # zero second layer: identity plus the per-token bias
    z = oracle.token_mixing_block(2, X, gamma, beta, W1, b1, np.zeros_like(W2), b2)
    assert np.array_equal(z["Y"], X.astype(np.float64) + b2.astype(np.float64)[:, None])


# ---------------------------------------------------------------------------------------------
# the layer norm's gradients
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("groups", [1, 2])
def test_layernorm_backward_against_differences_of_the_forward(groups):
    """<dY, LN(X + h E) - LN(X - h E)> / 2h -> <dX, E>.  X on a lattice and h = 2^-10, so that X +- h E is exact in
    FP32 (the forward oracle takes FP32 input); the central difference is then accurate to O(h^2)."""
    M, C = 5, 12
    X, gamma, beta = data(30, M, C, "L")
    dY = inputs.matrix(31, M, C, "R")
    dX, dg, db = oracle.layernorm_backward(X, gamma, dY, groups)
    h = 2.0 ** -10
    rng = np.random.default_rng(1)
    for _ in range(6):
        E = rng.integers(-1, 2, (M, C)).astype(np.float32)
        fp = oracle.layernorm((X + np.float32(h) * E).astype(np.float32), gamma, beta, groups)
        fm = oracle.layernorm((X - np.float32(h) * E).astype(np.float32), gamma, beta, groups)
        lhs = (dY.astype(np.float64) * (fp - fm)).sum() / (2 * h)
        rhs = (dX * E).sum()
        assert abs(lhs - rhs) <= 2e-5 * (np.abs(dX).sum() + 1)
    # gamma and beta enter linearly: the differences are exact
    for c in (0, 5, C - 1):
        e = np.zeros(C, dtype=np.float32)
        e[c] = 1.0
        dgc = (dY.astype(np.float64) * (oracle.layernorm(X, gamma + e, beta, groups) - oracle.layernorm(X, gamma, beta, groups))).sum()
        dbc = (dY.astype(np.float64) * (oracle.layernorm(X, gamma, beta + e, groups) - oracle.layernorm(X, gamma, beta, groups))).sum()
        assert abs(dgc - dg[c]) <= 1e-12 * (abs(dg[c]) + 1) and abs(dbc - db[c]) <= 1e-12 * (abs(db[c]) + 1)


@pytest.mark.parametrize("groups", [1, 2])
def test_layernorm_backward_against_the_library_in_double(groups):
    M, C = 7, 10
    X, gamma, beta = data(32, M, C, shift=0.3)
    dY = inputs.matrix(33, M, C, "R")
    n = C // groups
    Xt = torch.from_numpy(X).double().requires_grad_(True)
    gt = torch.from_numpy(gamma).double().requires_grad_(True)
    bt = torch.from_numpy(beta).double().requires_grad_(True)
    out = torch.cat([torch.nn.functional.layer_norm(Xt[:, b * n:(b + 1) * n], (n,), gt[b * n:(b + 1) * n],
                                                    bt[b * n:(b + 1) * n], EPS) for b in range(groups)], dim=1)
    out.backward(torch.from_numpy(dY).double())
    dX, dg, db, SX, Sg, Sb = oracle.layernorm_backward(X, gamma, dY, groups, magnitude=True)
    assert np.all(np.abs(dX - Xt.grad.numpy()) <= 1e-12 * SX)
    assert np.all(np.abs(dg - gt.grad.numpy()) <= 1e-12 * Sg) and np.all(np.abs(db - bt.grad.numpy()) <= 1e-12 * Sb)


def test_layernorm_backward_invariants():
    M, C = 6, 16
    X, gamma, beta = data(34, M, C, shift=-0.4)
    dY = inputs.matrix(35, M, C, "R")
    dX, dg, db = oracle.layernorm_backward(X, gamma, dY, 2)
    # the output does not change when a constant is added to a block's channels: dX sums to zero per block
    assert np.all(np.abs(dX[:, :8].sum(axis=1)) <= 1e-12) and np.all(np.abs(dX[:, 8:].sum(axis=1)) <= 1e-12)
    # a gradient along gamma-scaled constants is annihilated: dY = c / gamma per row gives g = const, xhat-free
    dZ = (np.ones((M, C)) / gamma.astype(np.float64)).astype(np.float32)
    dX0, _, _ = oracle.layernorm_backward(X, gamma, dZ, 1)
    assert np.all(np.abs(dX0) <= 1e-5 * np.abs(dX).max())
    # dbeta is the column sum, dgamma with gamma = None is that of gamma = 1
    assert np.allclose(db, oracle.bias_backward(dY), rtol=0, atol=1e-13)
    a = oracle.layernorm_backward(X, None, dY, 1)
    b = oracle.layernorm_backward(X, np.ones(C, np.float32), dY, 1)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    with pytest.raises(RuntimeError):
        oracle.layernorm_backward(X[:, :9], None, dY[:, :9], 2)


@pytest.mark.parametrize("ways", [1, 2])
def test_mixing_block_backward_against_the_library_autograd_in_double(ways):
    M, C, Hd = 6, 8, 10
    X, gamma, beta, W1, _, W2, b2 = block_operands(40, M, C, Hd)
    b1 = inputs.matrix(42, 1, Hd, "R")[0]
    dY = inputs.matrix(41, M, C, "R")
    groups = oracle.ln_groups(ways)
    n = C // groups
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64)).requires_grad_(True)
    Xt, gt, bt, W1t, b1t, W2t, b2t = t(X), t(gamma), t(beta), t(W1), t(b1), t(W2), t(b2)
    Xn = torch.cat([torch.nn.functional.layer_norm(Xt[:, k * n:(k + 1) * n], (n,), gt[k * n:(k + 1) * n],
                                                   bt[k * n:(k + 1) * n], EPS) for k in range(groups)], dim=1)
    Y = Xt + torch.nn.functional.gelu(Xn @ W1t.T + b1t) @ W2t.T + b2t
    Y.backward(torch.from_numpy(dY).double())
    r = oracle.mixing_block_backward(ways, X, gamma, beta, W1, b1, W2, dY)
    for name, ref in (("dX", Xt.grad), ("dgamma", gt.grad), ("dbeta", bt.grad), ("dW1", W1t.grad), ("db1", b1t.grad),
                      ("dW2", W2t.grad), ("db2", b2t.grad)):
        ref = ref.numpy()
        # Xn, H, dA and dXn are handed on in FP32 by the method
        assert np.all(np.abs(r[name] - ref) <= 2e-6 * (np.abs(ref) + np.abs(ref).max())), name
    # the pieces in sequence
    Xn32 = oracle.layernorm(X, gamma, beta, groups).astype(np.float32)
    m = oracle.mlp_backward(Xn32, W1, b1, W2, dY)
    assert np.array_equal(r["dXn"], m["dX"] - dY) and np.array_equal(r["dW1"], m["dW1"])
    dXl, dg, db = oracle.layernorm_backward(X, gamma, r["dXn"].astype(np.float32), groups)
    assert np.array_equal(r["dX"], dY + dXl) and np.array_equal(r["dgamma"], dg) and np.array_equal(r["dbeta"], db)


@pytest.mark.parametrize("ways", [1, 2])
def test_token_mixing_block_backward_against_the_library_autograd_in_double(ways):
    T, C, D = 6, 8, 10
    X, gamma, beta = data(44, T, C, shift=0.2)
    W1 = inputs.matrix(45, T, D, "R", inputs.W_SCALE_EXP)
    W2 = inputs.matrix(46, T, D, "R", inputs.W_SCALE_EXP)
    b1, b2 = inputs.matrix(47, 1, D, "R")[0], inputs.matrix(48, 1, T, "R")[0]
    dY = inputs.matrix(49, T, C, "R")
    groups = oracle.ln_groups(ways)
    n = C // groups
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64)).requires_grad_(True)
    Xt, gt, bt, W1t, b1t, W2t, b2t = t(X), t(gamma), t(beta), t(W1), t(b1), t(W2), t(b2)
    Xn = torch.cat([torch.nn.functional.layer_norm(Xt[:, k * n:(k + 1) * n], (n,), gt[k * n:(k + 1) * n],
                                                   bt[k * n:(k + 1) * n], EPS) for k in range(groups)], dim=1)
    Y = Xt + W2t @ torch.nn.functional.gelu(Xn.T @ W1t + b1t).T + b2t[:, None]
    # the forward this is the gradient of is the pinned one
    fwd = oracle.token_mixing_block(ways, X, gamma, beta, W1, b1, W2, b2)
    assert np.all(np.abs(fwd["Y"] - Y.detach().numpy()) <= 1e-6 * fwd["SY"])
    Y.backward(torch.from_numpy(dY).double())
    r = oracle.token_mixing_block_backward(ways, X, gamma, beta, W1, b1, W2, dY)
    for name, ref in (("dX", Xt.grad), ("dgamma", gt.grad), ("dbeta", bt.grad), ("dW1", W1t.grad), ("db1", b1t.grad),
                      ("dW2", W2t.grad), ("db2", b2t.grad)):
        ref = ref.numpy()
        assert r[name].shape == ref.shape, name
        # Xn, H, dA and dXn are handed on in FP32 by the method
        assert np.all(np.abs(r[name] - ref) <= 2e-6 * (np.abs(ref) + np.abs(ref).max())), name
    assert np.array_equal(r["db2"], dY.astype(np.float64).sum(axis=1))      # few terms: the order does not matter here
