"""Pins for the oracle's mixed-precision chains and for the block partition (no GPU).

The chains (`mlp_backward_reduced`, `mixing_block_backward_reduced`, `token_mixing_block_reduced`,
`token_mixing_block_backward_reduced` and their full-precision counterparts) follow Sec. 3 (the mixing block),
Sec. 4.1 (the backward products), Sec. 5 (the transposed layer) and Sec. 6.1 (mixed precision: only the
operands of a matrix product are rounded).  None of the pins below calls the oracle's own pieces to build an
expected value:

* all-integer operands for which every rounding is the identity and GELU is the identity on the values it
  sees: each chain must then equal its full-precision counterpart bit for bit, and both must equal the chain
  written with integer matrix products;
* tiny shapes, every quantity written out element by element in Python floats (`math.erf`, the library's
  bfloat16 conversion), general values, so that every rounding point shows in the result;
* planted mistakes (the pre-activation rounded before GELU, an unrounded product, a rounded skip connection,
  a derivative taken at the rounded point, truncation instead of rounding to nearest) which the second pin
  must catch;
* `shard_blocks` against literal blocks, against the per-tensor partitions and the zero-redundancy rule of Sec. 4.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2507_05753_amd import inputs


# ---------------------------------------------------------------------------------------------
# scalar arithmetic of the mode, independent of the oracle
# ---------------------------------------------------------------------------------------------
def rb(x: float) -> float:
    """x (an FP32 value) rounded to bfloat16 by the library's conversion."""
    return float(torch.tensor(float(x), dtype=torch.float32).to(torch.bfloat16).to(torch.float32).item())


def f32(x: float) -> float:
    return float(np.float32(x))


def product(a: float, b: float, terms: int) -> float:
    """One product of two FP32 values as the mode forms it (Sec. 6.1 read for this chip): the operands rounded to
    bfloat16, or split in hi + lo with the lo * lo term dropped."""
    if terms == 0:                  # full precision: the exact product
        return float(a) * float(b)
    if terms == 1:
        return rb(a) * rb(b)
    ah, bh = rb(a), rb(b)
    al, bl = rb(f32(a - ah)), rb(f32(b - bh))
    return ah * bh + ah * bl + al * bh


def gelu_s(a: float) -> float:
    return 0.5 * a * (1.0 + math.erf(a / math.sqrt(2.0)))


def gelu_grad_s(a: float) -> float:
    return 0.5 * (1.0 + math.erf(a / math.sqrt(2.0))) + a * math.exp(-0.5 * a * a) / math.sqrt(2.0 * math.pi)


def norm_rows(X, gamma, beta, groups, eps):
    """Layer norm over each channel block of each row, element by element: (xhat, rstd, out)."""
    M, C = len(X), len(X[0])
    n = C // groups
    xhat = [[0.0] * C for _ in range(M)]
    rstd = [[0.0] * groups for _ in range(M)]
    out = [[0.0] * C for _ in range(M)]
    for i in range(M):
        for b in range(groups):
            cs = range(b * n, (b + 1) * n)
            mu = sum(float(X[i][c]) for c in cs) / n
            var = sum((float(X[i][c]) - mu) ** 2 for c in cs) / n
            rstd[i][b] = 1.0 / math.sqrt(var + eps)
            for c in cs:
                xhat[i][c] = (float(X[i][c]) - mu) * rstd[i][b]
                out[i][c] = xhat[i][c] * float(gamma[c]) + float(beta[c])
    return xhat, rstd, out


def norm_rows_backward(xhat, rstd, gamma, dOut, groups):
    """Gradient of the layer norm with respect to its input, element by element (the derivative of the definition:
    mean and variance depend on every channel of the block)."""
    M, C = len(xhat), len(xhat[0])
    n = C // groups
    dX = [[0.0] * C for _ in range(M)]
    for i in range(M):
        for b in range(groups):
            cs = range(b * n, (b + 1) * n)
            g = {c: float(dOut[i][c]) * float(gamma[c]) for c in cs}
            mg = sum(g[c] for c in cs) / n
            mgx = sum(g[c] * xhat[i][c] for c in cs) / n
            for c in cs:
                dX[i][c] = (g[c] - mg - xhat[i][c] * mgx) * rstd[i][b]
    return dX


def close(got, want, scale=None, tol=1e-12):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    s = np.abs(want).max() + 1e-300 if scale is None else scale
    assert np.all(np.abs(got - want) <= tol * s), float(np.abs(got - want).max() / s)


# ---------------------------------------------------------------------------------------------
# the channel-mixing MLP's backward and the block around it, element by element
# ---------------------------------------------------------------------------------------------
def mlp_backward_by_hand(X, W1, b1, W2, dY, terms, with_skip=True):
    M, C, Hd = len(X), len(X[0]), len(W1)
    A = [[float(b1[h]) + sum(product(X[i][c], W1[h][c], terms) for c in range(C)) for h in range(Hd)] for i in range(M)]
    H32 = [[f32(gelu_s(A[i][h])) for h in range(Hd)] for i in range(M)]
    dH = [[sum(product(dY[i][c], W2[c][h], terms) for c in range(C)) for h in range(Hd)] for i in range(M)]
    dW2 = [[sum(product(dY[i][c], H32[i][h], terms) for i in range(M)) for h in range(Hd)] for c in range(C)]
    dA = [[dH[i][h] * gelu_grad_s(A[i][h]) for h in range(Hd)] for i in range(M)]
    dA32 = [[f32(v) for v in row] for row in dA]
    dXm = [[sum(product(dA32[i][h], W1[h][c], terms) for h in range(Hd)) for c in range(C)] for i in range(M)]
    dW1 = [[sum(product(dA32[i][h], X[i][c], terms) for i in range(M)) for c in range(C)] for h in range(Hd)]
    db1 = [sum(dA32[i][h] for i in range(M)) for h in range(Hd)]
    db2 = [sum(float(dY[i][c]) for i in range(M)) for c in range(C)]
    dX = [[dXm[i][c] + (float(dY[i][c]) if with_skip else 0.0) for c in range(C)] for i in range(M)]
    return dict(A=A, dH=dH, dA=dA, dX=dX, dW1=dW1, db1=db1, dW2=dW2, db2=db2)


def mixing_block_backward_by_hand(groups, X, gamma, beta, W1, b1, W2, dY, terms, eps):
    xhat, rstd, xn = norm_rows(X, gamma, beta, groups, eps)
    Xn32 = [[f32(v) for v in row] for row in xn]
    r = mlp_backward_by_hand(Xn32, W1, b1, W2, dY, terms, with_skip=False)
    dXn32 = [[f32(v) for v in row] for row in r["dX"]]
    dXl = norm_rows_backward(xhat, rstd, gamma, dXn32, groups)
    M, C = len(X), len(X[0])
    r["dXn"] = r["dX"]
    r["dX"] = [[float(dY[i][c]) + dXl[i][c] for c in range(C)] for i in range(M)]
    r["dgamma"] = [sum(dXn32[i][c] * xhat[i][c] for i in range(M)) for c in range(C)]
    r["dbeta"] = [sum(dXn32[i][c] for i in range(M)) for c in range(C)]
    return r


def mlp_data(seed, M, C, Hd):
    X = inputs.matrix(seed, M, C, "R") * np.float32(1.7)
    W1 = inputs.matrix(seed + 1, Hd, C, "R") * np.float32(0.9)
    W2 = inputs.matrix(seed + 2, C, Hd, "R") * np.float32(1.1)
    b1 = inputs.matrix(seed + 3, 1, Hd, "R")[0]
    dY = inputs.matrix(seed + 4, M, C, "R") * np.float32(1.3)
    gamma = (inputs.matrix(seed + 5, 1, C, "R")[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(seed + 6, 1, C, "R")[0]
    return X, W1, b1, W2, dY, gamma, beta


def check_mlp_backward_reduced(terms):
    X, W1, b1, W2, dY, _, _ = mlp_data(500, 5, 6, 4)
    got = oracle.mlp_backward_reduced(X, W1, b1, W2, dY, terms)
    want = mlp_backward_by_hand(X, W1, b1, W2, dY, terms)
    for name in want:
        close(got[name], want[name])


def check_mixing_block_backward_reduced(terms, ways):
    X, W1, b1, W2, dY, gamma, beta = mlp_data(520, 5, 6, 4)
    got = oracle.mixing_block_backward_reduced(ways, X, gamma, beta, W1, b1, W2, dY, terms, eps=1e-5)
    want = mixing_block_backward_by_hand(oracle.ln_groups(ways), X, gamma, beta, W1, b1, W2, dY, terms, 1e-5)
    for name in want:
        close(got[name], want[name], tol=1e-11)


@pytest.mark.parametrize("terms", [1, 3])
def test_mlp_backward_reduced_element_by_element(terms):
    check_mlp_backward_reduced(terms)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("terms", [1, 3])
def test_mixing_block_backward_reduced_element_by_element(terms, ways):
    check_mixing_block_backward_reduced(terms, ways)


def test_full_precision_chains_element_by_element():
    # the same hand evaluation with exact products pins the full-precision chains a second time
    X, W1, b1, W2, dY, gamma, beta = mlp_data(540, 5, 6, 4)
    want = mlp_backward_by_hand(X, W1, b1, W2, dY, 0)
    wantb = mixing_block_backward_by_hand(2, X, gamma, beta, W1, b1, W2, dY, 0, 1e-5)
    got = oracle.mlp_backward(X, W1, b1, W2, dY)
    for name in want:
        close(got[name], want[name])
    gotb = oracle.mixing_block_backward(2, X, gamma, beta, W1, b1, W2, dY)
    for name in wantb:
        close(gotb[name], wantb[name], tol=1e-11)


# ---------------------------------------------------------------------------------------------
# the token-mixing half, forward and backward, element by element
# ---------------------------------------------------------------------------------------------
def token_block_by_hand(groups, X, gamma, beta, W1, b1, W2, b2, dY, terms, eps):
    """X [T x C]; W1, W2 [T x D]; b1 [D]; b2 [T]; dY [T x C] (Sec. 3: the MLP runs along the token axis of the
    layer-normed input, per channel; Sec. 5: its first layer contracts over the tokens without a transpose)."""
    T, C, D = len(X), len(X[0]), len(W1[0])
    xhat, rstd, xn = norm_rows(X, gamma, beta, groups, eps)
    Xn32 = [[f32(v) for v in row] for row in xn]
    A = [[float(b1[d]) + sum(product(Xn32[t][c], W1[t][d], terms) for t in range(T)) for d in range(D)] for c in range(C)]
    H = [[gelu_s(A[c][d]) for d in range(D)] for c in range(C)]
    H32 = [[f32(v) for v in row] for row in H]
    Y = [[float(X[t][c]) + sum(product(W2[t][d], H32[c][d], terms) for d in range(D)) + float(b2[t]) for c in range(C)]
         for t in range(T)]
    dW2 = [[sum(product(dY[t][c], H32[c][d], terms) for c in range(C)) for d in range(D)] for t in range(T)]
    dH = [[sum(product(dY[t][c], W2[t][d], terms) for t in range(T)) for d in range(D)] for c in range(C)]
    db2 = [sum(float(dY[t][c]) for c in range(C)) for t in range(T)]
    dA = [[dH[c][d] * gelu_grad_s(A[c][d]) for d in range(D)] for c in range(C)]
    dA32 = [[f32(v) for v in row] for row in dA]
    dXn = [[sum(product(W1[t][d], dA32[c][d], terms) for d in range(D)) for c in range(C)] for t in range(T)]
    dW1 = [[sum(product(Xn32[t][c], dA32[c][d], terms) for c in range(C)) for d in range(D)] for t in range(T)]
    db1 = [sum(dA32[c][d] for c in range(C)) for d in range(D)]
    dXn32 = [[f32(v) for v in row] for row in dXn]
    dXl = norm_rows_backward(xhat, rstd, gamma, dXn32, groups)
    dX = [[float(dY[t][c]) + dXl[t][c] for c in range(C)] for t in range(T)]
    dgamma = [sum(dXn32[t][c] * xhat[t][c] for t in range(T)) for c in range(C)]
    dbeta = [sum(dXn32[t][c] for t in range(T)) for c in range(C)]
    fwd = dict(Xn=xn, H=H, Y=Y)
    bwd = dict(A=A, dH=dH, dA=dA, dXn=dXn, dX=dX, dW1=dW1, db1=db1, dW2=dW2, db2=db2, dgamma=dgamma, dbeta=dbeta)
    return fwd, bwd


def token_data(seed, T, C, D):
    X = (inputs.matrix(seed, T, C, "R") * np.float32(1.7) + np.float32(0.2)).astype(np.float32)
    W1 = inputs.matrix(seed + 1, T, D, "R") * np.float32(0.9)
    W2 = inputs.matrix(seed + 2, T, D, "R") * np.float32(1.1)
    b1 = inputs.matrix(seed + 3, 1, D, "R")[0]
    b2 = inputs.matrix(seed + 4, 1, T, "R")[0]
    dY = inputs.matrix(seed + 5, T, C, "R") * np.float32(1.3)
    gamma = (inputs.matrix(seed + 6, 1, C, "R")[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(seed + 7, 1, C, "R")[0]
    return X, W1, b1, W2, b2, dY, gamma, beta


def check_token_block_reduced(terms, ways):
    X, W1, b1, W2, b2, dY, gamma, beta = token_data(560, 5, 6, 4)
    fwd, bwd = token_block_by_hand(oracle.ln_groups(ways), X, gamma, beta, W1, b1, W2, b2, dY, terms, 1e-5)
    got = oracle.token_mixing_block_reduced(ways, X, gamma, beta, W1, b1, W2, b2, terms)
    for name in fwd:
        close(got[name], fwd[name], tol=1e-11)
    gotb = oracle.token_mixing_block_backward_reduced(ways, X, gamma, beta, W1, b1, W2, dY, terms)
    for name in bwd:
        close(gotb[name], bwd[name], tol=1e-11)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("terms", [1, 3])
def test_token_mixing_block_reduced_element_by_element(terms, ways):
    check_token_block_reduced(terms, ways)


# ---------------------------------------------------------------------------------------------
# planted mistakes: each changes one piece the chains are built from; the element-by-element pins must fail
# ---------------------------------------------------------------------------------------------
def _round_first(fn):
    return lambda a, *rest, **kw: fn(oracle.round_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64), *rest, **kw)


def _truncate(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)


def _unrounded_backward(X, W, dY, terms=1, nthreads=None, absolute=False):
    return oracle.backward(X, W, dY, nthreads, absolute)


def _unrounded_linear(X, W, b=None, terms=1, nthreads=None, absolute=False):
    return (oracle.magnitude if absolute else oracle.linear)(X, W, b, nthreads)


def _rounded_sum(fn):
    return lambda dY, *rest, **kw: fn(oracle.round_bf16(np.asarray(dY, dtype=np.float32)), *rest, **kw)


PLANTS = {
    "pre-activation rounded before GELU": ("gelu", _round_first),
    "GELU derivative taken at the rounded pre-activation": ("gelu_grad", _round_first),
    "backward products on unrounded operands": ("backward_reduced", lambda fn: _unrounded_backward),
    "pre-activation recomputed in full precision": ("linear_reduced", lambda fn: _unrounded_linear),
    "truncation instead of rounding to nearest": ("round_bf16", lambda fn: _truncate),
    "bias gradient from rounded values": ("bias_backward", _rounded_sum),
}


@pytest.mark.parametrize("plant", sorted(PLANTS))
def test_planted_mistakes_are_caught_by_the_mlp_pin(plant, monkeypatch):
    name, make = PLANTS[plant]
    monkeypatch.setattr(oracle, name, make(getattr(oracle, name)))
    with pytest.raises(AssertionError):
        check_mlp_backward_reduced(1)
    with pytest.raises(AssertionError):
        check_mixing_block_backward_reduced(1, 2)


TOKEN_PLANTS = dict(PLANTS)
TOKEN_PLANTS["transposed layer's backward on unrounded operands"] = (
    "backward_xtw_reduced", lambda fn: (lambda X, W, dY, terms=1, nthreads=None, absolute=False:
                                        oracle.backward_xtw(X, W, dY, nthreads, absolute)))
TOKEN_PLANTS["transposed layer's forward on unrounded operands"] = (
    "linear_xtw_reduced", lambda fn: (lambda X, W, b=None, terms=1, nthreads=None, absolute=False:
                                      oracle.linear_xtw(X, W, b, nthreads, absolute)))
del TOKEN_PLANTS["pre-activation recomputed in full precision"]     # (this chain's pre-activation is the transposed layer's)


@pytest.mark.parametrize("plant", sorted(TOKEN_PLANTS))
def test_planted_mistakes_are_caught_by_the_token_pin(plant, monkeypatch):
    name, make = TOKEN_PLANTS[plant]
    monkeypatch.setattr(oracle, name, make(getattr(oracle, name)))
    with pytest.raises(AssertionError):
        check_token_block_reduced(1, 2)


def test_a_rounded_skip_connection_would_show():
    # the skip connection adds dY itself (Sec. 6.1: only operands of products are rounded): with its rounding in
    # dY's place the hand evaluation moves away from the oracle by far more than the pins' tolerance
    X, W1, b1, W2, dY, gamma, beta = mlp_data(500, 5, 6, 4)
    got = oracle.mlp_backward_reduced(X, W1, b1, W2, dY, 1)
    want = mlp_backward_by_hand(X, W1, b1, W2, dY, 1)
    wrong = np.asarray(want["dX"]) - dY.astype(np.float64) + oracle.round_bf16(dY).astype(np.float64)
    assert np.abs(wrong - got["dX"]).max() > 1e-4 > np.abs(np.asarray(want["dX"]) - got["dX"]).max()


# ---------------------------------------------------------------------------------------------
# all-integer operands: every rounding is the identity, GELU is the identity on what it sees
# ---------------------------------------------------------------------------------------------
def balanced_rows(rng, M, C, groups):
    """Rows of +-1 with as many +1 as -1 in every channel block: mean 0, variance 1, so with eps = 0 the
    normalised row is the row itself."""
    n = C // groups
    X = np.empty((M, C), dtype=np.float32)
    for i in range(M):
        for b in range(groups):
            X[i, b * n:(b + 1) * n] = rng.permutation(np.repeat([1.0, -1.0], n // 2))
    return X


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("terms", [1, 3])
def test_integer_channel_mixing_chain(terms, ways):
    rng = np.random.default_rng(600 + ways)
    M, C, Hd = 6, 8, 5
    groups = oracle.ln_groups(ways)
    X = balanced_rows(rng, M, C, groups)
    gamma = rng.integers(1, 3, C).astype(np.float32)
    beta = rng.integers(-1, 2, C).astype(np.float32)
    W1 = rng.integers(0, 2, (Hd, C)).astype(np.float32)
    b1 = np.full(Hd, 40.0, dtype=np.float32)       # pre-activations are integers >= 16: gelu(x) = x, gelu'(x) = 1 in double
    W2 = rng.integers(-1, 2, (C, Hd)).astype(np.float32)
    dY = rng.integers(-2, 3, (M, C)).astype(np.float32)
    i64 = lambda a: a.astype(np.int64)
    Xn = i64(X) * i64(gamma) + i64(beta)
    A = Xn @ i64(W1).T + 40
    assert A.min() >= 16 and A.max() <= 256
    dH = i64(dY) @ i64(W2)
    dW2 = i64(dY).T @ A                              # H = A
    dXn = dH @ i64(W1)                               # dA = dH
    dW1 = dH.T @ Xn
    red = oracle.mixing_block_backward_reduced(ways, X, gamma, beta, W1, b1, W2, dY, terms, eps=0.0)
    full = oracle.mixing_block_backward(ways, X, gamma, beta, W1, b1, W2, dY, eps=0.0)
    for name in ("A", "dH", "dA", "dXn", "dX", "dW1", "db1", "dW2", "db2", "dgamma", "dbeta"):
        assert np.array_equal(red[name], full[name]), name
    for name, want in (("A", A), ("dH", dH), ("dA", dH), ("dXn", dXn), ("dW1", dW1), ("dW2", dW2),
                       ("db1", dH.sum(axis=0)), ("db2", i64(dY).sum(axis=0)), ("dbeta", dXn.sum(axis=0)),
                       ("dgamma", (dXn * i64(X)).sum(axis=0))):
        assert np.array_equal(red[name], want.astype(np.float64)), name
    # the norm's backward on these rows (xhat = x = +-1, rstd = 1, n channels a block), in integers times 1 / n
    n = C // groups
    g = dXn * i64(gamma)
    dXl = np.empty((M, C))
    for b in range(groups):
        sl = slice(b * n, (b + 1) * n)
        dXl[:, sl] = g[:, sl] - g[:, sl].sum(axis=1, keepdims=True) / n \
            - i64(X)[:, sl] * ((g[:, sl] * i64(X)[:, sl]).sum(axis=1, keepdims=True) / n)
    assert np.array_equal(red["dX"], dY + dXl)
    # the MLP alone, with its own skip connection
    m = oracle.mlp_backward_reduced(Xn.astype(np.float32), W1, b1, W2, dY, terms)
    assert np.array_equal(m["dX"], (i64(dY) + dXn).astype(np.float64))
    assert np.array_equal(m["dW1"], dW1.astype(np.float64))


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("terms", [1, 3])
def test_integer_token_mixing_chain(terms, ways):
    rng = np.random.default_rng(620 + ways)
    T, C, D = 6, 8, 5
    groups = oracle.ln_groups(ways)
    X = balanced_rows(rng, T, C, groups)
    gamma = rng.integers(1, 3, C).astype(np.float32)
    beta = rng.integers(-1, 2, C).astype(np.float32)
    W1 = rng.integers(0, 2, (T, D)).astype(np.float32)
    b1 = np.full(D, 40.0, dtype=np.float32)
    W2 = rng.integers(-1, 2, (T, D)).astype(np.float32)
    b2 = rng.integers(-3, 4, T).astype(np.float32)
    dY = rng.integers(-2, 3, (T, C)).astype(np.float32)
    i64 = lambda a: a.astype(np.int64)
    Xn = i64(X) * i64(gamma) + i64(beta)
    A = Xn.T @ i64(W1) + 40                          # C x D
    assert A.min() >= 16 and A.max() <= 256
    Y = i64(X) + i64(W2) @ A.T + i64(b2)[:, None]
    dW2 = i64(dY) @ A                                # T x D
    dH = i64(dY).T @ i64(W2)                         # C x D
    dXn = i64(W1) @ dH.T                             # T x C
    dW1 = Xn @ dH                                    # T x D
    fr = oracle.token_mixing_block_reduced(ways, X, gamma, beta, W1, b1, W2, b2, terms, eps=0.0)
    ff = oracle.token_mixing_block(ways, X, gamma, beta, W1, b1, W2, b2, eps=0.0)
    for name in ("H", "Y", "Xn"):
        assert np.array_equal(fr[name], ff[name]), name
    assert np.array_equal(fr["H"], A.astype(np.float64)) and np.array_equal(fr["Y"], Y.astype(np.float64))
    red = oracle.token_mixing_block_backward_reduced(ways, X, gamma, beta, W1, b1, W2, dY, terms, eps=0.0)
    full = oracle.token_mixing_block_backward(ways, X, gamma, beta, W1, b1, W2, dY, eps=0.0)
    for name in ("A", "dH", "dA", "dXn", "dX", "dW1", "db1", "dW2", "db2", "dgamma", "dbeta"):
        assert np.array_equal(red[name], full[name]), name
    for name, want in (("A", A), ("dH", dH), ("dA", dH), ("dXn", dXn), ("dW1", dW1), ("dW2", dW2),
                       ("db1", dH.sum(axis=0)), ("db2", i64(dY).sum(axis=1)), ("dbeta", dXn.sum(axis=0)),
                       ("dgamma", (dXn * i64(X)).sum(axis=0))):
        assert np.array_equal(red[name], want.astype(np.float64)), name
    assert dW2.shape == (T, D) and dH.shape == (C, D)


# ---------------------------------------------------------------------------------------------
# the partition every matrix of the method uses
# ---------------------------------------------------------------------------------------------
def test_shard_blocks_literal():
    A = np.arange(24, dtype=np.float32).reshape(4, 6)
    one = oracle.shard_blocks(A, 1)
    assert len(one) == 1 and np.array_equal(one[0], A)
    two = oracle.shard_blocks(A, 2)
    assert np.array_equal(two[0], [[0, 1, 2], [6, 7, 8], [12, 13, 14], [18, 19, 20]])
    assert np.array_equal(two[1], [[3, 4, 5], [9, 10, 11], [15, 16, 17], [21, 22, 23]])
    four = oracle.shard_blocks(A, 4)
    assert np.array_equal(four[0], [[0, 1, 2], [6, 7, 8]])            # block (0, 0) on rank 0
    assert np.array_equal(four[1], [[3, 4, 5], [9, 10, 11]])          # block (0, 1) on rank 1
    assert np.array_equal(four[2], [[12, 13, 14], [18, 19, 20]])      # block (1, 0) on rank 2
    assert np.array_equal(four[3], [[15, 16, 17], [21, 22, 23]])      # block (1, 1) on rank 3
    for s in one + two + four:
        assert s.flags["C_CONTIGUOUS"]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("R,Cc", [(2, 2), (6, 10), (14, 4)])
def test_shard_blocks_is_the_partition_of_every_tensor(ways, R, Cc):
    A = inputs.matrix(700 + ways, R, Cc, "R")
    blocks = oracle.shard_blocks(A, ways)
    # the same partition as the activations', the weights' and the outputs' (Sec. 4.1 / 4.2: all split alike)
    for other in (oracle.shard_x(A, ways), oracle.shard_w(A, ways), oracle.shard_y(A, ways)):
        assert len(other) == len(blocks) and all(np.array_equal(a, b) for a, b in zip(other, blocks))
    # zero redundancy (Sec. 4): the blocks hold every element exactly once, and gathering them gives the matrix back
    ids = np.arange(R * Cc, dtype=np.float32).reshape(R, Cc)
    held = np.concatenate([b.ravel() for b in oracle.shard_blocks(ids, ways)])
    assert held.size == R * Cc and np.array_equal(np.sort(held), ids.ravel())
    assert np.array_equal(oracle.gather_y(blocks, ways), A)
    assert sum(b.nbytes for b in blocks) == A.nbytes


def test_shard_blocks_rejects_what_does_not_split():
    A = np.zeros((3, 5), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.shard_blocks(A, 2)
    with pytest.raises(ValueError):
        oracle.shard_blocks(np.zeros((3, 4), dtype=np.float32), 4)
    with pytest.raises(ValueError):
        oracle.shard_blocks(A, 3)
