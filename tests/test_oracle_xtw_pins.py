"""Pins for the oracle of the transposed linear layer Y = X^T W + b (no GPU).

The definition is pinned to the already pinned forward oracle through explicitly transposed
operands ((X^T)(W^T)^T = X^T W), by exact integer brute force on tiny shapes, by closed forms, by a
library matmul in double, and by the adjoint identity with the backward oracle (dW = dY^T X is the
same contraction).  The block-wise routine is pinned by exact equality with the definition on
integer and lattice inputs, by block-constant operands whose blocks can be told apart, and by
planted mistakes (a wrong peer block, a dropped term) that must break that equality.
"""
import itertools

import numpy as np
import pytest

import oracle
from paper_2507_05753_amd import inputs


def rng_ints(seed, shape, lo=-3, hi=3):
    k = inputs.keys(seed, np.arange(int(np.prod(shape)), dtype=np.uint64))
    return ((k >> np.uint64(33)) % np.uint64(hi - lo + 1)).astype(np.int64).reshape(shape) + lo


def operands(seed, T, C, D, mode="R", bias=True):
    X = inputs.matrix(seed, T, C, mode)
    W = inputs.matrix(seed + inputs.W_STREAM, T, D, mode, inputs.W_SCALE_EXP)
    b = inputs.matrix(seed + inputs.B_STREAM, 1, D, mode)[0] if bias else None
    return X, W, b


@pytest.mark.parametrize("T,C,D", [(5, 7, 3), (12, 10, 14), (33, 64, 18), (64, 6, 130)])
def test_equals_the_forward_oracle_on_transposed_operands(T, C, D):
    X, W, b = operands(71, T, C, D, "L")      # lattice values: both orders of summation are exact
    want = oracle.linear(np.ascontiguousarray(X.T), np.ascontiguousarray(W.T), b)
    assert np.array_equal(oracle.linear_xtw(X, W, b), want)
    want_mag = oracle.magnitude(np.ascontiguousarray(X.T), np.ascontiguousarray(W.T), b)
    assert np.array_equal(oracle.magnitude_xtw(X, W, b), want_mag)
    X, W, b = operands(72, T, C, D, "R")      # general values: same terms in the same order
    want = oracle.linear(np.ascontiguousarray(X.T), np.ascontiguousarray(W.T), b)
    assert np.array_equal(oracle.linear_xtw(X, W, b), want)


@pytest.mark.parametrize("T,C,D", list(itertools.product((2, 4, 6), repeat=3)))
def test_integer_brute_force(T, C, D):
    seed = 900 + 36 * T + 6 * C + D
    X, W, b = rng_ints(seed, (T, C)), rng_ints(seed + 1, (T, D)), rng_ints(seed + 2, (D,))
    want = np.array([[int(b[d]) + sum(int(X[t, c]) * int(W[t, d]) for t in range(T)) for d in range(D)]
                     for c in range(C)], dtype=np.float64)
    Xf, Wf, bf = X.astype(np.float32), W.astype(np.float32), b.astype(np.float32)
    assert np.array_equal(oracle.linear_xtw(Xf, Wf, bf), want)
    for ways in (1, 2, 4):
        assert np.array_equal(oracle.jigsaw_xtw(ways, Xf, Wf, bf), want)


def test_closed_forms():
    T, C, D = 8, 8, 6
    X, W, b = operands(73, T, C, D)
    assert np.array_equal(oracle.linear_xtw(np.eye(T, dtype=np.float32), W), W.astype(np.float64))   # X = I: Y = W
    perm = np.array([3, 0, 7, 1, 6, 2, 5, 4])
    P = np.eye(T, dtype=np.float32)[:, perm]       # X^T W picks rows of W: Y[c] = W[perm[c]]
    assert np.array_equal(oracle.linear_xtw(P, W), W[perm].astype(np.float64))
    ones = np.ones((T, C), dtype=np.float32)       # every row of Y is the column sums of W, plus b
    colsum = np.zeros(D)
    for t in range(T):
        colsum += W[t].astype(np.float64)
    assert np.array_equal(oracle.linear_xtw(ones, W, b), np.tile(colsum + b, (C, 1)))
    for (t, c) in [(0, 0), (5, 2), (7, 7)]:        # single non-zero in X: one row of Y is a multiple of W[t]
        E = np.zeros((T, C), dtype=np.float32)
        E[t, c] = 2.0
        want = np.zeros((C, D))
        want[c] = 2.0 * W[t].astype(np.float64)
        assert np.array_equal(oracle.linear_xtw(E, W), want)
    # transposition is really there: a non-square X whose transpose has another shape
    Xr = inputs.matrix(74, 4, 9, "L")
    Wr = inputs.matrix(75, 4, 5, "L")
    assert oracle.linear_xtw(Xr, Wr).shape == (9, 5)


@pytest.mark.parametrize("T,C,D", [(7, 5, 3), (40, 33, 21), (128, 64, 96)])
def test_library_matmul_in_double(T, C, D):
    X, W, b = operands(76, T, C, D)
    want = X.astype(np.float64).T @ W.astype(np.float64) + b.astype(np.float64)
    S = oracle.magnitude_xtw(X, W, b)
    assert np.all(np.abs(oracle.linear_xtw(X, W, b) - want) <= 4 * T * np.finfo(np.float64).eps * S)


def test_same_contraction_as_the_weight_gradient():
    # dW = dY^T X of the layer Y = X W^T is a product of this form: dW = xtw(dY, X)
    M, K, N = 12, 10, 14
    X, Wf, _ = inputs.layer_inputs(77, M, K, N, "L")
    dY = inputs.matrix(78, M, N, "L")
    _, dW = oracle.backward(X, Wf, dY)
    assert np.array_equal(oracle.linear_xtw(dY, X), dW)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("T,C,D", [(6, 4, 2), (10, 12, 14), (34, 18, 66), (64, 130, 12)])
def test_blockwise_equals_definition_exactly_on_lattice_inputs(ways, T, C, D):
    X, W, b = operands(79, T, C, D, "L")
    assert np.array_equal(oracle.jigsaw_xtw(ways, X, W, b), oracle.linear_xtw(X, W, b))
    X, W, _ = operands(80, T, C, D, "L", bias=False)
    assert np.array_equal(oracle.jigsaw_xtw(ways, X, W), oracle.linear_xtw(X, W))


@pytest.mark.parametrize("ways", [2, 4])
def test_blockwise_within_rounding_on_general_inputs(ways):
    T, C, D = 96, 40, 56
    X, W, b = operands(81, T, C, D)
    S = oracle.magnitude_xtw(X, W, b)
    err = np.abs(oracle.jigsaw_xtw(ways, X, W, b) - oracle.linear_xtw(X, W, b))
    assert np.all(err <= 8 * np.finfo(np.float64).eps * S)


def test_block_constant_operands_show_which_blocks_meet():
    # X block (i, j) = x[i][j] everywhere, W block (i, c) = w[i][c]: Y block (a, c) must be
    # (T / 2) * (x[0][a] w[0][c] + x[1][a] w[1][c]): any other pairing of blocks gives another number
    T, C, D = 8, 6, 10
    x = np.array([[1.0, 2.0], [4.0, 8.0]])
    w = np.array([[16.0, 32.0], [64.0, 128.0]])
    X = np.kron(x, np.ones((T // 2, C // 2))).astype(np.float32)
    W = np.kron(w, np.ones((T // 2, D // 2))).astype(np.float32)
    want = np.kron((T // 2) * (x.T @ w), np.ones((C // 2, D // 2)))
    for ways in (1, 2, 4):
        assert np.array_equal(oracle.jigsaw_xtw(ways, X, W), want)


def test_planted_mistakes_are_caught():
    # the checks above would notice a wrong block pairing: emulate two plausible ones in numpy
    T, C, D = 8, 6, 10
    X, W, _ = operands(82, T, C, D, "L", bias=False)
    good = oracle.linear_xtw(X, W)
    Xd, Wd = X.astype(np.float64), W.astype(np.float64)
    Th, Ch, Dh = T // 2, C // 2, D // 2
    # (1) the received term built from the wrong token half of W
    wrong = np.zeros_like(good)
    for a in range(2):
        for c in range(2):
            blk = Xd[:Th, a * Ch:(a + 1) * Ch].T @ Wd[:Th, c * Dh:(c + 1) * Dh] \
                + Xd[Th:, a * Ch:(a + 1) * Ch].T @ Wd[:Th, c * Dh:(c + 1) * Dh]
            wrong[a * Ch:(a + 1) * Ch, c * Dh:(c + 1) * Dh] = blk
    assert not np.array_equal(wrong, good)
    # (2) no transposition of the activation block (possible when the block is square)
    Xs = inputs.matrix(83, 6, 6, "L")
    Ws = inputs.matrix(84, 6, 4, "L")
    assert not np.array_equal(Xs.astype(np.float64) @ Ws.astype(np.float64), oracle.linear_xtw(Xs, Ws))


def test_argument_checks():
    X, W, b = operands(85, 6, 5, 4)
    with pytest.raises(RuntimeError):
        oracle.jigsaw_xtw(2, X, W, b)            # odd number of channels
    X, W, b = operands(85, 5, 6, 4)
    with pytest.raises(RuntimeError):
        oracle.jigsaw_xtw(4, X, W, b)            # odd number of tokens
    with pytest.raises(RuntimeError):
        oracle.jigsaw_xtw(3, X, W, b)
    assert oracle.jigsaw_xtw(2, X, W, b).shape == (6, 4)


# ---- backward of the transposed layer -------------------------------------------------------------------------
@pytest.mark.parametrize("T,C,D", [(2, 3, 4), (5, 7, 3), (6, 4, 9)])
def test_backward_xtw_integer_brute_force(T, C, D):
    X, W, G = rng_ints(81, (T, C)), rng_ints(82, (T, D)), rng_ints(83, (C, D))
    dX = [[sum(int(W[t, d]) * int(G[c, d]) for d in range(D)) for c in range(C)] for t in range(T)]
    dW = [[sum(int(X[t, c]) * int(G[c, d]) for c in range(C)) for d in range(D)] for t in range(T)]
    got = oracle.backward_xtw(X.astype(np.float32), W.astype(np.float32), G.astype(np.float32))
    assert np.array_equal(got[0], np.array(dX, dtype=np.float64))
    assert np.array_equal(got[1], np.array(dW, dtype=np.float64))
    mag = oracle.backward_xtw(X.astype(np.float32), W.astype(np.float32), G.astype(np.float32), absolute=True)
    assert np.array_equal(mag[0], np.abs(W).astype(np.float64) @ np.abs(G).T)
    assert np.array_equal(mag[1], np.abs(X).astype(np.float64) @ np.abs(G))


@pytest.mark.parametrize("T,C,D", [(12, 10, 14), (33, 64, 18)])
def test_backward_xtw_is_the_adjoint_of_the_forward(T, C, D):
    # <dY, X^T W> = <dX, X> = <dW, W>: both gradients are the adjoints of the same bilinear map (lattice values: exact)
    X, W, _ = operands(84, T, C, D, "L", bias=False)
    G = inputs.matrix(85, C, D, "L")
    dX, dW = oracle.backward_xtw(X, W, G)
    lhs = np.sum(G.astype(np.float64) * oracle.linear_xtw(X, W))
    assert lhs == np.sum(dX * X) == np.sum(dW * W)
    # and the library's autograd in double
    import torch
    Xt = torch.from_numpy(X).double().requires_grad_(True)
    Wt = torch.from_numpy(W).double().requires_grad_(True)
    (Xt.T @ Wt).backward(torch.from_numpy(G).double())
    assert np.array_equal(dX, Xt.grad.numpy()) and np.array_equal(dW, Wt.grad.numpy())
    # a transposed operand or a swapped role does not pass
    if C != D:
        with pytest.raises(AssertionError):
            oracle.backward_xtw(X, W, np.ascontiguousarray(G.T))
    wrong = oracle.backward_xtw(W[:, :min(C, D)], X[:, :min(C, D)], G[:min(C, D), :min(C, D)])
    right = oracle.backward_xtw(X[:, :min(C, D)], W[:, :min(C, D)], G[:min(C, D), :min(C, D)])
    assert not np.array_equal(wrong[0], right[0])
