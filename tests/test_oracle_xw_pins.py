"""Pins for the oracle of the third permutation of the layer, Y = X W with the weights stored K x N (no GPU).

Sec. 5 names three permutations (X W^T, X W, X^T W) without equations for the last two.  The definition is
pinned by integer brute force in exact arithmetic, by closed forms, by the pinned X W^T oracle on explicitly
transposed weights and by a library product in double; the block-wise routine by the definition (exactly on
lattice values), by block-constant operands evaluated by hand, and by which rank's blocks a term needs;
the gradients by the adjoint identities and the library's autograd in double.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2507_05753_amd import inputs


def data(seed, M, K, N, mode="R", bias=True):
    X = inputs.matrix(seed, M, K, mode)
    W = inputs.matrix(seed + 1000, K, N, mode, inputs.W_SCALE_EXP)
    b = inputs.matrix(seed + 2000, 1, N, mode)[0] if bias else None
    return X, W, b


@pytest.mark.parametrize("M,K,N", list(itertools.product((2, 4, 6), repeat=3)))
def test_integer_brute_force(M, K, N):
    rng = np.random.default_rng(M * 100 + K * 10 + N)
    X = rng.integers(-3, 4, (M, K))
    W = rng.integers(-3, 4, (K, N))
    b = rng.integers(-3, 4, N)
    want = [[int(b[j]) + sum(int(X[i][k]) * int(W[k][j]) for k in range(K)) for j in range(N)] for i in range(M)]
    Xf, Wf, bf = X.astype(np.float32), W.astype(np.float32), b.astype(np.float32)
    assert np.array_equal(oracle.linear_xw(Xf, Wf, bf), np.array(want, dtype=np.float64))
    for ways in (1, 2, 4):
        assert np.array_equal(oracle.jigsaw_xw(ways, Xf, Wf, bf), np.array(want, dtype=np.float64)), ways
    mag = [[abs(int(b[j])) + sum(abs(int(X[i][k]) * int(W[k][j])) for k in range(K)) for j in range(N)] for i in range(M)]
    assert np.array_equal(oracle.magnitude_xw(Xf, Wf, bf), np.array(mag, dtype=np.float64))


def test_is_the_plain_layer_on_transposed_weights():
    X, W, b = data(11, 9, 14, 6)
    # the same sums in the same order (k ascending): identical bits
    assert np.array_equal(oracle.linear_xw(X, W, b), oracle.linear(X, np.ascontiguousarray(W.T), b))
    assert np.array_equal(oracle.magnitude_xw(X, W, b), oracle.magnitude(X, np.ascontiguousarray(W.T), b))
    # and a library product in double
    ref = X.astype(np.float64) @ W.astype(np.float64) + b
    assert np.all(np.abs(oracle.linear_xw(X, W, b) - ref) <= 1e-14 * oracle.magnitude_xw(X, W, b))


def test_orientation_closed_forms():
    M, K = 5, 8
    X = inputs.matrix(12, M, K, "R")
    assert np.array_equal(oracle.linear_xw(X, np.eye(K, dtype=np.float32)), X.astype(np.float64))
    # a single weight W[k0][j0] = 1 moves column k0 of X into column j0 of Y: X W, not X W^T
    N = 8
    W = np.zeros((K, N), dtype=np.float32)
    W[2, 5] = 1.0
    Y = oracle.linear_xw(X, W)
    assert np.array_equal(Y[:, 5], X[:, 2].astype(np.float64)) and np.count_nonzero(Y[:, [0, 1, 2, 3, 4, 6, 7]]) == 0
    # X = e_i e_k^T picks row k of W into row i of Y
    Wg = inputs.matrix(13, K, N, "R")
    E = np.zeros((M, K), dtype=np.float32)
    E[3, 6] = 1.0
    Y = oracle.linear_xw(E, Wg)
    assert np.array_equal(Y[3], Wg[6].astype(np.float64)) and np.count_nonzero(np.delete(Y, 3, axis=0)) == 0
    # the shapes tell W from W^T when K != N
    assert oracle.linear_xw(X, inputs.matrix(14, K, 3, "R")).shape == (M, 3)
    # a square, unsymmetric W: the transposed product is another matrix
    Ws = inputs.matrix(15, K, K, "R")
    assert not np.array_equal(oracle.linear_xw(X, Ws), oracle.linear_xw(X, np.ascontiguousarray(Ws.T)))


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", [(6, 10, 8), (14, 4, 6), (2, 2, 2), (50, 34, 22)])
def test_block_wise_equals_the_definition(ways, M, K, N):
    X, W, b = data(20 + ways, M, K, N, "L")
    assert np.array_equal(oracle.jigsaw_xw(ways, X, W, b), oracle.linear_xw(X, W, b))     # lattice values: exact sums
    X, W, b = data(30 + ways, M, K, N, "R")
    S = oracle.magnitude_xw(X, W, b)
    assert np.all(np.abs(oracle.jigsaw_xw(ways, X, W, b) - oracle.linear_xw(X, W, b)) <= 1e-12 * S)


@pytest.mark.parametrize("ways", [2, 4])
def test_block_constant_operands_by_hand(ways):
    # X block (i, k) = x[i][k] everywhere, W block (k, c) = w[k][c]: Y block (i, c) = Kh * sum_k x[i][k] w[k][c] + b
    M, K, N = 4, 6, 8
    Kh = K // 2
    x = [[1.0, 2.0], [-3.0, 0.5]]
    w = [[0.25, -1.0], [2.0, 4.0]]
    bh = [0.5, -2.0]
    rows = 2 if ways == 4 else 1
    X = np.empty((M, K), dtype=np.float32)
    for i in range(M):
        for k in range(K):
            X[i, k] = x[(i * rows) // M][k // Kh]
    W = np.empty((K, N), dtype=np.float32)
    for k in range(K):
        for c in range(N):
            W[k, c] = w[k // Kh][c // (N // 2)]
    b = np.array([bh[c // (N // 2)] for c in range(N)], dtype=np.float32)
    Y = oracle.jigsaw_xw(ways, X, W, b)
    for i in range(M):
        for c in range(N):
            ib, cb = (i * rows) // M, c // (N // 2)
            assert Y[i, c] == Kh * (x[ib][0] * w[0][cb] + x[ib][1] * w[1][cb]) + bh[cb]


@pytest.mark.parametrize("ways", [2, 4])
def test_each_output_block_reads_the_blocks_the_decomposition_names(ways):
    # Y_(i,j) = X_(i,j) W_(j,j) + X_(i,1-j) W_(1-j,j): poisoning any other block must not change it
    M, K, N = 4, 4, 4
    X, W, _ = data(40, M, K, N, "L", bias=False)
    base = oracle.jigsaw_xw(ways, X, W)
    rows = 2 if ways == 4 else 1
    Mb = M // rows
    for i in range(rows):
        for j in range(2):
            Xp, Wp = X.copy(), W.copy()
            for ii in range(rows):            # every activation block of another row half
                if ii != i:
                    Xp[ii * Mb:(ii + 1) * Mb, :] = 77.0
            Wp[:, (1 - j) * 2:(2 - j) * 2] = 55.0            # the weight blocks of the other column half
            got = oracle.jigsaw_xw(ways, Xp, Wp)
            assert np.array_equal(got[i * Mb:(i + 1) * Mb, j * 2:(j + 1) * 2], base[i * Mb:(i + 1) * Mb, j * 2:(j + 1) * 2])


def test_zero_padding_and_linearity():
    X, W, b = data(50, 7, 9, 5, "L")
    Y = oracle.linear_xw(X, W, b)
    Xp = np.zeros((8, 10), dtype=np.float32); Xp[:7, :9] = X
    Wp = np.zeros((10, 6), dtype=np.float32); Wp[:9, :5] = W
    bp = np.zeros(6, dtype=np.float32); bp[:5] = b
    for ways in (2, 4):
        assert np.array_equal(oracle.jigsaw_xw(ways, Xp, Wp, bp)[:7, :5], Y)
    X2 = inputs.matrix(51, 7, 9, "L")
    lhs = oracle.linear_xw((np.float32(2.0) * X + X2).astype(np.float32), W)
    assert np.array_equal(lhs, 2.0 * oracle.linear_xw(X, W) + oracle.linear_xw(X2, W))


def test_gradients():
    M, K, N = 6, 10, 4
    X, W, _ = data(60, M, K, N, "L", bias=False)
    G = inputs.matrix(61, M, N, "L")
    dX, dW = oracle.backward_xw(X, W, G)
    assert dX.shape == (M, K) and dW.shape == (K, N)
    # adjoint identities, exact on lattice values: <dY, X W> = <dX, X> = <dW, W>
    lhs = np.sum(G.astype(np.float64) * oracle.linear_xw(X, W))
    assert lhs == np.sum(dX * X) == np.sum(dW * W)
    # integers written out
    want_dX = [[sum(float(G[i][j]) * float(W[k][j]) for j in range(N)) for k in range(K)] for i in range(M)]
    want_dW = [[sum(float(X[i][k]) * float(G[i][j]) for i in range(M)) for j in range(N)] for k in range(K)]
    assert np.array_equal(dX, np.array(want_dX)) and np.array_equal(dW, np.array(want_dW))
    # the library's autograd in double on general values
    X, W, _ = data(62, M, K, N, "R", bias=False)
    G = inputs.matrix(63, M, N, "R")
    tx = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    tw = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    (tx @ tw).backward(torch.tensor(G, dtype=torch.float64))
    dX, dW = oracle.backward_xw(X, W, G)
    sX, sW = oracle.backward_xw(X, W, G, absolute=True)
    assert np.all(np.abs(dX - tx.grad.numpy()) <= 1e-14 * sX) and np.all(np.abs(dW - tw.grad.numpy()) <= 1e-14 * sW)


def test_argument_checks():
    X, W, b = data(70, 4, 6, 8)
    with pytest.raises(RuntimeError):
        oracle.jigsaw_xw(3, X, W, b)
    with pytest.raises(RuntimeError):
        oracle.jigsaw_xw(2, X[:, :5], W[:5], b)          # odd K
    with pytest.raises(RuntimeError):
        oracle.jigsaw_xw(4, X[:3], W, b)                  # odd M
