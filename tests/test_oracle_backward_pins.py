"""Pins for the backward-pass oracle (no GPU).

dX = dY W and dW = dY^T X are pinned by the adjoint identities that tie them to the (already
pinned) forward oracle, <dY, f(dX', W)> = <dX, dX'> and <dY, f(X, dW')> = <dW, dW'> with f the
bias-free forward; by exact integer brute force on tiny shapes; by closed forms; by a library
matmul; and the block-wise routine by equality with the definition and by block-constant operands.
"""
import itertools

import numpy as np
import pytest

import oracle
from paper_2507_05753_amd import inputs


def rng_ints(seed, shape, lo=-3, hi=3):
    k = inputs.keys(seed, np.arange(int(np.prod(shape)), dtype=np.uint64))
    return ((k >> np.uint64(33)) % np.uint64(hi - lo + 1)).astype(np.int64).reshape(shape) + lo


def triple(seed, M, K, N, mode="R"):
    X, W, _ = inputs.layer_inputs(seed, M, K, N, mode)
    dY = inputs.matrix(seed + 3000, M, N, "L" if mode == "L" else "R")
    return X, W, dY


@pytest.mark.parametrize("M,K,N", [(5, 7, 3), (12, 10, 14), (33, 64, 18)])
def test_adjoint_identities_with_the_forward_oracle(M, K, N):
    X, W, dY = triple(91, M, K, N, "L")       # lattice values: every inner product below is exact
    dX, dW = oracle.backward(X, W, dY)
    Xp = inputs.matrix(92, M, K, "L")
    Wp = inputs.matrix(93, N, K, "L", -6)
    lhs = np.sum(dY.astype(np.float64) * oracle.linear(Xp, W))
    assert lhs == np.sum(dX * Xp.astype(np.float64))
    lhs = np.sum(dY.astype(np.float64) * oracle.linear(X, Wp))
    assert lhs == np.sum(dW * Wp.astype(np.float64))


@pytest.mark.parametrize("M,K,N", list(itertools.product((2, 4, 6), repeat=3)))
def test_integer_brute_force(M, K, N):
    seed = 500 + 36 * M + 6 * K + N
    X, W, G = rng_ints(seed, (M, K)), rng_ints(seed + 1, (N, K)), rng_ints(seed + 2, (M, N))
    dX = [[sum(int(G[i, j]) * int(W[j, k]) for j in range(N)) for k in range(K)] for i in range(M)]
    dW = [[sum(int(G[i, j]) * int(X[i, k]) for i in range(M)) for k in range(K)] for j in range(N)]
    Xf, Wf, Gf = X.astype(np.float32), W.astype(np.float32), G.astype(np.float32)
    for ways in (1, 2, 4):
        gX, gW = oracle.jigsaw_backward(ways, Xf, Wf, Gf)
        assert np.array_equal(gX, np.array(dX, dtype=np.float64))
        assert np.array_equal(gW, np.array(dW, dtype=np.float64))
    gX, gW = oracle.backward(Xf, Wf, Gf)
    assert np.array_equal(gX, np.array(dX, dtype=np.float64)) and np.array_equal(gW, np.array(dW, dtype=np.float64))


def test_closed_forms():
    M, K, N = 6, 8, 8
    X, W, dY = triple(94, M, K, N)
    dX, _ = oracle.backward(X, np.eye(K, dtype=np.float32), dY)      # W = I: dX = dY
    assert np.array_equal(dX, dY.astype(np.float64))
    for (i, j) in [(0, 0), (2, 5), (5, 7)]:
        E = np.zeros((M, N), np.float32)
        E[i, j] = 2.0
        for ways in (1, 2, 4):
            dX, dW = oracle.jigsaw_backward(ways, X, W, E)
            wantX = np.zeros((M, K)); wantX[i] = 2.0 * W[j].astype(np.float64)
            wantW = np.zeros((N, K)); wantW[j] = 2.0 * X[i].astype(np.float64)
            assert np.array_equal(dX, wantX) and np.array_equal(dW, wantW)


@pytest.mark.parametrize("M,K,N", [(5, 7, 3), (34, 130, 18), (64, 50, 100)])
def test_matches_library_matmul_and_magnitudes(M, K, N):
    X, W, dY = triple(95, M, K, N)
    dX, dW = oracle.backward(X, W, dY, nthreads=3)
    SX, SW = oracle.backward_magnitude(X, W, dY)
    X64, W64, G64 = X.astype(np.float64), W.astype(np.float64), dY.astype(np.float64)
    assert np.all(np.abs(dX - G64 @ W64) <= 1e-13 * SX)
    assert np.all(np.abs(dW - G64.T @ X64) <= 1e-13 * SW)
    assert np.allclose(SX, np.abs(G64) @ np.abs(W64), rtol=1e-13, atol=0)
    assert np.allclose(SW, np.abs(G64).T @ np.abs(X64), rtol=1e-13, atol=0)
    assert np.all(SX >= np.abs(dX)) and np.all(SW >= np.abs(dW))


@pytest.mark.parametrize("ways", [2, 4])
@pytest.mark.parametrize("M,K,N", [(100, 100, 100), (6, 10, 14), (50, 18, 2), (2, 2, 2)])
def test_blockwise_backward_equals_the_definition(ways, M, K, N):
    X, W, dY = triple(96, M, K, N)
    dX, dW = oracle.backward(X, W, dY)
    SX, SW = oracle.backward_magnitude(X, W, dY)
    gX, gW = oracle.jigsaw_backward(ways, X, W, dY)
    assert np.all(np.abs(gX - dX) <= 1e-12 * SX) and np.all(np.abs(gW - dW) <= 1e-12 * SW)
    XL, WL, GL = triple(97, M, K, N, "L")
    dX, dW = oracle.backward(XL, WL, GL)
    gX, gW = oracle.jigsaw_backward(ways, XL, WL, GL)
    assert np.array_equal(gX, dX) and np.array_equal(gW, dW)


def test_blockwise_backward_on_block_constant_operands():
    Mh, Kh, Nh = 3, 4, 5
    x = [2.0, -3.0, 5.0, 7.0]          # X block (i, j) = x[2 i + j]
    w = [11.0, 13.0, -17.0, 19.0]      # W block (c, j) = w[2 c + j]
    g = [1.0, -2.0, 4.0, 8.0]          # dY block (i, c) = g[2 i + c]
    blk = lambda v, r, c: np.full((r, c), v, np.float32)
    X = np.block([[blk(x[0], Mh, Kh), blk(x[1], Mh, Kh)], [blk(x[2], Mh, Kh), blk(x[3], Mh, Kh)]])
    W = np.block([[blk(w[0], Nh, Kh), blk(w[1], Nh, Kh)], [blk(w[2], Nh, Kh), blk(w[3], Nh, Kh)]])
    G = np.block([[blk(g[0], Mh, Nh), blk(g[1], Mh, Nh)], [blk(g[2], Mh, Nh), blk(g[3], Mh, Nh)]])
    dX, dW = oracle.jigsaw_backward(4, X, W, G)
    for i in range(2):
        for j in range(2):   # dX_(i,j) = sum_c dY_(i,c) W_(c,j): each entry sums Nh products per c
            want = Nh * (g[2 * i + 0] * w[0 + j] + g[2 * i + 1] * w[2 + j])
            assert np.all(dX[i * Mh:(i + 1) * Mh, j * Kh:(j + 1) * Kh] == want), (i, j)
    for c in range(2):
        for j in range(2):   # dW_(c,j) = sum_i dY_(i,c)^T X_(i,j)
            want = Mh * (g[0 + c] * x[0 + j] + g[2 + c] * x[2 + j])
            assert np.all(dW[c * Nh:(c + 1) * Nh, j * Kh:(j + 1) * Kh] == want), (c, j)


def test_freivalds_backward_is_the_projected_gradient():
    M, K, N = 40, 33, 21
    X, W, dY = triple(98, M, K, N)
    V = np.where(inputs.keys(99, np.arange(K * 2, dtype=np.uint64)).reshape(K, 2) >> np.uint64(63), 1.0, -1.0)
    dXv, bX, dWv, bW = oracle.freivalds_backward(X, W, dY, V, chunk_rows=7)
    dX, dW = oracle.backward(X, W, dY)
    SX, SW = oracle.backward_magnitude(X, W, dY)
    assert np.all(np.abs(dXv - dX @ V) <= 1e-13 * bX) and np.all(np.abs(dWv - dW @ V) <= 1e-13 * bW)
    assert np.allclose(bX, SX @ np.abs(V), rtol=1e-12) and np.allclose(bW, SW @ np.abs(V), rtol=1e-12)


# ---------------------------------------------------------------------------------------------
# the bias gradient: db[j] = sum_i dY[i][j]
# ---------------------------------------------------------------------------------------------
def test_bias_gradient_is_the_adjoint_of_the_bias_term():
    """b enters the forward as + 1 b^T, so <dY, f(X, W, b + e) - f(X, W, b)> = <db, e> for any e: tied to the
    (already pinned) forward oracle, on lattice values where every step is exact."""
    M, K, N = 7, 6, 5
    X, W, b = inputs.layer_inputs(71, M, K, N, "L", bias=True)
    dY = inputs.matrix(72, M, N, "L")
    e = inputs.matrix(73, 1, N, "L")[0]
    lhs = (dY.astype(np.float64) * (oracle.linear(X, W, b + e) - oracle.linear(X, W, b))).sum()
    assert lhs == (oracle.bias_backward(dY) * e.astype(np.float64)).sum()


def test_bias_gradient_closed_forms_and_brute_force():
    assert np.array_equal(oracle.bias_backward(np.ones((9, 4), np.float32)), np.full(4, 9.0))
    G = np.arange(12, dtype=np.float32).reshape(4, 3)            # columns 0 3 6 9 / 1 4 7 10 / 2 5 8 11
    assert np.array_equal(oracle.bias_backward(G), np.array([18.0, 22.0, 26.0]))
    assert np.array_equal(oracle.bias_backward(G.T.copy()), np.array([3.0, 12.0, 21.0, 30.0]))    # not the row sums of G
    R = inputs.matrix(74, 50, 7, "R")
    want = [sum(float(R[i, j]) for i in range(50)) for j in range(7)]
    assert np.allclose(oracle.bias_backward(R), want, rtol=0, atol=1e-13)
    assert np.array_equal(oracle.bias_backward(R, absolute=True), oracle.bias_backward(np.abs(R)))
    assert oracle.bias_backward(np.zeros((0, 3), np.float32)).tolist() == [0.0, 0.0, 0.0]
    # cancellation that FP32 accumulation would lose: 2^24, 1, -2^24 sums to 1
    C = np.array([[2.0 ** 24], [1.0], [-(2.0 ** 24)]], dtype=np.float32)
    assert oracle.bias_backward(C)[0] == 1.0
