"""Pins for the CPU oracle (no GPU, no HIP code).

The paper prints no worked numeric example of a Jigsaw product, so the oracle is
pinned by what the paper and the mathematics fix:

* closed forms (identity, permutation, all-ones, single-nonzero operands);
* exact integer brute force on tiny shapes, via the outer-product formulation
  (sum over k of column_k(X) (x) column_k(W)) in Python integers;
* a library matmul in double on rectangular shapes;
* the block identities of Eq. (2) (2-way) and Eq. (4) (4-way), both against the
  plain product and against the scalar form of those equations on
  block-constant operands (catches a mis-routed partial product);
* linearity, zero-padding invariance, and a cancellation case that only
  double-precision accumulation gets right.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
from paper_2507_05753_amd import inputs


def rng_ints(seed, shape, lo=-3, hi=3):
    k = inputs.keys(seed, np.arange(int(np.prod(shape)), dtype=np.uint64))
    return ((k >> np.uint64(33)) % np.uint64(hi - lo + 1)).astype(np.int64).reshape(shape) + lo


# --------------------------------------------------------------------------
# closed forms
# --------------------------------------------------------------------------
def test_identity_weight_returns_x_bit_exact():
    X = inputs.matrix(11, 7, 6, "R")
    Y = oracle.linear(X, np.eye(6, dtype=np.float32))
    assert np.array_equal(Y, X.astype(np.float64))
    for ways in (2, 4):
        Xe = inputs.matrix(11, 8, 6, "R")
        assert np.array_equal(oracle.jigsaw(ways, Xe, np.eye(6, dtype=np.float32)), Xe.astype(np.float64))


def test_permutation_weight_permutes_columns():
    K = 8
    perm = np.array([3, 0, 7, 1, 6, 2, 5, 4])
    W = np.zeros((K, K), dtype=np.float32)
    W[np.arange(K), perm] = 1.0  # Y[:, j] = X[:, perm[j]]
    X = inputs.matrix(12, 6, K, "R")
    for ways in (1, 2, 4):
        assert np.array_equal(oracle.jigsaw(ways, X, W), X[:, perm].astype(np.float64))


def test_all_ones_weight_gives_row_sums():
    X = inputs.matrix(13, 10, 12, "R")
    W = np.ones((4, 12), dtype=np.float32)
    want = np.array([math.fsum(float(v) for v in row) for row in X])
    for ways in (1, 2, 4):
        Y = oracle.jigsaw(ways, X, W)
        assert np.allclose(Y, want[:, None], rtol=0, atol=1e-14)


def test_single_nonzero_x_selects_a_weight_column():
    M, K, N = 6, 10, 8
    W = inputs.matrix(14, N, K, "R", -6)
    for (i, k) in [(0, 0), (2, 4), (3, 5), (5, 9)]:
        X = np.zeros((M, K), dtype=np.float32)
        X[i, k] = 0.5
        want = np.zeros((M, N))
        want[i, :] = 0.5 * W[:, k].astype(np.float64)  # W^T, not W: row k of W^T is column k of W
        for ways in (1, 2, 4):
            assert np.array_equal(oracle.jigsaw(ways, X, W), want)


def test_bias_is_added_once_with_its_sign():
    X = np.zeros((4, 6), dtype=np.float32)
    W = inputs.matrix(15, 8, 6, "R")
    b = np.arange(8, dtype=np.float32) - 3.5
    for ways in (1, 2, 4):
        assert np.array_equal(oracle.jigsaw(ways, X, W, b), np.tile(b.astype(np.float64), (4, 1)))
    assert np.array_equal(oracle.linear(X, W, b), np.tile(b.astype(np.float64), (4, 1)))


# --------------------------------------------------------------------------
# exact integer brute force on tiny shapes
# --------------------------------------------------------------------------
def outer_product_form(X, W, b):
    M, K = X.shape
    N = W.shape[0]
    Y = [[int(b[j]) for j in range(N)] for _ in range(M)]
    for k in range(K):
        xc = [int(X[i, k]) for i in range(M)]
        wc = [int(W[j, k]) for j in range(N)]
        for i in range(M):
            for j in range(N):
                Y[i][j] += xc[i] * wc[j]
    return np.array(Y, dtype=np.int64)


@pytest.mark.parametrize("M,K,N", list(itertools.product((2, 4, 6), repeat=3)))
def test_integer_brute_force_all_small_shapes(M, K, N):
    seed = 100 + 36 * M + 6 * K + N
    X = rng_ints(seed, (M, K))
    W = rng_ints(seed + 1, (N, K))
    b = rng_ints(seed + 2, (N,))
    want = outer_product_form(X, W, b)
    Xf, Wf, bf = X.astype(np.float32), W.astype(np.float32), b.astype(np.float32)
    assert np.array_equal(oracle.linear(Xf, Wf, bf), want.astype(np.float64))
    for ways in (1, 2, 4):
        assert np.array_equal(oracle.jigsaw(ways, Xf, Wf, bf), want.astype(np.float64))


# --------------------------------------------------------------------------
# a library routine, rectangular shapes
# --------------------------------------------------------------------------
@pytest.mark.parametrize("M,K,N", [(5, 7, 3), (33, 130, 18), (64, 50, 100), (1, 257, 2)])
def test_matches_library_matmul_in_double(M, K, N):
    X, W, b = inputs.layer_inputs(21, M, K, N, "R", bias=True)
    Y = oracle.linear(X, W, b, nthreads=3)
    ref = X.astype(np.float64) @ W.astype(np.float64).T + b.astype(np.float64)
    S = oracle.magnitude(X, W, b)
    assert np.all(np.abs(Y - ref) <= 1e-13 * S)
    Sref = np.abs(X.astype(np.float64)) @ np.abs(W.astype(np.float64)).T + np.abs(b.astype(np.float64))
    assert np.allclose(S, Sref, rtol=1e-13, atol=0)


def test_thread_count_does_not_change_bits():
    X, W, b = inputs.layer_inputs(22, 37, 64, 20, "R", bias=True)
    Y1 = oracle.linear(X, W, b, nthreads=1)
    for t in (2, 5, 64):
        assert np.array_equal(oracle.linear(X, W, b, nthreads=t), Y1)


# --------------------------------------------------------------------------
# block identities, Eq. (2) and Eq. (4)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("ways", [2, 4])
@pytest.mark.parametrize("M,K,N", [(100, 100, 100), (6, 10, 14), (50, 18, 2), (2, 2, 2)])
def test_block_identity_against_plain_product(ways, M, K, N):
    X, W, b = inputs.layer_inputs(31, M, K, N, "R", bias=True)
    Y = oracle.linear(X, W, b)
    S = oracle.magnitude(X, W, b)
    assert np.all(np.abs(oracle.jigsaw(ways, X, W, b) - Y) <= 1e-12 * S)
    XL, WL, bL = inputs.layer_inputs(32, M, K, N, "L", bias=True)
    assert np.array_equal(oracle.jigsaw(ways, XL, WL, bL), oracle.linear(XL, WL, bL))


def test_eq2_scalar_form_on_block_constant_operands():
    # X = [X_0, X_1], W_r split by rows into W_{r,0}, W_{r,1}; every block constant.
    M, Kh, Nh = 4, 3, 5
    a = [2.0, -3.0]                       # X_r = a[r]
    c = [[5.0, 7.0], [11.0, -13.0]]       # W_{r,q} = c[r][q]
    X = np.concatenate([np.full((M, Kh), a[r], np.float32) for r in range(2)], axis=1)
    W = np.concatenate([np.concatenate([np.full((Nh, Kh), c[r][q], np.float32) for q in range(2)], axis=0)
                        for r in range(2)], axis=1)
    Y = oracle.jigsaw(2, X, W)
    for q in range(2):  # output column-half q = X_0 W_{0,q}^T + X_1 W_{1,q}^T
        want = Kh * (a[0] * c[0][q] + a[1] * c[1][q])
        assert np.all(Y[:, q * Nh:(q + 1) * Nh] == want)


def test_eq4_scalar_form_on_block_constant_operands():
    Mh, Kh, Nh = 3, 4, 5
    a = [2.0, -3.0, 5.0, 7.0]
    c = [11.0, 13.0, -17.0, 19.0]
    blk = lambda v, r, cdim: np.full((r, cdim), v, np.float32)
    X = np.block([[blk(a[0], Mh, Kh), blk(a[1], Mh, Kh)], [blk(a[2], Mh, Kh), blk(a[3], Mh, Kh)]])
    W = np.block([[blk(c[0], Nh, Kh), blk(c[1], Nh, Kh)], [blk(c[2], Nh, Kh), blk(c[3], Nh, Kh)]])
    Y = oracle.jigsaw(4, X, W)
    want = [Kh * (a[0] * c[0] + a[1] * c[1]), Kh * (a[0] * c[2] + a[1] * c[3]),
            Kh * (a[2] * c[0] + a[3] * c[1]), Kh * (a[2] * c[2] + a[3] * c[3])]
    got = oracle.shard_y(Y, 4)
    for r in range(4):
        assert got[r].shape == (Mh, Nh)
        assert np.all(got[r] == want[r]), r


def test_rejects_odd_splits():
    X = np.zeros((3, 4), np.float32)
    W = np.zeros((4, 4), np.float32)
    with pytest.raises(RuntimeError):
        oracle.jigsaw(4, X, W)            # odd M
    with pytest.raises(RuntimeError):
        oracle.jigsaw(2, np.zeros((2, 3), np.float32), np.zeros((4, 3), np.float32))  # odd K
    with pytest.raises(RuntimeError):
        oracle.jigsaw(3, X, W)


# --------------------------------------------------------------------------
# invariants
# --------------------------------------------------------------------------
def test_linearity_exact_on_lattice_inputs():
    M, K, N = 10, 24, 12
    X1 = inputs.matrix(41, M, K, "L")
    X2 = inputs.matrix(42, M, K, "L")
    W = inputs.matrix(43, N, K, "L", -6)
    for ways in (1, 2, 4):
        lhs = oracle.jigsaw(ways, (4.0 * X1 + X2).astype(np.float32), W)
        rhs = 4.0 * oracle.jigsaw(ways, X1, W) + oracle.jigsaw(ways, X2, W)
        assert np.array_equal(lhs, rhs)


def test_zero_padding_k_and_n_reproduces_unpadded_result():
    M, K, N = 6, 9, 7
    X, W, b = inputs.layer_inputs(51, M, K, N, "R", bias=True)
    Xp = np.zeros((M, K + 1), np.float32); Xp[:, :K] = X
    Wp = np.zeros((N + 1, K + 1), np.float32); Wp[:N, :K] = W
    bp = np.zeros(N + 1, np.float32); bp[:N] = b
    Y = oracle.linear(X, W, b)
    for ways in (1, 2, 4):
        assert np.array_equal(oracle.jigsaw(ways, Xp, Wp, bp)[:, :N], Y)


def test_cancellation_needs_double_accumulation():
    X = np.array([[1e8, 1.0, -1e8]], dtype=np.float32)
    W = np.ones((2, 3), dtype=np.float32)
    assert np.array_equal(oracle.linear(X, W), np.array([[1.0, 1.0]]))


def test_magnitude_properties():
    X, W, b = inputs.layer_inputs(61, 9, 40, 11, "R", bias=True)
    S = oracle.magnitude(X, W, b)
    assert np.all(S >= np.abs(oracle.linear(X, W, b)))
    assert np.array_equal(oracle.magnitude(np.abs(X), np.abs(W), np.abs(b)), S)
    assert np.array_equal(oracle.linear(np.abs(X), np.abs(W), np.abs(b)), S)


def test_entries_and_row_ranges_follow_the_full_result():
    M, K, N = 23, 31, 17
    X, W, b = inputs.layer_inputs(71, M, K, N, "R", bias=True)
    Y = oracle.linear(X, W, b)
    S = oracle.magnitude(X, W, b)
    ii = np.array([0, 5, 22, 22, 7])
    jj = np.array([16, 0, 3, 16, 7])
    v, s = oracle.entries(X, W, ii, jj, b[jj])
    assert np.array_equal(v, Y[ii, jj])
    assert np.allclose(s, S[ii, jj], rtol=1e-14, atol=0)
    assert np.array_equal(oracle.linear_rows(X, W, b, 4, 19), Y[4:19])
    assert oracle.linear_rows(X, W, b, 5, 5).shape == (0, N)


# --------------------------------------------------------------------------
# layout definitions
# --------------------------------------------------------------------------
@pytest.mark.parametrize("ways", [1, 2, 4])
def test_shards_tile_the_matrices_without_redundancy(ways):
    M, K, N = 6, 8, 10
    X = np.arange(M * K, dtype=np.float32).reshape(M, K)
    W = np.arange(N * K, dtype=np.float32).reshape(N, K) + 1000
    Y = np.arange(M * N, dtype=np.float64).reshape(M, N)
    xs, ws, ys = oracle.shard_x(X, ways), oracle.shard_w(W, ways), oracle.shard_y(Y, ways)
    assert sum(s.size for s in xs) == X.size
    assert sum(s.size for s in ws) == W.size
    assert sum(s.size for s in ys) == Y.size
    assert sorted(np.concatenate([s.ravel() for s in xs]).tolist()) == X.ravel().tolist()
    assert sorted(np.concatenate([s.ravel() for s in ws]).tolist()) == W.ravel().tolist()
    assert np.array_equal(oracle.gather_y(ys, ways), Y)
    if ways == 2:
        assert xs[1][0, 0] == X[0, K // 2] and ws[1][0, 0] == W[0, K // 2] and ys[1][0, 0] == Y[0, N // 2]
    if ways == 4:
        assert xs[1][0, 0] == X[0, K // 2] and xs[2][0, 0] == X[M // 2, 0]
        assert ws[1][0, 0] == W[0, K // 2] and ws[2][0, 0] == W[N // 2, 0]
        assert ys[1][0, 0] == Y[0, N // 2] and ys[2][0, 0] == Y[M // 2, 0]
    b = np.arange(N, dtype=np.float32)
    bs = oracle.shard_b(b, ways)
    for r in range(ways):
        assert bs[r].shape[0] == ys[r].shape[1]
        j0 = 0 if ways == 1 else (r % 2) * (N // 2)
        assert bs[r][0] == b[j0]


def test_freivalds_reference_is_the_projected_product():
    M, K, N = 40, 33, 21
    X, W, b = inputs.layer_inputs(81, M, K, N, "R", bias=True)
    v = np.where(inputs.keys(82, np.arange(N, dtype=np.uint64)) >> np.uint64(63), 1.0, -1.0)
    yv, bound = oracle.freivalds_reference(X, W, b, v, chunk_rows=7)
    Y = oracle.linear(X, W, b)
    S = oracle.magnitude(X, W, b)
    assert np.all(np.abs(yv - Y @ v) <= 1e-13 * bound)
    assert np.allclose(bound, S @ np.abs(v), rtol=1e-13, atol=0)
    V = np.stack([v, -v, np.ones(N)], axis=1)
    yV, bV = oracle.freivalds_reference(X, W, b, V)
    assert yV.shape == (M, 3) and np.all(np.abs(yV - Y @ V) <= 1e-13 * bV)
    assert np.allclose(yV[:, 0], yv, rtol=0, atol=1e-13) and np.allclose(bV[:, 0], bound, rtol=1e-13, atol=0)
