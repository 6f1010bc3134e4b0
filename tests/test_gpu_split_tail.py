"""GPU parity of launches whose last partial round is split into runs of slabs (JG_TAIL_SPLIT).

Few, long tiles make the launcher cut K loops into runs that write scratch tiles, joined by a second
kernel.  Checked: against the oracle (tolerance; lattice inputs bit for bit), against the same plan with
JG_TAIL_WHOLE, run-to-run equality (no atomics anywhere), a ragged last slab inside a run, all three
operand layouts (forward, both backward products, the transposed layer) and grouped launches.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_05753_amd import inputs

pytestmark = pytest.mark.gpu
TOL = 1e-6


@pytest.fixture(scope="module")
def jg():
    from paper_2507_05753_amd import binding
    return binding


@pytest.fixture(scope="module")
def ctx(jg):
    c = jg.jg_init(0, torch.cuda.current_stream().cuda_stream)
    yield c
    torch.cuda.synchronize()
    jg.jg_free(c)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def forward(jg, ctx, X, W, b, ways, tail, op=0):
    from paper_2507_05753_amd.layer import JigsawLinear
    if op == jg.JG_OP_XTW:
        K, M = X.shape
        N = W.shape[1]
    else:
        M, K = X.shape
        N = W.shape[0]
    with JigsawLinear(M, K, N, ways, bias=b is not None, ctx=ctx, op=op, tail=tail) as L:
        split = L.query(jg.JG_Q_TAIL_SCRATCH_BYTES) > 0
        L.ws.fill_(0xFF)
        L.shard(dev(X), dev(W), dev(b) if b is not None else None)
        L.forward()
        Y = L.gather()
        torch.cuda.synchronize()
        return Y.cpu().numpy(), split


# (M, K, N): few tiles, many slabs; K = 4100 leaves a ragged last slab (128 slabs + 4 columns)
SHAPES = [(130, 4160, 258), (258, 4100, 136), (520, 8200, 264)]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_forward(jg, ctx, ways, M, K, N):
    X, W, b = inputs.layer_inputs(31, M, K, N, "R", bias=True)
    Y, split = forward(jg, ctx, X, W, b, ways, jg.JG_TAIL_SPLIT)
    assert split, "the shape is meant to split its tail"
    S = oracle.magnitude(X, W, b)
    err = np.abs(Y.astype(np.float64) - oracle.linear(X, W, b))
    assert np.all(err <= TOL * S), f"max err/S = {(err / S).max():.3e}"
    Y2, _ = forward(jg, ctx, X, W, b, ways, jg.JG_TAIL_SPLIT)
    assert np.array_equal(Y, Y2)                       # the same bits on every run
    Yw, split_w = forward(jg, ctx, X, W, b, ways, jg.JG_TAIL_WHOLE)
    assert not split_w
    assert np.all(np.abs(Yw.astype(np.float64) - Y) <= 2 * TOL * S)
    Xl, Wl, bl = inputs.layer_inputs(32, M, K, N, "L", bias=True)
    Yl, _ = forward(jg, ctx, Xl, Wl, bl, ways, jg.JG_TAIL_SPLIT)
    assert np.array_equal(Yl.astype(np.float64), oracle.linear(Xl, Wl, bl))


# Problems smaller than the chip (less than half a round of tiles): every tile's K loop is cut into short runs so
# that all compute units get work.  1000^3 is the second configuration of the workload table; the others put the
# run boundaries on a ragged last slab (K = 516 = 16 slabs + 4), on runs that span two tiles, and on edge tiles.
SMALL = [(1000, 1000, 1000), (384, 516, 256), (130, 1188, 258), (640, 260, 136)]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", SMALL)
def test_small_problems_fill_the_chip(jg, ctx, ways, M, K, N):
    X, W, b = inputs.layer_inputs(51, M, K, N, "R", bias=True)
    Y, split = forward(jg, ctx, X, W, b, ways, jg.JG_TAIL_SPLIT)
    if (M, K, N) == (1000, 1000, 1000):
        assert split, "64 tiles of 16 or 32 slabs on 256 compute units: meant to be cut into runs"
    S = oracle.magnitude(X, W, b)
    err = np.abs(Y.astype(np.float64) - oracle.linear(X, W, b))
    assert np.all(err <= TOL * S), f"max err/S = {(err / S).max():.3e}"
    Y2, _ = forward(jg, ctx, X, W, b, ways, jg.JG_TAIL_SPLIT)
    assert np.array_equal(Y, Y2)                       # the same bits on every run
    Xl, Wl, bl = inputs.layer_inputs(52, M, K, N, "L", bias=True)
    Yl, _ = forward(jg, ctx, Xl, Wl, bl, ways, jg.JG_TAIL_SPLIT)
    Yw, _ = forward(jg, ctx, Xl, Wl, bl, ways, jg.JG_TAIL_WHOLE)
    assert np.array_equal(Yl, Yw) and np.array_equal(Yl.astype(np.float64), oracle.linear(Xl, Wl, bl))


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("K,M,N", [(4160, 136, 264), (8200, 520, 264)])
def test_transposed_layer(jg, ctx, ways, K, M, N):
    X = inputs.matrix(33, K, M, "R")
    W = inputs.matrix(34, K, N, "R", inputs.W_SCALE_EXP)
    b = inputs.matrix(35, 1, N, "R")[0]
    Y, split = forward(jg, ctx, X, W, b, ways, jg.JG_TAIL_SPLIT, op=jg.JG_OP_XTW)
    assert split
    S = oracle.magnitude_xtw(X, W, b)
    err = np.abs(Y.astype(np.float64) - oracle.linear_xtw(X, W, b))
    assert np.all(err <= TOL * S), f"max err/S = {(err / S).max():.3e}"
    Xl, Wl = inputs.matrix(36, K, M, "L"), inputs.matrix(37, K, N, "L", inputs.W_SCALE_EXP)
    Yl, _ = forward(jg, ctx, Xl, Wl, None, ways, jg.JG_TAIL_SPLIT, op=jg.JG_OP_XTW)
    assert np.array_equal(Yl.astype(np.float64), oracle.linear_xtw(Xl, Wl))


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_backward(jg, ctx, ways):
    # dX = dY W contracts over N, dW = dY^T X over M: make both long, and the outputs few tiles
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K, N = 4160, 264, 4100
    for mode in ("R", "L"):
        X, W, _ = inputs.layer_inputs(38, M, K, N, mode)
        dY = inputs.matrix(39, M, N, mode)
        with JigsawLinear(M, K, N, ways, ctx=ctx) as L:
            L.alloc_backward()
            if ways < 4:     # (the 4-way blocks are short enough for the estimate to keep them whole)
                assert L.query(jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES) > 0
            L.bw_ws.fill_(0xFF)
            L.shard(dev(X), dev(W))
            L.shard_dy(dev(dY))
            L.backward()
            dX, dW = L.gather_dx().cpu().numpy(), L.gather_dw().cpu().numpy()
            L.backward()
            assert np.array_equal(dX, L.gather_dx().cpu().numpy()) and np.array_equal(dW, L.gather_dw().cpu().numpy())
        dX64, dW64 = oracle.backward(X, W, dY)
        if mode == "L":
            assert np.array_equal(dX.astype(np.float64), dX64) and np.array_equal(dW.astype(np.float64), dW64)
        else:
            SX, SW = oracle.backward_magnitude(X, W, dY)
            assert np.all(np.abs(dX - dX64) <= TOL * SX) and np.all(np.abs(dW - dW64) <= TOL * SW)


def test_same_sign_operands_across_runs(jg, ctx):
    # all-positive data, K = 16384: the runs' partial sums and their join stay within the bar
    M, K, N = 136, 16384, 264
    X = np.abs(inputs.matrix(40, M, K, "R"))
    W = np.abs(inputs.matrix(41, N, K, "R"))
    Y, split = forward(jg, ctx, X, W, None, 1, jg.JG_TAIL_SPLIT)
    assert split
    S = oracle.magnitude(X, W)
    err = np.abs(Y.astype(np.float64) - oracle.linear(X, W))
    assert np.all(err <= TOL * S), f"{(err / S).max():.3e}"
