"""GPU parity on seeded random shapes and options: the FP32 layer (forward with its combine / hand-off / tail
options and its fused epilogue, backward, the transposed layer) against the CPU oracle.

The fixed shape lists of the other test files are chosen by hand around tile, slab and alignment edges; here the
sizes come from the counter-based generator, so that aligned and unaligned operands (the asynchronous and the
guarded kernel), one-element and multi-tile extents and every option combination meet without a plan behind it.
Sizes are capped so that the oracle's full product stays fast.  The bar is the one of the fixed-shape tests:
1e-6 * S (1.5e-6 * S behind the GELU).
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


def cases(stream, n, cap):
    """(ways, M, K, N, six option bits): even where the partition halves a dimension, M * K * N <= cap."""
    k = inputs.keys(stream, np.arange(10 * n, dtype=np.uint64)).reshape(n, 10)
    out = []
    for row in k:
        ways = (1, 2, 4)[int(row[0] % np.uint64(3))]
        M = 1 + int(row[1] % np.uint64(700))
        K = 1 + int(row[2] % np.uint64(1500))
        N = 1 + int(row[3] % np.uint64(700))
        if int(row[4] % np.uint64(3)) == 0:          # a third of the cases: everything in whole 16-byte chunks
            M, K, N = (M + 7) // 8 * 8, (K + 7) // 8 * 8, (N + 7) // 8 * 8
        while M * K * N > cap:
            K = max(2, K // 2)
        if ways >= 2:
            M, K, N = M + (M & 1), K + (K & 1), N + (N & 1)
        out.append((ways, M, K, N) + tuple(int(row[5 + i] & np.uint64(1)) for i in range(5)))
    return out


@pytest.mark.parametrize("ways,M,K,N,bias,combine,weights,act,res", cases(6100, 40, 1.2e8))
def test_forward(jg, ctx, ways, M, K, N, bias, combine, weights, act, res):
    from paper_2507_05753_amd.layer import JigsawLinear
    X, W, b = inputs.layer_inputs(6200 + M + N, M, K, N, "R", bias=True)
    b = b if bias else None
    R = inputs.matrix(6300 + K, M, N, "R") if res else None
    tail = jg.JG_TAIL_WHOLE if (M + K) & 1 else jg.JG_TAIL_SPLIT
    with JigsawLinear(M, K, N, ways, bias=bool(bias), combine=combine, weights=weights, ctx=ctx, tail=tail) as L:
        if L.ws_bytes:
            L.ws.fill_(0xFF)
        for y in L.y:
            y.fill_(float("nan"))
        L.shard(dev(X), dev(W), dev(b) if bias else None)
        rs = None
        if res:
            rs = [torch.empty_like(y) for y in L.y]
            jg.jg_shard(L.plan, jg.JG_T_Y, dev(R).data_ptr(), N, [t.data_ptr() for t in rs])
        L.forward(residual=rs, activation=jg.JG_ACT_GELU if act else jg.JG_ACT_NONE)
        Y = L.gather().cpu().numpy().astype(np.float64)
    want, S = oracle.linear(X, W, b), oracle.magnitude(X, W, b)
    if act:
        want = oracle.gelu(want)
    if res:
        want, S = want + R, S + np.abs(R)
    err = np.abs(Y - want)
    assert np.all(err <= (1.5e-6 if act else TOL) * S), f"max err/S = {(err / S).max():.3e}"


@pytest.mark.parametrize("ways,M,K,N,b0,b1,b2,b3,b4", cases(6400, 24, 6e7))
def test_backward(jg, ctx, ways, M, K, N, b0, b1, b2, b3, b4):
    from paper_2507_05753_amd.layer import JigsawLinear
    X, W, _ = inputs.layer_inputs(6500 + M + N, M, K, N, "R")
    dY = inputs.matrix(6600 + K, M, N, "R")
    with JigsawLinear(M, K, N, ways, ctx=ctx, tail=jg.JG_TAIL_WHOLE if b0 else jg.JG_TAIL_SPLIT) as L:
        L.alloc_backward()
        if L.bw_ws_bytes:
            L.bw_ws.fill_(0xFF)
        for t in L.dx + L.dw:
            t.fill_(float("nan"))
        L.shard(dev(X), dev(W))
        L.shard_dy(dev(dY))
        L.backward()
        dX, dW = L.gather_dx().cpu().numpy().astype(np.float64), L.gather_dw().cpu().numpy().astype(np.float64)
    dX64, dW64 = oracle.backward(X, W, dY)
    SX, SW = oracle.backward_magnitude(X, W, dY)
    ex, ew = np.abs(dX - dX64), np.abs(dW - dW64)
    assert np.all(ex <= TOL * SX), f"dX max err/S = {(ex / SX).max():.3e}"
    assert np.all(ew <= TOL * SW), f"dW max err/S = {(ew / SW).max():.3e}"


@pytest.mark.parametrize("ways,M,K,N,bias,combine,weights,b3,b4", cases(6700, 24, 6e7))
def test_transposed_layer(jg, ctx, ways, M, K, N, bias, combine, weights, b3, b4):
    from paper_2507_05753_amd.layer import JigsawLinear
    X = inputs.matrix(6800 + M, K, M, "R")
    W = inputs.matrix(6900 + N, K, N, "R", inputs.W_SCALE_EXP)
    b = inputs.matrix(7000 + N, 1, N, "R")[0] if bias else None
    with JigsawLinear(M, K, N, ways, bias=bool(bias), combine=combine, weights=weights, ctx=ctx,
                      op=jg.JG_OP_XTW) as L:
        if L.ws_bytes:
            L.ws.fill_(0xFF)
        for y in L.y:
            y.fill_(float("nan"))
        L.shard(dev(X), dev(W), dev(b) if bias else None)
        L.forward()
        Y = L.gather().cpu().numpy().astype(np.float64)
    want, S = oracle.linear_xtw(X, W, b), oracle.magnitude_xtw(X, W, b)
    err = np.abs(Y - want)
    assert np.all(err <= TOL * S), f"max err/S = {(err / S).max():.3e}"
