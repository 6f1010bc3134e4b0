"""GPU checks at the boundary of the library: a context on a stream that is not the default one, non-finite
values staying in the rows and columns they belong to (the slab loaders clamp rows past an operand's edge and
rely on reads outside a buffer descriptor returning zero - a leak would show here), operands that span many
binades, and plans that outlive their context.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_05753_amd import binding as jg
from paper_2507_05753_amd import inputs
from paper_2507_05753_amd.layer import JigsawLinear

pytestmark = pytest.mark.gpu

TOL = 1e-6


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def poison(t, nbytes):
    if nbytes >= 4:
        t[: nbytes // 4 * 4].view(torch.float32).fill_(float("nan"))


def forward_backward(ctx, X, W, b, dY, ways, op):
    """Shard, forward, backward and gather on the context's stream (the caller has made it current)."""
    M, N = dY.shape
    K = X.shape[0] if op == jg.JG_OP_XTW else X.shape[1]
    with JigsawLinear(M, K, N, ways, bias=True, ctx=ctx, op=op) as L:
        poison(L.ws, L.ws_bytes)
        for y in L.y:
            y.fill_(float("nan"))
        # producer work on the same stream, right in front of the library's calls
        Xd, Wd, bd, Gd = dev(X) * 1.0, dev(W) * 1.0, dev(b) * 1.0, dev(dY) * 1.0
        L.shard(Xd, Wd, bd)
        L.forward()
        Y = L.gather()
        L.shard_dy(Gd)
        poison(L.bw_ws, L.bw_ws_bytes)
        L.backward()
        dX, dW = L.gather_dx(), L.gather_dw()
        db = torch.cat([t.clone() for t in L.bias_backward()])
        out = [t.cpu().numpy() for t in (Y, dX, dW, db)]       # (.cpu() waits for the current stream)
    return out


@pytest.mark.parametrize("op", ["XWT", "XTW", "XW"])
@pytest.mark.parametrize("ways", [1, 2, 4])
def test_a_stream_that_is_not_the_default_one(ways, op):
    opc = getattr(jg, "JG_OP_" + op)
    M, K, N = 264, 392, 136
    X = inputs.matrix(801, *((K, M) if op == "XTW" else (M, K)), "R")
    W = inputs.matrix(802, *((N, K) if op == "XWT" else (K, N)), "R", inputs.W_SCALE_EXP)
    b = inputs.matrix(803, 1, N, "R")[0]
    dY = inputs.matrix(804, M, N, "R")
    ctx0 = jg.jg_init(0, torch.cuda.current_stream().cuda_stream)
    want = forward_backward(ctx0, X, W, b, dY, ways, opc)
    jg.jg_free(ctx0)
    side = torch.cuda.Stream()
    assert side.cuda_stream != torch.cuda.current_stream().cuda_stream
    ctx1 = jg.jg_init(0, side.cuda_stream)
    # keep the default stream busy with unrelated work while the side stream runs the layer
    busy = torch.randn(4096, 4096, device="cuda")
    for _ in range(8):
        busy = busy @ busy * 1e-3
    with torch.cuda.stream(side):
        got = forward_backward(ctx1, X, W, b, dY, ways, opc)
    side.synchronize()
    torch.cuda.synchronize()
    jg.jg_free(ctx1)
    for g, w, name in zip(got, want, ("Y", "dX", "dW", "db")):
        assert np.isfinite(g).all(), name
        assert np.array_equal(g, w), f"{name} differs between the streams"


def run_forward(X, W, ways, dtype=jg.JG_F32, op=jg.JG_OP_XWT):
    M, K = X.shape
    N = W.shape[0] if op == jg.JG_OP_XWT else W.shape[1]
    with JigsawLinear(M, K, N, ways, dtype=dtype, op=op) as L:
        poison(L.ws, L.ws_bytes)
        L.shard(dev(X), dev(W))
        L.forward()
        Y = L.gather().cpu().numpy()
    return Y


# M, K, N chosen so that rows, columns and the contraction all end inside a tile and a slab
@pytest.mark.parametrize("dtype", [jg.JG_F32, jg.JG_BF16, jg.JG_BF16X3])
@pytest.mark.parametrize("ways", [1, 2, 4])
def test_a_nan_stays_in_its_row_and_an_inf_in_its_column(ways, dtype):
    M, K, N = 300, 208, 200
    X, W, _ = inputs.layer_inputs(811, M, K, N, "R")
    clean = run_forward(X, W, ways, dtype)
    assert np.isfinite(clean).all()
    # rows: an interior one, the last valid row of an edge tile (4-way: of a rank's block too), the first row
    for i, k in ((17, 5), (M - 1, K - 1), (M // 2 - 1, K // 2), (0, 0)):
        Xn = X.copy()
        Xn[i, k] = np.nan
        Y = run_forward(Xn, W, ways, dtype)
        assert np.isnan(Y[i]).all(), (i, k)
        keep = np.delete(np.arange(M), i)
        assert np.array_equal(Y[keep], clean[keep]), f"NaN in X[{i},{k}] changed another row"
    for j, k in ((3, 7), (N - 1, K - 1), (N // 2, K // 2 - 1)):
        Wn = W.copy()
        Wn[j, k] = np.inf
        Y = run_forward(X, Wn, ways, dtype)
        assert not np.isfinite(Y[:, j]).any(), (j, k)
        keep = np.delete(np.arange(N), j)
        assert np.array_equal(Y[:, keep], clean[:, keep]), f"Inf in W[{j},{k}] changed another column"


@pytest.mark.parametrize("ways", [1, 4])
def test_a_nan_stays_in_its_row_when_weights_are_read_along_their_stride(ways):
    # the X W permutation: the weight block is read along its row stride, rows past K come from outside the descriptor
    M, K, N = 300, 208, 200
    X = inputs.matrix(812, M, K, "R")
    W = inputs.matrix(813, K, N, "R", inputs.W_SCALE_EXP)
    clean = run_forward(X, W, ways, op=jg.JG_OP_XW)
    for i, k in ((M - 1, K - 1), (M // 2, 0)):
        Xn = X.copy()
        Xn[i, k] = np.nan
        Y = run_forward(Xn, W, ways, op=jg.JG_OP_XW)
        keep = np.delete(np.arange(M), i)
        assert np.isnan(Y[i]).all() and np.array_equal(Y[keep], clean[keep])
    Wn = W.copy()
    Wn[K - 1, N - 1] = np.inf
    Y = run_forward(X, Wn, ways, op=jg.JG_OP_XW)
    assert not np.isfinite(Y[:, N - 1]).any() and np.array_equal(Y[:, :N - 1], clean[:, :N - 1])


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_operands_spanning_forty_binades(ways):
    M, K, N = 200, 1000, 136
    X, W, b = inputs.layer_inputs(821, M, K, N, "R", bias=True)
    ex = (inputs.keys(822, np.arange(M * K, dtype=np.uint64)) % np.uint64(41)).astype(np.int64).reshape(M, K) - 20
    ew = (inputs.keys(823, np.arange(N * K, dtype=np.uint64)) % np.uint64(41)).astype(np.int64).reshape(N, K) - 20
    X = np.ldexp(X, ex).astype(np.float32)          # exact: the values keep their 24 bits
    W = np.ldexp(W, ew).astype(np.float32)
    with JigsawLinear(M, K, N, ways, bias=True) as L:
        L.shard(dev(X), dev(W), dev(b))
        L.forward()
        Y = L.gather().cpu().numpy()
        dY = inputs.matrix(824, M, N, "R")
        L.shard_dy(dev(dY))
        L.backward()
        dX, dW = L.gather_dx().cpu().numpy(), L.gather_dw().cpu().numpy()
    S = oracle.magnitude(X, W, b)
    err = np.abs(Y - oracle.linear(X, W, b))
    assert np.all(err <= TOL * S), float((err / S).max())
    wX, wW = oracle.backward(X, W, dY)
    sX, sW = oracle.backward_magnitude(X, W, dY)
    assert np.all(np.abs(dX - wX) <= TOL * sX) and np.all(np.abs(dW - wW) <= TOL * sW)


def test_plans_that_outlive_their_context_answer_queries_only():
    ctx = jg.jg_init(0, torch.cuda.current_stream().cuda_stream)
    plan = jg.jg_plan_create(ctx, 64, 64, 64, 2)
    xw = jg.jg_plan_create(ctx, 64, 64, 64, 4, op=jg.JG_OP_XW)
    gone = jg.jg_plan_create(ctx, 32, 32, 32, 1)
    jg.jg_plan_destroy(gone)
    jg.jg_free(ctx)
    assert jg.jg_plan_query(plan, jg.JG_Q_Y_COLS, 1) == 32
    t = torch.zeros(64 * 64, device="cuda")
    ptrs = [t.data_ptr()] * 4
    ws = torch.zeros(1 << 20, device="cuda")
    for p in (plan, xw):
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_linear_forward(p, ptrs, ptrs, None, ptrs, ws.data_ptr(), ws.numel() * 4)
        assert e.value.status == jg.JG_E_NULL
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_linear_backward(p, ptrs, ptrs, ptrs, ptrs, ptrs, ws.data_ptr(), ws.numel() * 4)
        assert e.value.status == jg.JG_E_NULL
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_shard(p, jg.JG_T_X, t.data_ptr(), 64, ptrs)
        assert e.value.status == jg.JG_E_NULL
        jg.jg_plan_destroy(p)


@pytest.mark.parametrize("ways", [1, 4])
def test_the_forward_can_be_captured_in_a_graph(ways):
    """Callers under HIP graph capture are whom jg_linear_forward_static is for: it allocates nothing, synchronises
    nothing and records no memset.  Captured on a side stream and replayed several times, with eager work and
    synchronisations between the replays; every replay must give the eager run's bits."""
    M, K, N = 1000, 1000, 1000
    X, W, b = inputs.layer_inputs(831, M, K, N, "R", bias=True)
    side = torch.cuda.Stream()
    ctx = jg.jg_init(0, side.cuda_stream)
    try:
        with torch.cuda.stream(side):
            L = JigsawLinear(M, K, N, ways, bias=True, ctx=ctx)
            L.shard(dev(X), dev(W), dev(b))
            L.forward()
            eager = L.gather().cpu().numpy()
        side.synchronize()
        args = ([t.data_ptr() for t in L.x], [t.data_ptr() for t in L.w], [t.data_ptr() for t in L.b],
                [t.data_ptr() for t in L.y])
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            jg.jg_linear_forward_static(L.plan, *args)
        for rep in range(4):
            for y in L.y:
                y.fill_(float("nan"))
            scratch = torch.randn(1 << 20, device="cuda").sum()       # eager work of the program between replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                got = L.gather().cpu().numpy()
            assert np.array_equal(got, eager), f"replay {rep} differs from the eager run"
            assert torch.isfinite(scratch)
        L.close()
    finally:
        jg.jg_free(ctx)
