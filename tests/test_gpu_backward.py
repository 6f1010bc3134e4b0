"""GPU parity of the backward pass (dX = dY W, dW = dY^T X) against the CPU oracle, element by
element, through the C ABI.  Same bars as the forward: 1e-6 of the magnitude of what is summed
(|dY| |W| and |dY|^T |X|), bit-exact on lattice inputs."""
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


def triple(seed, M, K, N, mode="R"):
    X, W, _ = inputs.layer_inputs(seed, M, K, N, mode)
    dY = inputs.matrix(seed + 3000, M, N, "L" if mode == "L" else "R")
    return X, W, dY


def run_backward(ctx, X, W, dY, ways):
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K = X.shape
    N = W.shape[0]
    with JigsawLinear(M, K, N, ways, ctx=ctx) as L:
        L.alloc_backward()
        if L.bw_ws_bytes:
            L.bw_ws.fill_(0xFF)                 # NaN pattern: stale workspace contents must not matter
        for t in L.dx + L.dw:
            t.fill_(float("nan"))
        L.shard(dev(X), dev(W))
        L.shard_dy(dev(dY))
        L.backward()
        dX, dW = L.gather_dx(), L.gather_dw()
        torch.cuda.synchronize()
        dy_shards = [t.cpu().numpy() for t in L.dy]
        return dX.cpu().numpy(), dW.cpu().numpy(), dy_shards


SHAPES = [
    (100, 100, 100),     # config 1: halves of 50 are not multiples of 4 (guarded kernels)
    (2, 2, 2),
    (130, 72, 258),      # ragged tiles in every dimension
    (258, 200, 136),
    (64, 520, 640),
    (300, 1032, 260),    # long contraction for dX (N) ... and below for dW (M)
    (2200, 136, 72),
    (1000, 1000, 1000),  # config 2
]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_backward_matches_oracle_within_tolerance(jg, ctx, ways, M, K, N):
    X, W, dY = triple(41, M, K, N)
    dX, dW, dy_sh = run_backward(ctx, X, W, dY, ways)
    for got, want in zip(dy_sh, oracle.shard_y(dY, ways)):     # dY is partitioned like Y
        assert np.array_equal(got, want)
    dX64, dW64 = oracle.backward(X, W, dY)
    SX, SW = oracle.backward_magnitude(X, W, dY)
    ex, ew = np.abs(dX - dX64), np.abs(dW - dW64)
    assert np.all(ex <= TOL * SX), f"dX max err/S = {(ex / SX).max():.3e}"
    assert np.all(ew <= TOL * SW), f"dW max err/S = {(ew / SW).max():.3e}"


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_backward_lattice_inputs_are_bit_exact(jg, ctx, ways, M, K, N):
    X, W, dY = triple(43, M, K, N, "L")
    dX, dW, _ = run_backward(ctx, X, W, dY, ways)
    dX64, dW64 = oracle.backward(X, W, dY)
    assert np.array_equal(dX.astype(np.float64), dX64)
    assert np.array_equal(dW.astype(np.float64), dW64)
    gX, gW = oracle.jigsaw_backward(ways, X, W, dY)              # the block-wise route reaches the same bits
    assert np.array_equal(dX.astype(np.float64), gX) and np.array_equal(dW.astype(np.float64), gW)


def test_backward_is_the_adjoint_of_the_gpu_forward(jg, ctx):
    """<dY, forward(X', W)> = <dX, X'> with both sides from the GPU path (lattice inputs: exact)."""
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K, N = 258, 200, 136
    X, W, dY = triple(47, M, K, N, "L")
    Xp = inputs.matrix(48, M, K, "L")
    for ways in (1, 2, 4):
        dX, dW, _ = run_backward(ctx, X, W, dY, ways)
        with JigsawLinear(M, K, N, ways, ctx=ctx) as L:
            L.shard(dev(Xp), dev(W))
            L.forward()
            Yp = L.gather().cpu().numpy()
        assert np.sum(dY.astype(np.float64) * Yp) == np.sum(dX.astype(np.float64) * Xp)


def test_backward_error_paths(jg, ctx):
    import ctypes
    lib = jg.raw()
    plan = jg.jg_plan_create(ctx, 64, 64, 64, 4)
    t = torch.zeros(64 * 64, dtype=torch.float32, device="cuda")
    good = [t.data_ptr()] * 4
    need = jg.jg_plan_query(plan, jg.JG_Q_BACKWARD_WORKSPACE_BYTES)
    assert need >= 4 * (64 * 64 + 64 * 64)     # one partial per dX and per dW element
    ws = torch.zeros(need + 256, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256

    def arr(ptrs):
        a = (ctypes.c_void_p * len(ptrs))(*ptrs)
        return ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p))

    bwd = lib.jg_linear_backward
    assert bwd(plan, arr(good), arr(good), None, arr(good), arr(good), base, need) == jg.JG_E_NULL
    assert bwd(plan, arr(good), arr(good), arr(good), arr(good), arr(good), None, need) == jg.JG_E_WORKSPACE
    assert bwd(plan, arr(good), arr(good), arr(good), arr(good), arr(good), base, need - 1) == jg.JG_E_WORKSPACE
    assert bwd(plan, arr(good), arr(good), arr(good), arr(good), arr(good), base + 4, need) == jg.JG_E_ALIGN
    assert bwd(None, arr(good), arr(good), arr(good), arr(good), arr(good), base, need) == jg.JG_E_NULL
    assert lib.jg_gather_as(plan, 9, arr(good), t.data_ptr(), 64) == jg.JG_E_DTYPE
    assert lib.jg_gather_as(plan, jg.JG_T_X, arr(good), t.data_ptr(), 63) == jg.JG_E_SHAPE
    jg.jg_plan_destroy(plan)
    one = jg.jg_plan_create(ctx, 64, 64, 64, 1)
    assert jg.jg_plan_query(one, jg.JG_Q_BACKWARD_WORKSPACE_BYTES) == 0
    assert jg.jg_plan_query(one, jg.JG_Q_BACKWARD_FLOPS_TOTAL) == 4 * 64 ** 3
    jg.jg_plan_destroy(one)
    torch.cuda.synchronize()


@pytest.mark.parametrize("M,K,N,ways", [(1, 1, 1, 1), (1, 2, 2, 2), (2, 2, 2, 4), (2, 4096, 2, 2), (4098, 2, 4, 4),
                                         (3, 5, 7, 1), (129, 4, 132, 1), (128, 128, 128, 1), (256, 256, 256, 4)])
def test_backward_degenerate_and_exact_tile_shapes(jg, ctx, M, K, N, ways):
    X, W, dY = triple(53, M, K, N, "L")
    dX, dW, _ = run_backward(ctx, X, W, dY, ways)
    dX64, dW64 = oracle.backward(X, W, dY)
    assert np.array_equal(dX.astype(np.float64), dX64) and np.array_equal(dW.astype(np.float64), dW64)


def test_backward_leaves_its_inputs_alone_and_is_repeatable(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K, N = 258, 200, 136
    X, W, dY = triple(55, M, K, N)
    with JigsawLinear(M, K, N, 4, ctx=ctx) as L:
        L.shard(dev(X), dev(W))
        L.shard_dy(dev(dY))
        before = [t.clone() for t in L.x + L.w + L.dy]
        L.backward()
        a = (L.gather_dx().clone(), L.gather_dw().clone())
        L.backward()
        L.backward()
        c = (L.gather_dx(), L.gather_dw())
        torch.cuda.synchronize()
        assert all(torch.equal(p, q) for p, q in zip(before, L.x + L.w + L.dy))
        assert torch.equal(a[0], c[0]) and torch.equal(a[1], c[1])


# ---------------------------------------------------------------------------------------------
# the bias gradient: column sums of dY
# ---------------------------------------------------------------------------------------------
def run_bias_backward(jg, ctx, dY, ways, op=None):
    from paper_2507_05753_amd.layer import JigsawLinear
    M, N = dY.shape
    K = 8
    kw = {} if op is None else dict(op=op)
    with JigsawLinear(M, K, N, ways, bias=True, ctx=ctx, **kw) as L:
        L.shard_dy(dev(dY))
        db = L.bias_backward()
        for t in db:
            t.fill_(float("nan"))
        db = L.bias_backward()
        first = [t.cpu().numpy().copy() for t in db]
        L.bias_backward()
        torch.cuda.synchronize()
        assert all(np.array_equal(a, t.cpu().numpy()) for a, t in zip(first, L.db))      # the same bits again
        return first


def check_bias(db_shards, dY, ways):
    want, S = oracle.bias_backward(dY), oracle.bias_backward(dY, absolute=True)
    N = dY.shape[1]
    for r, got in enumerate(db_shards):
        sl = slice(0, N) if ways == 1 else slice((r % 2) * (N // 2), (r % 2 + 1) * (N // 2))
        err = np.abs(got.astype(np.float64) - want[sl])
        # accumulated in double and rounded once
        assert np.all(err <= 2.0 ** -24 * np.abs(want[sl]) * (1 + 1e-6) + 1e-12 * S[sl] + 1e-45), \
            f"rank {r}: max err/S = {(err / np.maximum(S[sl], 1e-300)).max():.3e}"
    if ways == 4:      # the slice of a column half is replicated on the two ranks of that column
        assert np.array_equal(db_shards[0], db_shards[2]) and np.array_equal(db_shards[1], db_shards[3])


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,N", [(2, 2), (100, 100), (130, 258), (258, 136), (2200, 72), (300, 1032), (7001 * 2, 66)])
def test_bias_gradient_matches_oracle(jg, ctx, ways, M, N):
    dY = inputs.matrix(47, M, N, "R")
    check_bias(run_bias_backward(jg, ctx, dY, ways), dY, ways)
    # same-sign data, where FP32 accumulation over the rows would be outside the bar
    dP = np.abs(dY) + np.float32(0.5)
    check_bias(run_bias_backward(jg, ctx, dP, ways), dP, ways)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,N", [(4098, 200), (2 * 2049, 72), (640, 4320), (126, 64)])
def test_bias_gradient_with_and_without_workspace(jg, ctx, ways, M, N):
    """With a workspace the rows are summed in ranges by several workgroups per strip (the last range ragged), without
    one a single workgroup per strip walks all rows: both within half a unit of the exact sum."""
    from paper_2507_05753_amd.layer import JigsawLinear
    dY = np.abs(inputs.matrix(49, M, N, "R")) + np.float32(0.25)
    with JigsawLinear(M, 8, N, ways, bias=True, ctx=ctx) as L:
        L.shard_dy(dev(dY))
        need = L.query(jg.JG_Q_BIAS_BACKWARD_WORKSPACE_BYTES)
        assert (need > 0) == (M // (2 if ways == 4 else 1) >= 128)
        ws = torch.full((max(need, 8),), 0xFF, dtype=torch.uint8, device="cuda")
        p = lambda ts: [t.data_ptr() for t in ts]
        out = {}
        for name, (ptr, size) in dict(none=(None, 0), full=(ws.data_ptr(), need), short=(ws.data_ptr(), max(need - 8, 0))).items():
            db = [torch.full((L.query(jg.JG_Q_B_LEN, r),), float("nan"), device="cuda") for r in range(ways)]
            jg.jg_bias_backward(L.plan, p(L.dy), p(db), ptr, size)
            out[name] = [t.cpu().numpy() for t in db]
            check_bias(out[name], dY, ways)
        assert all(np.array_equal(a, b) for a, b in zip(out["none"], out["short"]))       # too little room: one stage
        if need:
            with pytest.raises(jg.JigsawError) as e:
                jg.jg_bias_backward(L.plan, p(L.dy), p(db), ws.data_ptr() + 4, need)
            assert e.value.status == jg.JG_E_ALIGN


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_bias_gradient_on_lattice_data_and_transposed_plans(jg, ctx, ways):
    M, N = 258, 136
    dY = inputs.matrix(48, M, N, "L")
    want = oracle.bias_backward(dY)
    for op in (None, jg.JG_OP_XTW):                 # only the Y partition matters, which both ops share
        for r, got in enumerate(run_bias_backward(jg, ctx, dY, ways, op)):
            sl = slice(0, N) if ways == 1 else slice((r % 2) * (N // 2), (r % 2 + 1) * (N // 2))
            assert np.array_equal(got.astype(np.float64), want[sl])


@pytest.mark.timeout(300)
def test_bias_gradient_at_config_3(jg, ctx):
    cfg = inputs.CONFIGS[3]
    M, N = cfg["M"], cfg["N"]
    dYd = inputs.matrix_torch(4700, M, N, "R", device="cuda")
    dY = dYd.cpu().numpy()
    for ways in (1, 4):
        check_bias(run_bias_backward(jg, ctx, dY, ways), dY, ways)
