"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Floating-point bar: |Y_gpu - Y64| <= 1e-6 * S with S = |b| + |X| |W|^T (the magnitude of
what is summed).  Layout steps (shard, gather) and lattice-mode products (every partial
sum exactly representable in FP32) must match bit for bit.
"""
import ctypes

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


def run_layer(ctx, X, W, b, ways, combine=0, weights=0, poison=True):
    """shard -> forward -> gather through the C ABI; returns (Y, layer shards as numpy)."""
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K = X.shape
    N = W.shape[0]
    with JigsawLinear(M, K, N, ways, bias=b is not None, combine=combine, weights=weights, ctx=ctx) as L:
        if poison:   # stale workspace / output contents must not matter
            nf = L.ws.numel() // 4
            if nf:
                L.ws[: nf * 4].view(torch.float32).fill_(float("nan"))
            for y in L.y:
                y.fill_(float("nan"))
        L.shard(dev(X), dev(W), dev(b) if b is not None else None)
        L.forward()
        Y = L.gather()
        torch.cuda.synchronize()
        shards = dict(x=[t.cpu().numpy() for t in L.x], w=[t.cpu().numpy() for t in L.w],
                      y=[t.cpu().numpy() for t in L.y],
                      b=[t.cpu().numpy() for t in L.b] if b is not None else None)
        return Y.cpu().numpy(), shards


SHAPES = [
    (100, 100, 100),     # config 1: halves of 50 are not multiples of 4 (scalar load path)
    (2, 2, 2),           # smallest 4-way instance
    (130, 72, 258),      # ragged edges in M and N, K below one slab after halving
    (258, 200, 136),     # several tiles in M
    (64, 520, 640),      # several tiles in N, ragged K tail (260 = 8 slabs + 4)
    (300, 1032, 260),    # multi-tile in both, long K
]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_shard_and_gather_are_bit_exact(jg, ctx, ways, M, K, N):
    X, W, b = inputs.layer_inputs(7, M, K, N, "R", bias=True)
    Y, sh = run_layer(ctx, X, W, b, ways)
    for got, want in zip(sh["x"], oracle.shard_x(X, ways)):
        assert np.array_equal(got, want)
    for got, want in zip(sh["w"], oracle.shard_w(W, ways)):
        assert np.array_equal(got, want)
    for got, want in zip(sh["b"], oracle.shard_b(b, ways)):
        assert np.array_equal(got, want)
    assert np.array_equal(Y, oracle.gather_y(sh["y"], ways))


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("bias", [False, True])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_forward_matches_oracle_within_tolerance(jg, ctx, ways, bias, M, K, N):
    X, W, b = inputs.layer_inputs(11, M, K, N, "R", bias=bias)
    Y, _ = run_layer(ctx, X, W, b, ways)
    Y64 = oracle.linear(X, W, b)
    S = oracle.magnitude(X, W, b)
    err = np.abs(Y.astype(np.float64) - Y64)
    assert np.all(err <= TOL * S), f"max err/S = {(err / S).max():.3e}"


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", SHAPES + [(1000, 1000, 1000)])
def test_lattice_inputs_are_bit_exact(jg, ctx, ways, M, K, N):
    X, W, b = inputs.layer_inputs(13, M, K, N, "L", bias=True)
    Y, _ = run_layer(ctx, X, W, b, ways)
    want = oracle.linear(X, W, b).astype(np.float32)
    assert np.array_equal(want.astype(np.float64), oracle.linear(X, W, b))   # representable
    assert np.array_equal(Y, want)
    # the method's own steps reach the same bits (Eqs. (2), (4))
    assert np.array_equal(Y.astype(np.float64), oracle.jigsaw(ways, X, W, b))


@pytest.mark.parametrize("ways", [2, 4])
def test_options_agree(jg, ctx, ways):
    """Weight-block hand-off by copy or in place: same bits.  Fused or separate combine: the
    fused kernel starts its accumulators from the received partial, the separate kernel adds
    it last, so they agree to rounding (within twice the tolerance) and exactly on lattice inputs."""
    M, K, N = 258, 200, 136
    X, W, b = inputs.layer_inputs(17, M, K, N, "R", bias=True)
    S = oracle.magnitude(X, W, b)
    base, _ = run_layer(ctx, X, W, b, ways, 0, 0)
    direct, _ = run_layer(ctx, X, W, b, ways, 0, 1)
    assert np.array_equal(direct, base)
    sep, _ = run_layer(ctx, X, W, b, ways, 1, 0)
    sep_direct, _ = run_layer(ctx, X, W, b, ways, 1, 1)
    assert np.array_equal(sep_direct, sep)
    assert np.all(np.abs(sep.astype(np.float64) - base) <= 2 * TOL * S)
    Y64 = oracle.linear(X, W, b)
    assert np.all(np.abs(sep.astype(np.float64) - Y64) <= TOL * S)
    XL, WL, bL = inputs.layer_inputs(18, M, K, N, "L", bias=True)
    fusedL, _ = run_layer(ctx, XL, WL, bL, ways, 0, 0)
    sepL, _ = run_layer(ctx, XL, WL, bL, ways, 1, 0)
    assert np.array_equal(fusedL, sepL)
    assert np.array_equal(fusedL.astype(np.float64), oracle.linear(XL, WL, bL))


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", [(256, 4096, 256), (128, 16384, 128)])
def test_same_sign_data_stays_within_tolerance(jg, ctx, ways, M, K, N):
    """All products positive: nothing cancels, S = |Y|, and a single FP32 running sum over K
    would drift past 1e-6 of it; the kernel's two-level accumulation must not."""
    X, W, b = inputs.layer_inputs(29, M, K, N, "R", bias=True)
    X, W, b = np.abs(X) + np.float32(2.0 ** -10), np.abs(W) + np.float32(2.0 ** -16), np.abs(b)
    Y, _ = run_layer(ctx, X, W, b, ways)
    Y64 = oracle.linear(X, W, b)
    S = oracle.magnitude(X, W, b)
    assert np.array_equal(S, Y64)
    err = np.abs(Y.astype(np.float64) - Y64) / S
    assert err.max() <= TOL, f"max err/S = {err.max():.3e}"


def test_config_2_full_comparison(jg, ctx):
    cfg = inputs.CONFIGS[2]
    X, W, _ = inputs.layer_inputs(cfg["seed"], cfg["M"], cfg["K"], cfg["N"], "R")
    Y64 = oracle.linear(X, W)
    S = oracle.magnitude(X, W)
    ys = {}
    for ways in (1, 2, 4):
        Y, _ = run_layer(ctx, X, W, None, ways)
        err = np.abs(Y.astype(np.float64) - Y64)
        assert np.all(err <= TOL * S), (ways, (err / S).max())
        ys[ways] = Y
    # 1-, 2- and 4-way are the same layer (Sec. 6.2.1): within twice the tolerance of each other
    assert np.all(np.abs(ys[1].astype(np.float64) - ys[2]) <= 2 * TOL * S)
    assert np.all(np.abs(ys[1].astype(np.float64) - ys[4]) <= 2 * TOL * S)


def test_closed_forms_on_the_gpu(jg, ctx):
    K = 256
    X = inputs.matrix(19, 192, K, "R")
    eye = np.eye(K, dtype=np.float32)
    perm = np.argsort(inputs.keys(20, np.arange(K, dtype=np.uint64)))
    P = np.zeros((K, K), dtype=np.float32)
    P[np.arange(K), perm] = 1.0
    for ways in (1, 2, 4):
        Y, _ = run_layer(ctx, X, eye, None, ways)
        assert np.array_equal(Y, X)
        Y, _ = run_layer(ctx, X, P, None, ways)
        assert np.array_equal(Y, X[:, perm])


def test_repeated_forward_is_deterministic_and_stateless(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K, N = 258, 200, 136
    X1, W, b = inputs.layer_inputs(23, M, K, N, "L", bias=True)
    X2 = inputs.matrix(24, M, K, "L")
    with JigsawLinear(M, K, N, 4, bias=True, ctx=ctx) as L:
        L.shard(dev(X1), dev(W), dev(b))
        L.forward()
        a = L.gather().cpu().numpy()
        L.shard(X=dev(X2))
        L.forward()
        L.shard(X=dev(X1))
        L.forward()
        L.forward()
        c = L.gather().cpu().numpy()
    assert np.array_equal(a, c)
    assert np.array_equal(a.astype(np.float64), oracle.linear(X1, W, b))


def test_error_paths_with_a_live_context(jg, ctx):
    lib = jg.raw()
    M, K, N = 64, 64, 64
    plan = jg.jg_plan_create(ctx, M, K, N, 2)
    t = torch.zeros(M * N, dtype=torch.float32, device="cuda")
    good = [t.data_ptr(), t.data_ptr()]
    ws_bytes = jg.jg_plan_query(plan, jg.JG_Q_WORKSPACE_BYTES)
    ws = torch.zeros(ws_bytes + 512, dtype=torch.uint8, device="cuda")

    def arr(ptrs):
        a = (ctypes.c_void_p * len(ptrs))(*ptrs)
        return ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p))

    fwd = lib.jg_linear_forward
    assert fwd(plan, None, arr(good), None, arr(good), ws.data_ptr(), ws_bytes) == jg.JG_E_NULL
    assert fwd(plan, arr([good[0], None]), arr(good), None, arr(good), ws.data_ptr(), ws_bytes) == jg.JG_E_NULL
    assert fwd(plan, arr(good), arr(good), None, arr(good), None, ws_bytes) == jg.JG_E_WORKSPACE
    assert fwd(plan, arr(good), arr(good), None, arr(good), ws.data_ptr(), ws_bytes - 1) == jg.JG_E_WORKSPACE
    base = (ws.data_ptr() + 255) // 256 * 256
    assert fwd(plan, arr(good), arr(good), None, arr(good), base + 4, ws_bytes) == jg.JG_E_ALIGN
    assert fwd(plan, arr([good[0] + 2, good[1]]), arr(good), None, arr(good), base, ws_bytes) == jg.JG_E_ALIGN
    assert lib.jg_shard(plan, 7, t.data_ptr(), K, arr(good)) == jg.JG_E_DTYPE
    assert lib.jg_shard(plan, jg.JG_T_X, t.data_ptr(), K - 1, arr(good)) == jg.JG_E_SHAPE
    assert lib.jg_gather(plan, arr(good), t.data_ptr(), N - 1) == jg.JG_E_SHAPE
    assert lib.jg_gather(plan, arr(good), None, N) == jg.JG_E_NULL
    jg.jg_plan_destroy(plan)
    biased = jg.jg_plan_create(ctx, M, K, N, 2, has_bias=True)
    assert fwd(biased, arr(good), arr(good), None, arr(good), base, ws_bytes) == jg.JG_E_NULL
    jg.jg_plan_destroy(biased)
    out = ctypes.c_void_p()
    assert lib.jg_init(ctypes.byref(out), 99, None) == jg.JG_E_HIP
    assert lib.jg_init(None, 0, None) == jg.JG_E_NULL
    torch.cuda.synchronize()


def test_profile_counts_launches(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear
    with JigsawLinear(256, 128, 128, 4, ctx=ctx, combine=jg.JG_COMBINE_SEPARATE) as L:
        for t in L.x + L.w:
            t.zero_()
        jg.jg_profile(ctx, True)
        for _ in range(3):
            L.forward()
        jg.jg_profile(ctx, False)
        L.forward()   # untimed
        ms, n = jg.jg_profile_read(ctx, jg.JG_KERNEL_GEMM)
        assert n == 6 and ms > 0
        assert jg.jg_profile_read(ctx, jg.JG_KERNEL_WEIGHT_COPY)[1] == 3
        assert jg.jg_profile_read(ctx, jg.JG_KERNEL_COMBINE)[1] == 3
        assert jg.jg_profile_read(ctx, jg.JG_KERNEL_GEMM)[1] == 0


@pytest.mark.parametrize("M,K,N,ways", [(1, 1, 1, 1), (1, 2, 2, 2), (2, 2, 2, 4), (1, 4096, 2, 2), (4098, 2, 2, 4),
                                         (3, 5, 7, 1), (129, 4, 129, 1), (128, 32, 128, 1), (256, 64, 128, 4)])
def test_degenerate_and_exact_tile_shapes(jg, ctx, M, K, N, ways):
    X, W, b = inputs.layer_inputs(31, M, K, N, "L", bias=True)
    Y, _ = run_layer(ctx, X, W, b, ways)
    assert np.array_equal(Y.astype(np.float64), oracle.linear(X, W, b))


def test_strided_global_views_and_untouched_inputs(jg, ctx):
    """jg_shard / jg_gather take a leading dimension: shard from and gather into views of wider
    matrices; inputs are never written, bytes outside the gathered region are left alone."""
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K, N, pad = 130, 72, 136, 12
    X, W, b = inputs.layer_inputs(33, M, K, N, "L", bias=True)
    Xw = torch.full((M, K + pad), 7.0, device="cuda"); Xw[:, :K] = dev(X)
    Ww = torch.full((N, K + pad), 7.0, device="cuda"); Ww[:, :K] = dev(W)
    Yw = torch.full((M, N + pad), -5.0, device="cuda")
    for ways in (1, 2, 4):
        with JigsawLinear(M, K, N, ways, bias=True, ctx=ctx) as L:
            L.shard(Xw[:, :K], Ww[:, :K], dev(b))
            x_before = [t.clone() for t in L.x]
            w_before = [t.clone() for t in L.w]
            L.forward()
            L.gather(Yw[:, :N])
            torch.cuda.synchronize()
            assert all(torch.equal(a, c) for a, c in zip(x_before, L.x))
            assert all(torch.equal(a, c) for a, c in zip(w_before, L.w))
        assert np.array_equal(Yw[:, :N].cpu().numpy().astype(np.float64), oracle.linear(X, W, b))
        assert torch.all(Yw[:, N:] == -5.0) and torch.all(Xw[:, K:] == 7.0)
