"""GPU parity of the reduced-precision modes (JG_BF16, JG_BF16X3) of the X W^T layer against the CPU oracle.

The mode's definition (operands rounded to bfloat16 on their bit pattern, products exact, sums FP32) is
what the oracle evaluates in double on the same rounded operands, so the bars are those of the FP32 layer:
the shards bit for bit, |Y_gpu - Y64| <= 1e-6 * S with S the magnitude of the rounded operands' products,
and bit-exact results on lattice inputs (which the rounding leaves unchanged).  The split mode is also held
to its distance from the full-precision layer.
"""
import time

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


def as_f32(t):
    """A bfloat16 device tensor as the FP32 values it stands for (exact)."""
    return t.float().cpu().numpy()


def terms_of(jg, dtype):
    return 3 if dtype == jg.JG_BF16X3 else 1


def run_layer(jg, ctx, X, W, b, ways, dtype, combine=0, weights=0, residual=None, act=0):
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K = X.shape
    N = W.shape[0]
    with JigsawLinear(M, K, N, ways, bias=b is not None, combine=combine, weights=weights, ctx=ctx, dtype=dtype) as L:
        if L.ws_bytes:
            L.ws.fill_(0xFF)
        for y in L.y:
            y.fill_(float("nan"))
        L.shard(dev(X), dev(W), dev(b) if b is not None else None)
        res = None
        if residual is not None:
            res = [torch.empty_like(y) for y in L.y]
            jg.jg_shard(L.plan, jg.JG_T_Y, dev(residual).data_ptr(), N, [t.data_ptr() for t in res])
        L.forward(residual=res, activation=act)
        Y = L.gather()
        torch.cuda.synchronize()
        return Y.cpu().numpy(), [as_f32(t) for t in L.x], [as_f32(t) for t in L.w]


# (M, K, N): K shares in whole 8-element chunks; ragged last slabs (K % 64 != 0), ragged tile edges,
# several tiles in M and in N, K long enough for many slabs
SHAPES = [(2, 16, 2), (100, 80, 100), (130, 144, 258), (258, 1040, 136), (520, 272, 600), (300, 4112, 260)]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_shards_hold_the_rounded_operands(jg, ctx, ways, dtype_name, M, K, N):
    dtype = getattr(jg, dtype_name)
    X, W, b = inputs.layer_inputs(401, M, K, N, "R", bias=True)
    X = (X * np.float32(3.0)).astype(np.float32)
    _, xs, ws = run_layer(jg, ctx, X, W, b, ways, dtype)
    for got, src in ((xs, oracle.shard_x(X, ways)), (ws, oracle.shard_w(W, ways))):
        for g, blk in zip(got, src):
            cols = blk.shape[1]
            plane = (cols + 63) // 64 * 64          # every plane of a shard row is padded to whole 128-byte lines
            if dtype == jg.JG_BF16:
                assert g.shape[1] == plane
                assert np.array_equal(g[:, :cols], oracle.round_bf16(blk))
            else:
                assert g.shape[1] == 2 * plane
                hi, lo = oracle.split_bf16(blk)
                assert np.array_equal(g[:, :cols], hi) and np.array_equal(g[:, plane:plane + cols], lo)


@pytest.mark.parametrize("ways", [1, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_shard_from_a_strided_unaligned_global_tensor(jg, ctx, ways, dtype_name):
    """The global FP32 tensors may have any leading dimension and 4-byte alignment (element-wise reads then)."""
    from paper_2507_05753_amd.layer import JigsawLinear
    dtype = getattr(jg, dtype_name)
    M, K, N = 66, 80, 36
    X, W, _ = inputs.layer_inputs(412, M, K, N, "R")
    Xbig = torch.full((M, K + 3), float("nan"), device="cuda")
    Xbig[:, :K] = dev(X)
    Wflat = torch.full((N * K + 1,), float("nan"), device="cuda")       # W starts 4 bytes into an aligned buffer
    Wview = Wflat[1:].view(N, K)
    Wview.copy_(dev(W))
    with JigsawLinear(M, K, N, ways, ctx=ctx, dtype=dtype) as L:
        jg.jg_shard(L.plan, jg.JG_T_X, Xbig.data_ptr(), K + 3, [t.data_ptr() for t in L.x])
        jg.jg_shard(L.plan, jg.JG_T_W, Wview.data_ptr(), K, [t.data_ptr() for t in L.w])
        L.forward()
        Y = L.gather().cpu().numpy()
    t = terms_of(jg, dtype)
    S = oracle.linear_reduced(X, W, None, t, absolute=True)
    assert np.all(np.abs(Y.astype(np.float64) - oracle.linear_reduced(X, W, None, t)) <= TOL * S)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("bias", [False, True])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_forward_matches_oracle_within_tolerance(jg, ctx, ways, dtype_name, bias, M, K, N):
    dtype = getattr(jg, dtype_name)
    X, W, b = inputs.layer_inputs(402, M, K, N, "R", bias=bias)
    Y, _, _ = run_layer(jg, ctx, X, W, b, ways, dtype)
    t = terms_of(jg, dtype)
    want = oracle.linear_reduced(X, W, b, t)
    S = oracle.linear_reduced(X, W, b, t, absolute=True)
    err = np.abs(Y.astype(np.float64) - want)
    assert np.all(err <= TOL * S), f"max err/S = {(err / S).max():.3e}"
    # the mode is what it says: far from (JG_BF16) or close to (JG_BF16X3) the full-precision layer
    full = np.abs(Y.astype(np.float64) - oracle.linear(X, W, b)) / oracle.magnitude(X, W, b)
    if dtype == jg.JG_BF16X3:
        assert full.max() <= 2.0 ** -15
    elif K >= 80:
        assert full.max() > 1e-5


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_lattice_inputs_are_bit_exact(jg, ctx, ways, dtype_name, M, K, N):
    dtype = getattr(jg, dtype_name)
    X, W, b = inputs.layer_inputs(403, M, K, N, "L", bias=True)
    Y, _, _ = run_layer(jg, ctx, X, W, b, ways, dtype)
    want = oracle.linear(X, W, b)
    assert np.array_equal(want.astype(np.float32).astype(np.float64), want)
    assert np.array_equal(Y.astype(np.float64), want)


@pytest.mark.parametrize("ways", [2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("combine,weights", [(1, 0), (0, 1), (1, 1)])
def test_option_variants(jg, ctx, ways, dtype_name, combine, weights):
    dtype = getattr(jg, dtype_name)
    M, K, N = 258, 272, 136
    X, W, b = inputs.layer_inputs(404, M, K, N, "L", bias=True)
    base, _, _ = run_layer(jg, ctx, X, W, b, ways, dtype)
    other, _, _ = run_layer(jg, ctx, X, W, b, ways, dtype, combine=combine, weights=weights)
    assert np.array_equal(base, other)
    X, W, b = inputs.layer_inputs(405, M, K, N, "R", bias=True)
    got, _, _ = run_layer(jg, ctx, X, W, b, ways, dtype, combine=combine, weights=weights)
    t = terms_of(jg, dtype)
    S = oracle.linear_reduced(X, W, b, t, absolute=True)
    assert np.all(np.abs(got.astype(np.float64) - oracle.linear_reduced(X, W, b, t)) <= TOL * S)


@pytest.mark.parametrize("ways", [1, 4])
def test_epilogue_rides_along(jg, ctx, ways):
    M, K, N = 300, 272, 260
    X, W, b = inputs.layer_inputs(406, M, K, N, "R", bias=True)
    R = inputs.matrix(407, M, N, "R")
    Y, _, _ = run_layer(jg, ctx, X, W, b, ways, jg.JG_BF16, residual=R, act=jg.JG_ACT_GELU)
    want = oracle.gelu(oracle.linear_reduced(X, W, b, 1)) + R.astype(np.float64)
    S = oracle.linear_reduced(X, W, b, 1, absolute=True) + np.abs(R)
    assert np.all(np.abs(Y.astype(np.float64) - want) <= TOL * S)


@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_split_tail_and_whole_tiles_agree(jg, ctx, dtype_name):
    """Tiles of a last partial round are cut into runs of slabs that a second kernel adds in ascending k order:
    another order of the FP32 additions (inside the tolerance), the same numbers on lattice inputs, and the same
    bits from run to run."""
    from paper_2507_05753_amd.layer import JigsawLinear
    dtype = getattr(jg, dtype_name)
    M, K, N = 300, 8208, 260          # 4 tiles of 257 (771 with split operands) slabs: cut into 16 runs each
    t = terms_of(jg, dtype)
    for mode in ("L", "R"):
        X, W, b = inputs.layer_inputs(410, M, K, N, mode, bias=True)
        R = inputs.matrix(411, M, N, mode)
        want = oracle.gelu(oracle.linear_reduced(X, W, b, t)) + R if mode == "R" else oracle.linear(X, W, b) + R
        S = oracle.linear_reduced(X, W, b, t, absolute=True) + np.abs(R)
        got = {}
        for tail in (jg.JG_TAIL_SPLIT, jg.JG_TAIL_WHOLE):
            for ways in (1, 4):
                with JigsawLinear(M, K, N, ways, bias=True, ctx=ctx, dtype=dtype, tail=tail) as L:
                    assert (L.query(jg.JG_Q_TAIL_SCRATCH_BYTES) > 0) == (tail == jg.JG_TAIL_SPLIT)
                    L.ws.fill_(0xFF)
                    L.shard(dev(X), dev(W), dev(b))
                    res = [torch.empty_like(y) for y in L.y]
                    jg.jg_shard(L.plan, jg.JG_T_Y, dev(R).data_ptr(), N, [r.data_ptr() for r in res])
                    act = jg.JG_ACT_GELU if mode == "R" else jg.JG_ACT_NONE
                    L.forward(residual=res, activation=act)
                    Y = L.gather().cpu().numpy()
                    L.forward(residual=res, activation=act)
                    assert np.array_equal(Y, L.gather().cpu().numpy())          # deterministic
                got[(tail, ways)] = Y
                if mode == "L":
                    assert np.array_equal(Y.astype(np.float64), want)
                else:
                    assert np.all(np.abs(Y.astype(np.float64) - want) <= TOL * S)


@pytest.mark.parametrize("tail", [0, 1])
@pytest.mark.parametrize("K", [1024, 2000, 4096, 8192, 16384])
def test_same_sign_operands(jg, ctx, K, tail):
    # All-positive data: the running FP32 sum is the magnitude itself.  The 256 accumulators of a wavefront fill its
    # register file, so the kernel sums in one level; the second level is taken between launches (JG_ACC_LEVELS, the
    # default: chunks of the contraction, each launch adding on top of what the output holds), which keeps the drift
    # inside the bar of the layer at any K, with whole tiles and with a split tail.
    from paper_2507_05753_amd.layer import JigsawLinear
    M, N = 136, 264
    X = np.abs(inputs.matrix(408, M, K, "R"))
    W = np.abs(inputs.matrix(409, N, K, "R"))
    for dtype in (jg.JG_BF16, jg.JG_BF16X3):
        t = terms_of(jg, dtype)
        S = oracle.linear_reduced(X, W, None, t, absolute=True)
        want = oracle.linear_reduced(X, W, None, t)
        for ways in (1, 2):
            with JigsawLinear(M, K, N, ways, ctx=ctx, dtype=dtype, tail=tail) as L:
                L.shard(dev(X), dev(W))
                L.forward()
                Y = L.gather().cpu().numpy()
            err = np.abs(Y.astype(np.float64) - want)
            assert np.all(err <= TOL * S), f"dtype={dtype} ways={ways}: {(err / S).max():.3e}"


@pytest.mark.parametrize("dtype_name", ["bf16", "bf16x3"])
def test_single_level_option(jg, ctx, dtype_name):
    """JG_ACC_SINGLE: one launch per product whatever K.  The same bits as the default on lattice inputs (every sum is
    exact), inside the bar on zero-mean data, and one launch where the default takes several."""
    from paper_2507_05753_amd.layer import JigsawLinear
    dtype = jg.JG_BF16 if dtype_name == "bf16" else jg.JG_BF16X3
    t = terms_of(jg, dtype)
    M, K, N = 200, 4096, 136
    for mode in ("L", "R"):
        X, W, b = inputs.layer_inputs(431, M, K, N, mode, bias=True)
        got = {}
        for acc in (jg.JG_ACC_LEVELS, jg.JG_ACC_SINGLE):
            with JigsawLinear(M, K, N, 2, bias=True, ctx=ctx, dtype=dtype, accumulate=acc) as L:
                L.shard(dev(X), dev(W), dev(b))
                L.forward()
                got[acc] = L.gather().cpu().numpy()
                launches = L.query(jg.JG_Q_GEMM_LAUNCHES)
            assert (launches == 2) if acc == jg.JG_ACC_SINGLE else (launches in (4, 6)), (acc, launches)
        want = oracle.linear_reduced(X, W, b, t)
        S = oracle.linear_reduced(X, W, b, t, absolute=True)
        for acc, Y in got.items():
            assert np.all(np.abs(Y - want) <= TOL * S), (mode, acc)
        if mode == "L":
            assert np.array_equal(got[jg.JG_ACC_LEVELS], got[jg.JG_ACC_SINGLE]) and np.array_equal(got[0], want)
    with pytest.raises(jg.JigsawError) as e:
        jg.jg_plan_create(ctx, 64, 64, 64, 2, dtype=dtype, accumulate=2)
    assert e.value.status == jg.JG_E_DTYPE


def random_cases(n):
    """Seeded shapes and options: every rank's share of K in whole 8-element chunks, sizes from one element to a
    few tiles, K from one chunk to dozens of slabs, small enough for the oracle's full product."""
    k = inputs.keys(5150, np.arange(8 * n, dtype=np.uint64)).reshape(n, 8)
    cases = []
    for row in k:
        ways = (1, 2, 4)[int(row[0] % np.uint64(3))]
        half = 2 if ways >= 2 else 1
        share = 8 * (1 + int(row[1] % np.uint64(160)))              # 8 .. 1280 per rank
        K = share * half
        M = 1 + int(row[2] % np.uint64(600))
        N = 1 + int(row[3] % np.uint64(600))
        if ways == 4:
            M += M & 1
        if ways >= 2:
            N += N & 1
        while M * N * K > 1.5e8:
            M = max(2, M // 2 + (M // 2 & 1))
        cases.append((ways, M, K, N, int(row[4] & np.uint64(1)), int(row[5] & np.uint64(1)), int(row[6] & np.uint64(1)),
                      int(row[7] & np.uint64(1))))
    return cases


@pytest.mark.parametrize("ways,M,K,N,x3,bias,act,res", random_cases(36))
def test_random_shapes_and_options(jg, ctx, ways, M, K, N, x3, bias, act, res):
    dtype = jg.JG_BF16X3 if x3 else jg.JG_BF16
    t = 3 if x3 else 1
    X, W, b = inputs.layer_inputs(5200 + M, M, K, N, "R", bias=True)
    b = b if bias else None
    R = inputs.matrix(5300 + N, M, N, "R") if res else None
    Y, _, _ = run_layer(jg, ctx, X, W, b, ways, dtype, residual=R, act=jg.JG_ACT_GELU if act else jg.JG_ACT_NONE)
    want = oracle.linear_reduced(X, W, b, t)
    S = oracle.linear_reduced(X, W, b, t, absolute=True)
    if act:
        want = oracle.gelu(want)
    if res:
        want = want + R
        S = S + np.abs(R)
    err = np.abs(Y.astype(np.float64) - want)
    bar = TOL * S
    assert np.all(err <= bar), f"max err/S = {(err / S).max():.3e}"


def test_calls_that_need_fp32_shards_are_refused(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear
    with JigsawLinear(16, 32, 16, 2, ctx=ctx, dtype=jg.JG_BF16) as L:
        ptrs = [t.data_ptr() for t in L.y]
        for call in (lambda: jg.jg_gather_as(L.plan, jg.JG_T_X, ptrs, ptrs[0], 64),
                     lambda: jg.jg_gather_as(L.plan, jg.JG_T_W, ptrs, ptrs[0], 64),
                     lambda: jg.jg_shard_patches(L.plan, ptrs[0], 2, 8, 8, 4, ptrs)):
            with pytest.raises(jg.JigsawError) as e:
                call()
            assert e.value.status == jg.JG_E_DTYPE
        with pytest.raises(jg.JigsawError) as e:          # bfloat16 shards move in 16-byte pieces
            jg.jg_shard(L.plan, jg.JG_T_X, L.y[0].data_ptr(), 32, [ptrs[0] + 4, ptrs[1]])
        assert e.value.status == jg.JG_E_ALIGN
        with pytest.raises(jg.JigsawError) as e:          # the backward rounds its operands into a workspace
            jg.jg_linear_backward(L.plan, ptrs, ptrs, ptrs, ptrs, ptrs, None, 0)
        assert e.value.status == jg.JG_E_WORKSPACE


# --------------------------------------------------------------------------------------------
# the mixing MLP and the channel-mixing block in mixed precision (FP32 activations, bfloat16 products)
# --------------------------------------------------------------------------------------------
TOL_H = 1e-6 + 2.0 ** -23        # the layer's bar through GELU (slope <= 1.13; the product itself stays near 1e-7), and H's own FP32 rounding


def mlp_operands(seed, M, C, Hd):
    X = (inputs.matrix(seed, M, C, "R") + np.float32(0.25)).astype(np.float32)
    W1 = inputs.matrix(seed + 1, Hd, C, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, Hd, "R")[0]
    W2 = inputs.matrix(seed + 3, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 4, 1, C, "R")[0]
    return X, W1, b1, W2, b2


def check_mixed_chain(X, Xin, H, Y, W1, b1, W2, b2, t):
    """Xin: what the first product read (X, or the layer norm's FP32 output as the GPU stored it)."""
    S1 = oracle.linear_reduced(Xin, W1, b1, t, absolute=True)
    eh = np.abs(H.astype(np.float64) - oracle.gelu(oracle.linear_reduced(Xin, W1, b1, t)))
    assert np.all(eh <= TOL_H * S1), f"H: max err/S1 = {(eh / S1).max():.3e}"
    # the second layer on its own, from the H the GPU stored (both sides round the same FP32 values to bfloat16);
    # the skip connection adds X itself, not its rounding
    want = X.astype(np.float64) + oracle.linear_reduced(H, W2, b2, t)
    SY = np.abs(X.astype(np.float64)) + oracle.linear_reduced(H, W2, b2, t, absolute=True)
    ey = np.abs(Y.astype(np.float64) - want)
    assert np.all(ey <= TOL * SY), f"Y: max err/S = {(ey / SY).max():.3e}"
    return want


# C and Hd: every rank's share in whole 8-element chunks; ragged tiles and slabs
MLP_SHAPES = [(100, 96, 112), (130, 80, 272), (258, 272, 144), (300, 528, 1040)]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("M,C,Hd", MLP_SHAPES)
def test_mixed_precision_mlp(jg, ctx, ways, dtype_name, M, C, Hd):
    from paper_2507_05753_amd.layer import JigsawMLP
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    X, W1, b1, W2, b2 = mlp_operands(430, M, C, Hd)
    with JigsawMLP(M, C, Hd, ways, ctx=ctx, dtype=dtype) as L:
        L.ws.fill_(0xFF)
        L.shard(dev(X), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        H, Y = L.gather_h().cpu().numpy(), L.gather().cpu().numpy()
        L.forward()                                   # the inputs were not overwritten: the same again
        assert np.array_equal(Y, L.gather().cpu().numpy())
    check_mixed_chain(X, X, H, Y, W1, b1, W2, b2, t)
    # end to end against the oracle's own chain: apart from the few entries of H whose bfloat16 rounding
    # falls the other way for an error in the last FP32 bits, the two agree far inside one bfloat16 step
    r = oracle.mlp_reduced(X, W1, b1, W2, b2, t)
    assert np.all(np.abs(Y - r["Y"]) <= 2.0 ** -9 * r["SY"])
    assert np.abs(Y - oracle.mlp(X, W1, b1, W2, b2)["Y"]).max() > (1e-4 if t == 1 else 1e-8)   # it IS reduced precision


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_mixed_precision_mixing_block(jg, ctx, ways, dtype_name):
    from paper_2507_05753_amd.layer import JigsawMixing
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    M, C, Hd = 258, 272, 400
    X, W1, b1, W2, b2 = mlp_operands(440, M, C, Hd)
    gamma = (inputs.matrix(445, 1, C, "R")[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(446, 1, C, "R")[0]
    with JigsawMixing(M, C, Hd, ways, ctx=ctx, dtype=dtype) as L:
        L.shard(dev(X), dev(gamma), dev(beta), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        Xn, H, Y = L.gather_xn().cpu().numpy(), L.gather_h().cpu().numpy(), L.gather().cpu().numpy()
    want = oracle.layernorm(X, gamma, beta, oracle.ln_groups(ways))
    assert np.all(np.abs(Xn.astype(np.float64) - want) <= 2.0 ** -24 * np.abs(want) * (1 + 1e-6) + 1e-10)
    check_mixed_chain(X, Xn, H, Y, W1, b1, W2, b2, t)
    r = oracle.mixing_block_reduced(ways, X, gamma, beta, W1, b1, W2, b2, t)
    assert np.all(np.abs(Y - r["Y"]) <= 2.0 ** -9 * r["SY"])


@pytest.mark.parametrize("ways", [2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_mixed_precision_mlp_with_the_separate_combine(jg, ctx, ways, dtype_name):
    """With the fused combine the launch that writes H also writes its bfloat16 copy; with the separate one H is
    converted afterwards.  Both copies hold the roundings of the same FP32 values: the same Y bit for bit."""
    from paper_2507_05753_amd.layer import JigsawLinear, JigsawMLP
    dtype = getattr(jg, dtype_name)
    M, C, Hd = 258, 272, 400
    X, W1, b1, W2, b2 = mlp_operands(450, M, C, Hd)
    out = {}
    for combine in (jg.JG_COMBINE_FUSED, jg.JG_COMBINE_SEPARATE):
        with JigsawMLP(M, C, Hd, ways, ctx=ctx, dtype=dtype) as L:
            if combine == jg.JG_COMBINE_SEPARATE:        # swap the first layer's plan for one with the other combine
                alt = JigsawLinear(M, C, Hd, ways, bias=True, ctx=ctx, dtype=dtype, combine=combine)
                alt.y, alt.w, alt.b = L.first.y, L.first.w, L.first.b
                keep, L.first = L.first, alt
                need = alt.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES) + L.second.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES)
                L.ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
                L.ws_bytes = need
            L.ws.fill_(0xFF)
            L.shard(dev(X), dev(W1), dev(b1), dev(W2), dev(b2))
            L.forward()
            out[combine] = (L.gather_h().cpu().numpy(), L.gather().cpu().numpy())
            if combine == jg.JG_COMBINE_SEPARATE:
                L.first = keep
                alt.y = alt.w = alt.b = None
                alt.close()
    Hf, Yf = out[jg.JG_COMBINE_FUSED]
    Hs, Ys = out[jg.JG_COMBINE_SEPARATE]
    check_mixed_chain(X, X, Hs, Ys, W1, b1, W2, b2, terms_of(jg, dtype))
    # H itself may differ in the last bits (kept + received in another kernel); where it does not, Y must agree exactly
    if np.array_equal(Hf, Hs):
        assert np.array_equal(Yf, Ys)


def test_mixed_precision_chain_arguments(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear, JigsawMLP
    with JigsawMLP(64, 32, 48, 2, ctx=ctx, dtype=jg.JG_BF16) as L, \
            JigsawLinear(64, 48, 32, 2, bias=True, ctx=ctx) as F32, \
            JigsawLinear(64, 48, 32, 2, bias=True, ctx=ctx, dtype=jg.JG_BF16X3) as X3:
        f, s = L.first, L.second
        p = lambda ts: [x.data_ptr() for x in ts]
        need = f.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES) + s.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES)
        assert need == L.ws_bytes and need > f.query(jg.JG_Q_WORKSPACE_BYTES) + s.query(jg.JG_Q_WORKSPACE_BYTES)
        args = lambda second, ws_bytes: (f.plan, second.plan, p(L.xin), p(f.w), p(f.b), p(second.w), p(second.b),
                                         p(f.y), p(s.y), L.ws.data_ptr(), ws_bytes)
        for other in (F32, X3):                           # both layers in the same precision
            with pytest.raises(jg.JigsawError) as e:
                jg.jg_mlp_forward(*args(other, L.ws_bytes))
            assert e.value.status == jg.JG_E_DTYPE
        with pytest.raises(jg.JigsawError) as e:          # room for one layer and its input is not enough
            jg.jg_mlp_forward(*args(s, max(f.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES), s.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES))))
        assert e.value.status == jg.JG_E_WORKSPACE
        # an FP32 plan's chain workspace is its workspace
        assert F32.query(jg.JG_Q_CHAIN_WORKSPACE_BYTES) == F32.query(jg.JG_Q_WORKSPACE_BYTES)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_mixed_precision_mlp_at_channel_mixing_size(jg, dtype_name):
    """The channel-mixing MLP of the paper's 1-billion-parameter model (Sec. 6.2.1) at full size, in the launch
    configuration bench.py --op mlp --dtype times: sampled rows element by element, every entry finite."""
    from paper_2507_05753_amd.layer import JigsawMLP
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    cfg = inputs.MLP_CONFIGS["channel_mixing_1b"]
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    Xd = inputs.matrix_torch(seed, M, C, "R", device="cuda")
    W1d = inputs.matrix_torch(seed + 1, Hd, C, "R", inputs.W_SCALE_EXP, device="cuda")
    W2d = inputs.matrix_torch(seed + 3, C, Hd, "R", inputs.W_SCALE_EXP, device="cuda")
    b1 = inputs.matrix(seed + 2, 1, Hd, "R")[0]
    b2 = inputs.matrix(seed + 4, 1, C, "R")[0]
    W1, W2 = W1d.cpu().numpy(), W2d.cpu().numpy()
    k = inputs.keys(7100, np.arange(20, dtype=np.uint64))
    rows = np.unique(np.concatenate([(k % np.uint64(M)).astype(np.int64), [0, M // 2 - 1, M // 2, M - 1]]))
    idx = torch.from_numpy(rows).cuda()
    Xs = Xd[idx].cpu().numpy()
    for ways in (1, 4):
        with JigsawMLP(M, C, Hd, ways, dtype=dtype) as L:
            L.shard(Xd, W1d, dev(b1), W2d, dev(b2))
            L.forward()
            H, Y = L.gather_h(), L.gather()
            torch.cuda.synchronize()
            assert torch.isfinite(Y).all() and torch.isfinite(H).all()
            Hs, Ys = H[idx].cpu().numpy(), Y[idx].cpu().numpy()
        check_mixed_chain(Xs, Xs, Hs, Ys, W1, b1, W2, b2, t)


# --------------------------------------------------------------------------------------------
# full size: config 3 (n = 1e8 items)
# --------------------------------------------------------------------------------------------
def note(capsys, msg):
    with capsys.disabled():
        print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def pm1(seed, n, cols):
    bits = inputs.keys(seed, np.arange(n * cols, dtype=np.uint64)) >> np.uint64(63)
    return np.where(bits.reshape(n, cols) == 1, 1.0, -1.0)


@pytest.mark.timeout(900)
def test_config3_full_size(jg, capsys):
    from paper_2507_05753_amd.layer import JigsawLinear
    cfg = inputs.CONFIGS[3]
    M, K, N, seed = cfg["M"], cfg["K"], cfg["N"], cfg["seed"]
    Xd = inputs.matrix_torch(seed, M, K, "R", 0, device="cuda")
    Wd = inputs.matrix_torch(seed + inputs.W_STREAM, N, K, "R", inputs.W_SCALE_EXP, device="cuda")
    X, W = Xd.cpu().numpy(), Wd.cpu().numpy()
    k = inputs.keys(8000, np.arange(400, dtype=np.uint64))
    I = np.unique(np.concatenate([(k[:200] % np.uint64(M)).astype(np.int64), [0, M // 2 - 1, M // 2, M - 1]]))
    J = np.unique(np.concatenate([(k[200:] % np.uint64(N)).astype(np.int64), [0, N // 2 - 1, N // 2, N - 1]]))
    V = pm1(8001, N, 2)
    for dtype, t in ((jg.JG_BF16, 1), (jg.JG_BF16X3, 3)):
        # references from the rounded operands: sampled entries one by one, and Y v = X (W^T v) in double
        if t == 1:
            planes = [(oracle.round_bf16(X), oracle.round_bf16(W))]
        else:
            Xh, Xl = oracle.split_bf16(X)
            Wh, Wl = oracle.split_bf16(W)
            planes = [(Xh, Wh), (Xh, Wl), (Xl, Wh)]
        want = np.zeros((I.size, J.size))
        mag = np.zeros((I.size, J.size))
        fre = np.zeros((M, 2))
        frb = np.zeros((M, 2))
        for A, B in planes:
            want += oracle.linear(A[I], B[J])
            mag += oracle.magnitude(A[I], B[J])
            A64, B64 = A.astype(np.float64), B.astype(np.float64)
            fre += A64 @ (B64.T @ V)
            frb += np.abs(A64) @ (np.abs(B64).T @ np.abs(V))
            del A64, B64
        del planes
        note(capsys, f"reduced precision, terms={t}: references ready")
        for ways in (1, 4):
            with JigsawLinear(M, K, N, ways, dtype=dtype) as L:
                if L.ws_bytes:
                    L.ws.fill_(0xFF)
                L.shard(Xd, Wd)
                L.forward()
                Y = L.gather()
                torch.cuda.synchronize()
                Y = Y.cpu().numpy()
            assert np.isfinite(Y).all()
            err = np.abs(Y.astype(np.float64) @ V - fre)
            assert np.all(err <= TOL * frb), f"ways={ways}: Freivalds worst {(err / frb).max():.3e}"
            e = np.abs(Y[np.ix_(I, J)] - want) / mag
            assert e.max() <= TOL, (ways, e.max())
            note(capsys, f"terms={t} ways={ways}: Freivalds {(err / frb).max():.2e}, {e.size} entries max err/S {e.max():.2e}")


# ---------------------------------------------------------------------------------------------
# the transposed layer Y = X^T W in reduced precision: the shard step writes contraction-major bfloat16 shards
# ---------------------------------------------------------------------------------------------
# (K = tokens, M = channels, N): any K (the shard step pads a rank's share of it to whole 8-element chunks with zeros)
XTW_SHAPES = [(16, 2, 2), (30, 6, 4), (80, 100, 100), (142, 130, 258), (1040, 258, 136), (272, 520, 600), (4100, 74, 260)]


def run_xtw(jg, ctx, X, W, b, ways, dtype, combine=0, weights=0):
    from paper_2507_05753_amd.layer import JigsawLinear
    K, M = X.shape
    N = W.shape[1]
    with JigsawLinear(M, K, N, ways, bias=b is not None, combine=combine, weights=weights, ctx=ctx, dtype=dtype,
                      op=jg.JG_OP_XTW) as L:
        if L.ws_bytes:
            L.ws.fill_(0xFF)
        for t in L.y:
            t.fill_(float("nan"))
        L.shard(dev(X), dev(W), dev(b) if b is not None else None)
        L.forward()
        Y = L.gather()
        torch.cuda.synchronize()
        return Y.cpu().numpy(), [as_f32(t) for t in L.x], [as_f32(t) for t in L.w]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("K,M,N", XTW_SHAPES)
def test_transposed_layer_shards_and_forward(jg, ctx, ways, dtype_name, K, M, N):
    dtype = getattr(jg, dtype_name)
    X = (inputs.matrix(430, K, M, "R") * np.float32(3.0)).astype(np.float32)
    W = inputs.matrix(431, K, N, "R", inputs.W_SCALE_EXP)
    b = inputs.matrix(432, 1, N, "R")[0]
    Y, xs, ws = run_xtw(jg, ctx, X, W, b, ways, dtype)
    # the shards: block (row half, column half) of the FP32 matrix, transposed, rounded (or split) element by element
    rows, cols = (2 if ways == 4 else 1), (2 if ways >= 2 else 1)
    for got, src in ((xs, X), (ws, W)):
        kr, cc = src.shape[0] // rows, src.shape[1] // cols
        plane = (kr + 63) // 64 * 64
        for r, g in enumerate(got):
            i, j = (r // 2, r % 2) if ways == 4 else (0, r)
            blk = np.ascontiguousarray(src[i * kr:(i + 1) * kr, j * cc:(j + 1) * cc].T)
            assert g.shape[0] == cc
            if dtype == jg.JG_BF16:
                assert g.shape[1] == plane and np.array_equal(g[:, :kr], oracle.round_bf16(blk))
            else:
                hi, lo = oracle.split_bf16(blk)
                assert g.shape[1] == 2 * plane
                assert np.array_equal(g[:, :kr], hi) and np.array_equal(g[:, plane:plane + kr], lo)
    t = terms_of(jg, dtype)
    want = oracle.linear_xtw_reduced(X, W, b, t)
    S = oracle.linear_xtw_reduced(X, W, b, t, absolute=True)
    err = np.abs(Y.astype(np.float64) - want)
    assert np.all(err <= TOL * S), f"max err/S = {(err / S).max():.3e}"
    full = np.abs(Y.astype(np.float64) - oracle.linear_xtw(X, W, b)) / oracle.magnitude_xtw(X, W, b)
    if dtype == jg.JG_BF16X3:
        assert full.max() <= 2.0 ** -15
    elif K >= 80:
        assert full.max() > 1e-5


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_transposed_layer_is_bit_exact_on_lattice_inputs(jg, ctx, ways, dtype_name):
    K, M, N = 528, 264, 136
    X, W = inputs.matrix(433, K, M, "L"), inputs.matrix(434, K, N, "L")
    b = inputs.matrix(435, 1, N, "L")[0]
    Y, _, _ = run_xtw(jg, ctx, X, W, b, ways, getattr(jg, dtype_name))
    assert np.array_equal(Y.astype(np.float64), oracle.linear_xtw(X, W, b))


@pytest.mark.parametrize("ways", [2, 4])
@pytest.mark.parametrize("combine,weights", [(1, 0), (0, 1), (1, 1)])
def test_transposed_layer_option_variants(jg, ctx, ways, combine, weights):
    K, M, N = 272, 130, 258
    X, W = inputs.matrix(436, K, M, "R"), inputs.matrix(437, K, N, "R", inputs.W_SCALE_EXP)
    b = inputs.matrix(438, 1, N, "R")[0]
    base, _, _ = run_xtw(jg, ctx, X, W, b, ways, jg.JG_BF16)
    Y, _, _ = run_xtw(jg, ctx, X, W, b, ways, jg.JG_BF16, combine, weights)
    S = oracle.linear_xtw_reduced(X, W, b, 1, absolute=True)
    assert np.all(np.abs(Y.astype(np.float64) - oracle.linear_xtw_reduced(X, W, b, 1)) <= TOL * S)
    if combine == 0:
        assert np.array_equal(Y, base)      # where the activation block is read from does not change the arithmetic


@pytest.mark.timeout(600)
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_transposed_layer_at_token_mixing_size(jg, capsys, dtype_name):
    """The first token-mixing linear of the 1B model (16200 tokens, 4320 channels, 8640 hidden) in reduced precision,
    in the launch configuration bench.py --op xtw --dtype ... times: whole rows of Y for sampled channels against the
    oracle, everything finite.  (The 4-way form halves 16200 tokens to 8100, not a multiple of 8: the zero padding.)"""
    from paper_2507_05753_amd.layer import JigsawLinear
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    cfg = inputs.XTW_CONFIGS["token_mixing_1b"]
    K, M, N, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    Xd = inputs.matrix_torch(seed, K, M, "R", device="cuda")
    Wd = inputs.matrix_torch(seed + inputs.W_STREAM, K, N, "R", inputs.W_SCALE_EXP, device="cuda")
    W = Wd.cpu().numpy()
    k = inputs.keys(5100, np.arange(12, dtype=np.uint64))
    I = np.unique(np.concatenate([(k % np.uint64(M)).astype(np.int64), [0, M // 2 - 1, M // 2, M - 1]]))
    Xs = np.ascontiguousarray(Xd[:, torch.from_numpy(I).cuda()].cpu().numpy())        # the sampled channels' columns
    want = oracle.linear_xtw_reduced(Xs, W, None, t)
    S = oracle.linear_xtw_reduced(Xs, W, None, t, absolute=True)
    note(capsys, f"{dtype_name} transposed layer: oracle rows ready ({I.size} channels x {N})")
    for ways in (1, 2, 4):
        with JigsawLinear(M, K, N, ways, op=jg.JG_OP_XTW, dtype=dtype) as L:
            L.ws.fill_(0xFF)
            L.shard(Xd, Wd)
            L.forward()
            Y = L.gather()
            torch.cuda.synchronize()
            assert torch.isfinite(Y).all()
            Ys = Y[torch.from_numpy(I).cuda()].cpu().numpy().astype(np.float64)
            del Y
        torch.cuda.empty_cache()
        e = (np.abs(Ys - want) / S).max()
        assert e <= TOL, (ways, e)
        note(capsys, f"{dtype_name} transposed layer ways={ways}: {Ys.size} entries max err/S {e:.2e}")


# ---------------------------------------------------------------------------------------------
# the token-mixing half of a mixing block in mixed precision
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("T,C,D", [(100, 100, 112), (130, 72, 272), (264, 136, 80), (520, 300, 1040)])
def test_mixed_precision_token_mixing_block(jg, ctx, ways, dtype_name, T, C, D):
    """Layer by layer against the oracle applied to what the GPU fed the layer (Xn and H are FP32 outputs; the
    products read their bfloat16 roundings), then loosely against the oracle's own chain."""
    from paper_2507_05753_amd.layer import JigsawTokenMixing
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    X = (inputs.matrix(450, T, C, "R") + np.float32(0.25)).astype(np.float32)
    gamma = (inputs.matrix(451, 1, C, "R")[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(452, 1, C, "R")[0]
    W1, W2 = inputs.matrix(453, T, D, "R", inputs.W_SCALE_EXP), inputs.matrix(454, T, D, "R", inputs.W_SCALE_EXP)
    b1, b2 = inputs.matrix(455, 1, D, "R")[0], inputs.matrix(456, 1, T, "R")[0]
    with JigsawTokenMixing(T, C, D, ways, ctx=ctx, dtype=dtype) as L:
        L.ws.fill_(0xFF)
        L.shard(dev(X), dev(gamma), dev(beta), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        Xn, H, Y = L.gather_xn().cpu().numpy(), L.gather_h().cpu().numpy(), L.gather().cpu().numpy()
        L.forward()                                   # the inputs were not overwritten: the same again
        assert np.array_equal(Y, L.gather().cpu().numpy())
    want = oracle.layernorm(X, gamma, beta, oracle.ln_groups(ways))
    assert np.all(np.abs(Xn.astype(np.float64) - want) <= 2.0 ** -24 * np.abs(want) * (1 + 1e-6) + 1e-10)
    S1 = oracle.linear_xtw_reduced(Xn, W1, b1, t, absolute=True)
    eh = np.abs(H.astype(np.float64) - oracle.gelu(oracle.linear_xtw_reduced(Xn, W1, b1, t)))
    assert np.all(eh <= 1.7e-6 * S1), f"H: {(eh / S1).max():.2e}"
    wantY = X.astype(np.float64) + oracle.linear_reduced(W2, H, None, t) + b2.astype(np.float64)[:, None]
    SY = np.abs(X) + oracle.linear_reduced(W2, H, None, t, absolute=True) + np.abs(b2)[:, None]
    ey = np.abs(Y.astype(np.float64) - wantY)
    assert np.all(ey <= TOL * SY), f"Y: {(ey / SY).max():.2e}"
    r = oracle.token_mixing_block_reduced(ways, X, gamma, beta, W1, b1, W2, b2, t)
    assert np.all(np.abs(Y - r["Y"]) <= 1e-4 * r["SY"])
    if t == 1:      # and it is the mixed-precision block, not the FP32 one
        assert np.abs(Y - oracle.token_mixing_block(ways, X, gamma, beta, W1, b1, W2, b2)["Y"]).max() > 1e-5


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_mixed_precision_whole_mixing_block(jg, ctx, ways, dtype_name):
    """Token half, then channel half on its FP32 output shards in place, both in mixed precision: the channel half
    against the oracle applied to what the token half produced, the whole loosely against the oracle's chain."""
    from paper_2507_05753_amd.layer import JigsawMixerBlock
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    T, C, Dt, Dc = 264, 272, 144, 208
    X = (inputs.matrix(470, T, C, "R") + np.float32(0.25)).astype(np.float32)
    vec = lambda s, n, shift=0.0: (inputs.matrix(s, 1, n, "R")[0] + np.float32(shift)).astype(np.float32)
    g1, be1, g2, be2 = vec(471, C, 1.5), vec(472, C), vec(473, C, 1.5), vec(474, C)
    W1, W2 = inputs.matrix(475, T, Dt, "R", inputs.W_SCALE_EXP), inputs.matrix(476, T, Dt, "R", inputs.W_SCALE_EXP)
    b1, b2 = vec(477, Dt), vec(478, T)
    V1, V2 = inputs.matrix(479, Dc, C, "R", inputs.W_SCALE_EXP), inputs.matrix(480, C, Dc, "R", inputs.W_SCALE_EXP)
    c1, c2 = vec(481, Dc), vec(482, C)
    with JigsawMixerBlock(T, C, Dt, Dc, ways, ctx=ctx, dtype=dtype) as L:
        L.shard(dev(X), token=dict(gamma=dev(g1), beta=dev(be1), W1=dev(W1), b1=dev(b1), W2=dev(W2), b2=dev(b2)),
                channel=dict(gamma=dev(g2), beta=dev(be2), W1=dev(V1), b1=dev(c1), W2=dev(V2), b2=dev(c2)))
        L.forward()
        U = L.gather_token_output().cpu().numpy()
        Un, G, Y = L.channel.gather_xn().cpu().numpy(), L.channel.gather_h().cpu().numpy(), L.gather().cpu().numpy()
    r1 = oracle.token_mixing_block_reduced(ways, X, g1, be1, W1, b1, W2, b2, t)
    assert np.all(np.abs(U - r1["Y"]) <= 1e-4 * r1["SY"])
    want = oracle.layernorm(U, g2, be2, oracle.ln_groups(ways))
    assert np.all(np.abs(Un.astype(np.float64) - want) <= 2.0 ** -24 * np.abs(want) * (1 + 1e-6) + 1e-10)
    check_mixed_chain(U, Un, G, Y, V1, c1, V2, c2, t)


# ---------------------------------------------------------------------------------------------
# backward of the plain layer in reduced precision
# ---------------------------------------------------------------------------------------------
# (M, K, N) below: a rank's share of N and (the plan's own rule) of K in whole 8-element chunks; M free (ragged tiles,
# token counts that the conversion pads with zeros)


def run_backward_reduced(jg, ctx, X, W, dY, ways, dtype):
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K = X.shape
    N = W.shape[0]
    with JigsawLinear(M, K, N, ways, ctx=ctx, dtype=dtype) as L:
        L.shard_master(dev(X), dev(W))
        L.shard_dy(dev(dY))
        L.bw_ws.fill_(0xFF)
        L.backward()
        dX, dW = L.gather_dx().cpu().numpy(), L.gather_dw().cpu().numpy()
        L.backward()
        assert np.array_equal(dX, L.gather_dx().cpu().numpy()) and np.array_equal(dW, L.gather_dw().cpu().numpy())
    return dX, dW


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("M,K,N", [(2, 16, 16), (100, 80, 112), (130, 144, 272), (258, 272, 144), (525, 304, 1040),
                                   (64, 1040, 48)])
def test_backward_in_reduced_precision(jg, ctx, ways, dtype_name, M, K, N):
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    if ways == 4 and M % 2:
        M += 1
    X, W, _ = inputs.layer_inputs(490, M, K, N, "R")
    X = (X * np.float32(3.0)).astype(np.float32)
    dY = inputs.matrix(491, M, N, "R")
    dX, dW = run_backward_reduced(jg, ctx, X, W, dY, ways, dtype)
    wX, wW = oracle.backward_reduced(X, W, dY, t)
    SX, SW = oracle.backward_reduced(X, W, dY, t, absolute=True)
    ex, ew = np.abs(dX - wX), np.abs(dW - wW)
    assert np.all(ex <= TOL * SX), f"dX: {(ex / np.maximum(SX, 1e-300)).max():.3e}"
    assert np.all(ew <= TOL * SW), f"dW: {(ew / np.maximum(SW, 1e-300)).max():.3e}"
    fX, fW = oracle.backward(X, W, dY)
    mX, mW = oracle.backward_magnitude(X, W, dY)
    if dtype == jg.JG_BF16X3:       # close to the full-precision backward
        assert np.all(np.abs(dX - fX) <= 2.0 ** -15 * mX) and np.all(np.abs(dW - fW) <= 2.0 ** -15 * mW)
    elif N >= 100:                  # visibly the rounded one
        assert (np.abs(dX - fX) / mX).max() > 1e-5


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_backward_in_reduced_precision_is_bit_exact_on_lattice_inputs(jg, ctx, ways, dtype_name):
    M, K, N = 132, 208, 80
    X, W, _ = inputs.layer_inputs(492, M, K, N, "L")
    dY = inputs.matrix(493, M, N, "L")
    dX, dW = run_backward_reduced(jg, ctx, X, W, dY, ways, getattr(jg, dtype_name))
    wX, wW = oracle.backward(X, W, dY)
    assert np.array_equal(dX.astype(np.float64), wX) and np.array_equal(dW.astype(np.float64), wW)


def test_backward_in_reduced_precision_checks_its_arguments(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear
    with JigsawLinear(64, 32, 20, 2, ctx=ctx, dtype=jg.JG_BF16) as L:      # N / 2 = 10: not whole chunks
        L.alloc_backward()
        p = lambda ts: [t.data_ptr() for t in ts]
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_linear_backward(L.plan, p(L.x32), p(L.w32), p(L.dy), p(L.dx), p(L.dw), L.bw_ws.data_ptr(), L.bw_ws_bytes)
        assert e.value.status == jg.JG_E_SHAPE
    with JigsawLinear(64, 32, 32, 2, ctx=ctx, dtype=jg.JG_BF16) as L:
        L.alloc_backward()
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_linear_backward(L.plan, p(L.x32), p(L.w32), p(L.dy), p(L.dx), p(L.dw), L.bw_ws.data_ptr(), L.bw_ws_bytes - 1)
        assert e.value.status == jg.JG_E_WORKSPACE
    with JigsawLinear(20, 64, 32, 2, ctx=ctx, dtype=jg.JG_BF16, op=jg.JG_OP_XTW) as L:      # M / 2 = 10 channels
        L.alloc_backward()
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_linear_backward(L.plan, p(L.x32), p(L.w32), p(L.dy), p(L.dx), p(L.dw), L.bw_ws.data_ptr(), L.bw_ws_bytes)
        assert e.value.status == jg.JG_E_SHAPE


@pytest.mark.timeout(900)
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_backward_in_reduced_precision_at_config3(jg, capsys, dtype_name):
    """Config 3 at full size, in the launch configuration bench.py --op backward --dtype ... times: whole rows of dX
    for sampled tokens and whole rows of dW for sampled output channels against the oracle, everything finite."""
    from paper_2507_05753_amd.layer import JigsawLinear
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    cfg = inputs.CONFIGS[3]
    M, K, N, seed = cfg["M"], cfg["K"], cfg["N"], cfg["seed"]
    Xd = inputs.matrix_torch(seed, M, K, cfg["x_mode"], device="cuda")
    Wd = inputs.matrix_torch(seed + inputs.W_STREAM, N, K, "R", inputs.W_SCALE_EXP, device="cuda")
    dYd = inputs.matrix_torch(seed + 3000, M, N, "R", device="cuda")
    k = inputs.keys(5200, np.arange(24, dtype=np.uint64))
    rows = np.unique(np.concatenate([(k[:12] % np.uint64(M)).astype(np.int64), [0, M // 2 - 1, M // 2, M - 1]]))
    outs = np.unique(np.concatenate([(k[12:] % np.uint64(N)).astype(np.int64), [0, N // 2 - 1, N // 2, N - 1]]))
    ri, oi = torch.from_numpy(rows).cuda(), torch.from_numpy(outs).cuda()
    W = Wd.cpu().numpy()
    dY_r = dYd[ri].cpu().numpy()
    # dX rows: rnd(dY[rows]) rnd(W);  dW rows: rnd(dY[:, outs])^T rnd(X) - both are A B^T products of the forward oracle
    wantX = oracle.linear_reduced(dY_r, np.ascontiguousarray(W.T), None, t)
    SX = oracle.linear_reduced(dY_r, np.ascontiguousarray(W.T), None, t, absolute=True)
    dYt = np.ascontiguousarray(dYd[:, oi].cpu().numpy().T)
    Xt = np.ascontiguousarray(Xd.cpu().numpy().T)
    wantW = oracle.linear_reduced(dYt, Xt, None, t)
    SW = oracle.linear_reduced(dYt, Xt, None, t, absolute=True)
    del Xt
    note(capsys, f"{dtype_name} backward: oracle rows ready ({rows.size} tokens of dX, {outs.size} rows of dW)")
    for ways in (1, 4):
        with JigsawLinear(M, K, N, ways, dtype=dtype) as L:
            L.shard_master(Xd, Wd)
            L.shard_dy(dYd)
            L.bw_ws.fill_(0xFF)
            L.backward()
            dX, dW = L.gather_dx(), L.gather_dw()
            torch.cuda.synchronize()
            assert torch.isfinite(dX).all() and torch.isfinite(dW).all()
            dXs, dWs = dX[ri].cpu().numpy().astype(np.float64), dW[oi].cpu().numpy().astype(np.float64)
            del dX, dW
        torch.cuda.empty_cache()
        ex, ew = (np.abs(dXs - wantX) / SX).max(), (np.abs(dWs - wantW) / SW).max()
        assert ex <= TOL and ew <= TOL, (ways, ex, ew)
        note(capsys, f"{dtype_name} backward ways={ways}: dX max err/S {ex:.2e} ({dXs.size} entries), dW {ew:.2e} ({dWs.size})")


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("K,M,N", [(2, 16, 16), (100, 112, 80), (130, 272, 144), (258, 144, 272), (521 * 2, 304, 1040)])
def test_backward_of_the_transposed_layer_in_reduced_precision(jg, ctx, ways, dtype_name, K, M, N):
    """dX = rnd(W) rnd(dY)^T and dW = rnd(X) rnd(dY): 1e-6 * S against the oracle (K = tokens, any count; a rank's
    share of the channels M and of the columns N in whole 8-element chunks)."""
    from paper_2507_05753_amd.layer import JigsawLinear
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    X = (inputs.matrix(495, K, M, "R") * np.float32(3.0)).astype(np.float32)
    W = inputs.matrix(496, K, N, "R", inputs.W_SCALE_EXP)
    dY = inputs.matrix(497, M, N, "R")
    with JigsawLinear(M, K, N, ways, ctx=ctx, dtype=dtype, op=jg.JG_OP_XTW) as L:
        L.shard_master(dev(X), dev(W))
        L.shard_dy(dev(dY))
        L.bw_ws.fill_(0xFF)
        L.backward()
        dX, dW = L.gather_dx().cpu().numpy(), L.gather_dw().cpu().numpy()
        L.backward()
        assert np.array_equal(dX, L.gather_dx().cpu().numpy()) and np.array_equal(dW, L.gather_dw().cpu().numpy())
    wX, wW = oracle.backward_xtw_reduced(X, W, dY, t)
    SX, SW = oracle.backward_xtw_reduced(X, W, dY, t, absolute=True)
    ex, ew = np.abs(dX - wX), np.abs(dW - wW)
    assert np.all(ex <= TOL * SX), f"dX: {(ex / np.maximum(SX, 1e-300)).max():.3e}"
    assert np.all(ew <= TOL * SW), f"dW: {(ew / np.maximum(SW, 1e-300)).max():.3e}"
    XL, WL, GL = inputs.matrix(498, K, M, "L"), inputs.matrix(499, K, N, "L"), inputs.matrix(500, M, N, "L")
    with JigsawLinear(M, K, N, ways, ctx=ctx, dtype=dtype, op=jg.JG_OP_XTW) as L:
        L.shard_master(dev(XL), dev(WL))
        L.shard_dy(dev(GL))
        L.backward()
        eX, eW = oracle.backward_xtw(XL, WL, GL)
        assert np.array_equal(L.gather_dx().cpu().numpy().astype(np.float64), eX)
        assert np.array_equal(L.gather_dw().cpu().numpy().astype(np.float64), eW)


@pytest.mark.parametrize("ways", [1, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
def test_mixed_precision_whole_mixing_block_backward(jg, ctx, ways, dtype_name):
    """Backward of a whole mixing block in mixed precision: the channel half's, then the token half's on its FP32 dX
    shards in place; the halves are checked step by step in their own tests, here the chain against the oracle's."""
    from paper_2507_05753_amd.layer import JigsawMixerBlock
    dtype = getattr(jg, dtype_name)
    t = terms_of(jg, dtype)
    T, C, Dt, Dc = 264, 272, 144, 208
    X = (inputs.matrix(520, T, C, "R") + np.float32(0.25)).astype(np.float32)
    vec = lambda s, n, shift=0.0: (inputs.matrix(s, 1, n, "R")[0] + np.float32(shift)).astype(np.float32)
    g1, be1, g2, be2 = vec(521, C, 1.5), vec(522, C), vec(523, C, 1.5), vec(524, C)
    W1, W2 = inputs.matrix(525, T, Dt, "R", inputs.W_SCALE_EXP), inputs.matrix(526, T, Dt, "R", inputs.W_SCALE_EXP)
    b1, b2 = vec(527, Dt), vec(528, T)
    V1, V2 = inputs.matrix(529, Dc, C, "R", inputs.W_SCALE_EXP), inputs.matrix(530, C, Dc, "R", inputs.W_SCALE_EXP)
    c1, c2 = vec(531, Dc), vec(532, C)
    dY = inputs.matrix(533, T, C, "R")
    with JigsawMixerBlock(T, C, Dt, Dc, ways, ctx=ctx, dtype=dtype, keep_masters=True) as L:
        L.shard(dev(X), token=dict(gamma=dev(g1), beta=dev(be1), W1=dev(W1), b1=dev(b1), W2=dev(W2), b2=dev(b2)),
                channel=dict(gamma=dev(g2), beta=dev(be2), W1=dev(V1), b1=dev(c1), W2=dev(V2), b2=dev(c2)))
        L.forward()
        L.backward(dev(dY))
        dX = L.gather_dx().cpu().numpy()
        dW1, dV2 = L.token.gather_grad("dw1").cpu().numpy(), L.channel.gather_grad("dw2").cpu().numpy()
        mid = L.channel.gather_grad("dx")
        L.token.backward(mid)                        # the same gradient, sharded from the gathered matrix: the same bits
        assert np.array_equal(dX, L.gather_dx().cpu().numpy())
    U = oracle.token_mixing_block_reduced(ways, X, g1, be1, W1, b1, W2, b2, t)["Y"].astype(np.float32)
    rc = oracle.mixing_block_backward_reduced(ways, U, g2, be2, V1, c1, V2, dY, t)
    rt = oracle.token_mixing_block_backward_reduced(ways, X, g1, be1, W1, b1, W2, rc["dX"].astype(np.float32), t)
    loose = 3e-3 if t == 1 else 1e-4
    for got, ref, name in ((dX, rt["dX"], "dX"), (dW1, rt["dW1"], "dW1"), (dV2, rc["dW2"], "dV2")):
        assert np.all(np.abs(got - ref) <= loose * (np.abs(ref) + np.abs(ref).max())), name
