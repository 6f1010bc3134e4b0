"""GPU parity of the fused epilogue (bias, GELU, residual) and of the mixing MLP against the CPU oracle.

Bars: the linear part as everywhere (1e-6 of the summand magnitude).  Through GELU an error e in the
pre-activation shows as at most 1.13 |e| (the largest slope of x Phi(x)), and the FP32 erf adds about
1e-7 of |x| <= S1; the product itself stays near 1e-7 * S1, so H is held to the layer's own 1e-6 * S1.  In Y that error is carried by |W2| (PY = S1 |W2|^T):
|Y - Y64| <= 1e-6 * SY + 1e-6 * PY.  Without an activation, lattice inputs stay bit-exact.
"""
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2507_05753_amd import inputs

pytestmark = pytest.mark.gpu
TOL = 1e-6
TOL_H = 1e-6


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


def run_ex(jg, ctx, X, W, b, R, act, ways, combine=0, op=0):
    """shard -> jg_linear_forward_ex -> gather; R is a global residual (shaped like Y) or None."""
    from paper_2507_05753_amd.layer import JigsawLinear
    if op == jg.JG_OP_XTW:
        K, M = X.shape
        N = W.shape[1]
    else:
        M, K = X.shape
        N = W.shape[0]
    with JigsawLinear(M, K, N, ways, bias=b is not None, combine=combine, ctx=ctx, op=op) as L:
        L.ws.fill_(0xFF)
        L.shard(dev(X), dev(W), dev(b) if b is not None else None)
        res = None
        if R is not None:
            res = [torch.empty_like(y) for y in L.y]
            jg.jg_shard(L.plan, jg.JG_T_Y, dev(R).data_ptr(), N, [t.data_ptr() for t in res])
        L.forward(residual=res, activation=act)
        Y = L.gather()
        torch.cuda.synchronize()
        return Y.cpu().numpy()


SHAPES = [(100, 100, 100), (130, 72, 258), (258, 200, 136), (300, 1032, 260), (130, 4160, 258)]   # last: split tail


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_gelu_epilogue(jg, ctx, ways, M, K, N):
    X, W, b = inputs.layer_inputs(51, M, K, N, "R", bias=True)
    b = (b * 0.5).astype(np.float32)
    H = run_ex(jg, ctx, X, W, b, None, jg.JG_ACT_GELU, ways)
    want = oracle.gelu(oracle.linear(X, W, b))
    S = oracle.magnitude(X, W, b)
    err = np.abs(H.astype(np.float64) - want)
    assert np.all(err <= TOL_H * S), f"max err/S = {(err / S).max():.3e}"
    # the activation was really applied: it differs from the linear output by far more than the bar
    assert np.abs(want - oracle.linear(X, W, b)).max() > 1e-2


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", SHAPES)
def test_residual_epilogue_is_bit_exact_on_lattice_inputs(jg, ctx, ways, M, K, N):
    X, W, b = inputs.layer_inputs(52, M, K, N, "L", bias=True)
    R = inputs.matrix(53, M, N, "L")
    Y = run_ex(jg, ctx, X, W, b, R, jg.JG_ACT_NONE, ways)
    want = oracle.linear(X, W, b) + R.astype(np.float64)
    assert np.array_equal(Y.astype(np.float64), want)


@pytest.mark.parametrize("ways", [2, 4])
def test_separate_combine_and_transposed_layer_take_the_same_epilogue(jg, ctx, ways):
    M, K, N = 258, 200, 136
    X, W, b = inputs.layer_inputs(54, M, K, N, "R", bias=True)
    R = inputs.matrix(55, M, N, "R")
    fused = run_ex(jg, ctx, X, W, b, R, jg.JG_ACT_GELU, ways)
    sep = run_ex(jg, ctx, X, W, b, R, jg.JG_ACT_GELU, ways, combine=jg.JG_COMBINE_SEPARATE)
    want = oracle.gelu(oracle.linear(X, W, b)) + R.astype(np.float64)
    S = oracle.magnitude(X, W, b) + np.abs(R)
    for got in (fused, sep):
        assert np.all(np.abs(got.astype(np.float64) - want) <= TOL_H * S)
    # transposed layer: X [K x M], W [K x N]
    Xt = inputs.matrix(56, 200, 264, "R")
    Wt = inputs.matrix(57, 200, 136, "R", inputs.W_SCALE_EXP)
    bt = inputs.matrix(58, 1, 136, "R")[0]
    Rt = inputs.matrix(59, 264, 136, "R")
    got = run_ex(jg, ctx, Xt, Wt, bt, Rt, jg.JG_ACT_GELU, ways, op=jg.JG_OP_XTW)
    want = oracle.gelu(oracle.linear_xtw(Xt, Wt, bt)) + Rt.astype(np.float64)
    S = oracle.magnitude_xtw(Xt, Wt, bt) + np.abs(Rt)
    assert np.all(np.abs(got.astype(np.float64) - want) <= TOL_H * S)


def mlp_operands(seed, M, C, Hd, mode="R"):
    X = inputs.matrix(seed, M, C, mode)
    W1 = inputs.matrix(seed + 1, Hd, C, mode, inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, Hd, mode)[0]
    W2 = inputs.matrix(seed + 3, C, Hd, mode, inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 4, 1, C, mode)[0]
    return X, W1, b1, W2, b2


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,C,Hd", [(100, 100, 100), (130, 72, 258), (258, 264, 136), (300, 520, 1032)])
def test_mlp_forward(jg, ctx, ways, M, C, Hd):
    from paper_2507_05753_amd.layer import JigsawMLP
    X, W1, b1, W2, b2 = mlp_operands(60, M, C, Hd)
    with JigsawMLP(M, C, Hd, ways, ctx=ctx) as L:
        Xd = dev(X)
        L.shard(Xd, dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        H, Y = L.gather_h().cpu().numpy(), L.gather().cpu().numpy()
        L.forward()                                      # X was not overwritten: the same again
        assert np.array_equal(Y, L.gather().cpu().numpy())
        assert torch.equal(Xd.cpu(), torch.from_numpy(X))
    r = oracle.mlp(X, W1, b1, W2, b2)
    eh = np.abs(H.astype(np.float64) - r["H"])
    assert np.all(eh <= TOL_H * r["S1"]), f"H: max err/S1 = {(eh / r['S1']).max():.3e}"
    ey = np.abs(Y.astype(np.float64) - r["Y"])
    bound = TOL * r["SY"] + TOL_H * r["PY"]
    assert np.all(ey <= bound), f"Y: max err/bound = {(ey / bound).max():.3e}"
    # the second layer on its own, at the usual bar: from the H the GPU produced
    want2 = oracle.linear(H, W2, b2) + X.astype(np.float64)
    S2 = oracle.magnitude(H, W2, b2) + np.abs(X)
    assert np.all(np.abs(Y.astype(np.float64) - want2) <= TOL * S2)


def test_mlp_plans_must_chain(jg, ctx):
    a = jg.jg_plan_create(ctx, 64, 32, 48, 2, True)
    good = jg.jg_plan_create(ctx, 64, 48, 32, 2, True)
    ptr = [256, 512]
    for bad_args, status in ((dict(M=64, K=48, N=30), jg.JG_E_SHAPE), (dict(M=62, K=48, N=32), jg.JG_E_SHAPE),
                             (dict(M=64, K=40, N=32), jg.JG_E_SHAPE)):
        b = jg.jg_plan_create(ctx, bad_args["M"], bad_args["K"], bad_args["N"], 2, True)
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_mlp_forward(a, b, ptr, ptr, ptr, ptr, ptr, ptr, ptr, None, 0)
        assert e.value.status == status
        jg.jg_plan_destroy(b)
    b = jg.jg_plan_create(ctx, 64, 48, 32, 4, True)
    with pytest.raises(jg.JigsawError) as e:
        jg.jg_mlp_forward(a, b, ptr, ptr, ptr, ptr, ptr, ptr, ptr, None, 0)
    assert e.value.status == jg.JG_E_WAYS
    with pytest.raises(jg.JigsawError) as e:
        jg.jg_linear_forward_ex(good, ptr, ptr, ptr, None, 7, ptr, None, 0)
    assert e.value.status == jg.JG_E_DTYPE
    for p in (a, good, b):
        jg.jg_plan_destroy(p)


# --------------------------------------------------------------------------------------------
# full size: the channel-mixing MLP of the paper's 1-billion-parameter model (Sec. 6.2.1: embedding
# dimension 4320, channel-mixing hidden dimension 4320) over 16200 tokens
# --------------------------------------------------------------------------------------------
def note(capsys, msg):
    with capsys.disabled():
        print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


@pytest.mark.timeout(600)
def test_channel_mixing_size(jg, capsys):
    from paper_2507_05753_amd.layer import JigsawMLP
    cfg = inputs.MLP_CONFIGS["channel_mixing_1b"]
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    Xd = inputs.matrix_torch(seed, M, C, "R", device="cuda")
    W1 = inputs.matrix(seed + 1, Hd, C, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, Hd, "R")[0]
    W2 = inputs.matrix(seed + 3, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 4, 1, C, "R")[0]
    k = inputs.keys(6000, np.arange(96, dtype=np.uint64))
    rows = np.unique(np.concatenate([(k % np.uint64(M)).astype(np.int64), [0, M // 2 - 1, M // 2, M - 1]]))
    Xs = inputs.matrix_rows(seed, C, rows, "R")
    assert np.array_equal(Xd[torch.from_numpy(rows).cuda()].cpu().numpy(), Xs)
    r = oracle.mlp(Xs, W1, b1, W2, b2)          # whole rows of H and Y for the sampled tokens
    note(capsys, f"channel mixing: oracle rows ready ({rows.size} tokens)")
    W1d, b1d, W2d, b2d = dev(W1), dev(b1), dev(W2), dev(b2)
    for ways in (1, 2, 4):
        with JigsawMLP(M, C, Hd, ways) as L:
            L.ws.fill_(0xFF)
            L.shard(Xd, W1d, b1d, W2d, b2d)
            L.forward()
            H, Y = L.gather_h(), L.gather()
            torch.cuda.synchronize()
            assert torch.isfinite(H).all() and torch.isfinite(Y).all()
            idx = torch.from_numpy(rows).cuda()
            H32 = H[idx].cpu().numpy()
            Hs, Ys = H32.astype(np.float64), Y[idx].cpu().numpy().astype(np.float64)
            del H, Y
        torch.cuda.empty_cache()
        eh = np.abs(Hs - r["H"]) / r["S1"]
        ey = np.abs(Ys - r["Y"]) / (TOL * r["SY"] + TOL_H * r["PY"])
        assert eh.max() <= TOL_H and ey.max() <= 1.0, (ways, eh.max(), ey.max())
        e2 = np.abs(Ys - (oracle.linear(H32, W2, b2) + Xs)) / (oracle.magnitude(H32, W2, b2) + np.abs(Xs))
        assert e2.max() <= TOL, (ways, e2.max())      # the second layer alone, from the GPU's own H
        note(capsys, f"channel mixing ways={ways}: H max err/S1 {eh.max():.2e}, layer 2 max err/S {e2.max():.2e}, Y max err/bound {ey.max():.2e} "
                     f"({rows.size} x {C} entries each)")


# ---------------------------------------------------------------------------------------------
# backward of the MLP: the chain rule through the layers' backward passes, checked step by step
# ---------------------------------------------------------------------------------------------
def check_mlp_backward(L, X, W1, b1, W2, dY, ways, xkey="dx", t=0):
    """xkey "dx": the MLP with its skip connection; "dxn": the MLP inside a block, dA W1 alone.  t: 0 for FP32 plans,
    1 / 3 for the mixed-precision modes (every product against the oracle's reduced routine)."""
    lin = (lambda a, w, b: oracle.linear_reduced(a, w, b, t)) if t else oracle.linear
    lin_mag = (lambda a, w, b: oracle.linear_reduced(a, w, b, t, absolute=True)) if t else oracle.magnitude
    bwd = (lambda a, w, g_: oracle.backward_reduced(a, w, g_, t)) if t else oracle.backward
    bwd_mag = (lambda a, w, g_: oracle.backward_reduced(a, w, g_, t, absolute=True)) if t else oracle.backward_magnitude
    g = {k: L.gather_grad(k).cpu().numpy() for k in ("a", "dh", "da", xkey, "dw1", "dw2", "db1", "db2")}
    H = L.gather_h().cpu().numpy()
    f64 = lambda a: a.astype(np.float64)
    rel = lambda err, S: (err / np.maximum(S, 1e-300)).max()
    # A recomputed: one forward layer
    A64, SA = lin(X, W1, b1), lin_mag(X, W1, b1)
    assert np.all(np.abs(f64(g["a"]) - A64) <= 1e-6 * SA), f"A: {rel(np.abs(f64(g['a']) - A64), SA):.2e}"
    # second layer's backward from the H the forward stored
    dH64, dW264 = bwd(H, W2, dY)
    SH, SW2 = bwd_mag(H, W2, dY)
    assert np.all(np.abs(f64(g["dh"]) - dH64) <= 1e-6 * SH), f"dH: {rel(np.abs(f64(g['dh']) - dH64), SH):.2e}"
    assert np.all(np.abs(f64(g["dw2"]) - dW264) <= 1e-6 * SW2), f"dW2: {rel(np.abs(f64(g['dw2']) - dW264), SW2):.2e}"
    db2 = oracle.bias_backward(dY)
    assert np.all(np.abs(f64(g["db2"]) - db2) <= 2.0 ** -23 * np.abs(db2) + 1e-12 * oracle.bias_backward(dY, absolute=True))
    # dA from the A and dH the GPU stored: evaluated in double, rounded once
    dA64 = f64(g["dh"]) * oracle.gelu_grad(f64(g["a"]))
    assert np.all(np.abs(f64(g["da"]) - dA64) <= 2.0 ** -23 * np.abs(dA64) + 1e-45), "dA"
    # first layer's backward from the dA the GPU stored, plus the skip connection
    dX64, dW164 = bwd(X, W1, g["da"])
    SX, SW1 = bwd_mag(X, W1, g["da"])
    skip = f64(dY) if xkey == "dx" else 0.0
    ex = np.abs(f64(g[xkey]) - (dX64 + skip))
    assert np.all(ex <= 1e-6 * (SX + np.abs(skip))), f"{xkey}: {rel(ex, SX + np.abs(skip)):.2e}"
    assert np.all(np.abs(f64(g["dw1"]) - dW164) <= 1e-6 * SW1), f"dW1: {rel(np.abs(f64(g['dw1']) - dW164), SW1):.2e}"
    db1 = oracle.bias_backward(g["da"])
    assert np.all(np.abs(f64(g["db1"]) - db1) <= 2.0 ** -23 * np.abs(db1) + 1e-12 * oracle.bias_backward(g["da"], absolute=True))
    return g


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,C,Hd", [(100, 100, 100), (130, 72, 258), (258, 264, 136), (300, 520, 1032)])
def test_mlp_backward(jg, ctx, ways, M, C, Hd):
    from paper_2507_05753_amd.layer import JigsawMLP
    X, W1, b1 = inputs.layer_inputs(350, M, C, Hd, "R", bias=True)
    W2 = inputs.matrix(351, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(352, 1, C, "R")[0]
    dY = inputs.matrix(353, M, C, "R")
    with JigsawMLP(M, C, Hd, ways, ctx=ctx) as L:
        L.shard(dev(X), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        L.backward(dev(dY))
        g = check_mlp_backward(L, X, W1, b1, W2, dY, ways)
        L.backward(dev(dY))                                    # nothing it reads was overwritten: the same again
        assert np.array_equal(g["dx"], L.gather_grad("dx").cpu().numpy())
        assert np.array_equal(g["dw1"], L.gather_grad("dw1").cpu().numpy())
    # end to end against the oracle's own chain (A is recomputed in FP32 here, in double there)
    r = oracle.mlp_backward(X, W1, b1, W2, dY)
    for name in ("dx", "dw1", "dw2"):
        ref = r["dX" if name == "dx" else "dW1" if name == "dw1" else "dW2"]
        assert np.all(np.abs(g[name] - ref) <= 1e-4 * (np.abs(ref) + np.abs(ref).max())), name


@pytest.mark.parametrize("ways", [1, 4])
def test_gelu_derivative_over_its_range(jg, ctx, ways):
    """dA = dH * gelu'(A) with A chosen column by column: X = 0 makes the recomputed pre-activation equal to b1 exactly,
    and b1 sweeps [-5.8, 5.8] (the kernel's table of Taylor polynomials for erf), every float within 250 units in the
    last place of the derivative's root near -0.7518 (where Phi(x) and x phi(x) cancel and the bar of one rounding of
    the exact product is hardest), and the tails up to +-6.3 (the library's erf; further out 1 + erf(x / sqrt 2) has
    too few bits left for two libraries to agree to a rounding of the product).  Checked against the oracle on the A
    and dH the GPU stored, to one rounding; an infinite or NaN pre-activation gives NaN, as the definition does."""
    from paper_2507_05753_amd.layer import JigsawMLP
    root = np.float32(-0.7517916)
    near = [root]
    for _ in range(250):
        near.append(np.nextafter(near[-1], np.float32(-1)))
    lo = root
    for _ in range(249):
        lo = np.nextafter(lo, np.float32(0))
        near.append(lo)
    b1 = np.concatenate([np.linspace(-5.8, 5.8, 1500).astype(np.float32), np.array(near, dtype=np.float32),
                         np.linspace(-6.3, -5.8, 24).astype(np.float32), np.linspace(5.8, 6.3, 24).astype(np.float32)])
    Hd = b1.size
    assert Hd == 2048
    M, C = 64, 64
    X = np.zeros((M, C), dtype=np.float32)
    W1 = inputs.matrix(356, Hd, C, "R", inputs.W_SCALE_EXP)
    W2 = inputs.matrix(357, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(358, 1, C, "R")[0]
    dY = inputs.matrix(359, M, C, "R")
    f64 = lambda a: a.astype(np.float64)
    with JigsawMLP(M, C, Hd, ways, ctx=ctx) as L:
        L.shard(dev(X), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        L.backward(dev(dY))
        A, dH, dA = (L.gather_grad(k).cpu().numpy() for k in ("a", "dh", "da"))
        assert np.array_equal(A, np.broadcast_to(b1, (M, Hd)))
        want = f64(dH) * oracle.gelu_grad(f64(A))
        assert np.all(np.abs(f64(dA) - want) <= 2.0 ** -23 * np.abs(want) + 1e-45), \
            float((np.abs(f64(dA) - want) / np.maximum(np.abs(want), 1e-300)).max())
        assert np.count_nonzero(dA) > 0.99 * dA.size
        # non-finite pre-activations
        b1n = b1.copy()
        b1n[[3, 700, 1501]] = [np.inf, -np.inf, np.nan]
        L.shard(None, None, dev(b1n), None, None)
        L.forward()
        L.backward(dev(dY))
        dAn = L.gather_grad("da").cpu().numpy()
        assert np.isnan(dAn[:, [3, 700, 1501]]).all()
        keep = np.delete(np.arange(Hd), [3, 700, 1501])
        assert np.array_equal(dAn[:, keep], dA[:, keep])


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,C,Hd", [(100, 100, 100), (130, 72, 258), (258, 264, 136), (300, 520, 1032)])
def test_mixing_block_backward(jg, ctx, ways, M, C, Hd):
    from paper_2507_05753_amd.layer import JigsawMixing
    X, W1, b1 = inputs.layer_inputs(360, M, C, Hd, "R", bias=True)
    X = (X + np.float32(0.25)).astype(np.float32)
    W2 = inputs.matrix(361, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(362, 1, C, "R")[0]
    dY = inputs.matrix(363, M, C, "R")
    gamma = (inputs.matrix(364, 1, C, "R")[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(365, 1, C, "R")[0]
    HALF_ULP = 2.0 ** -24
    with JigsawMixing(M, C, Hd, ways, ctx=ctx) as L:
        L.shard(dev(X), dev(gamma), dev(beta), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        L.backward(dev(dY))
        Xn = L.gather_xn().cpu().numpy()
        # the MLP's chain on the Xn the forward stored, without a skip connection of its own
        g = check_mlp_backward(L, Xn, W1, b1, W2, dY, ways, xkey="dxn")
        # the norm's backward from the dXn the GPU stored, the block's skip connection added before the rounding
        dXl, dg, db, SX, Sg, Sb = oracle.layernorm_backward(X, gamma, g["dxn"], oracle.ln_groups(ways), magnitude=True)
        want = dY.astype(np.float64) + dXl
        dx = L.gather_grad("dx").cpu().numpy()
        assert np.all(np.abs(dx - want) <= HALF_ULP * np.abs(want) * (1 + 1e-6) + 1e-11 * (SX + np.abs(dY)) + 1e-45)
        dgam, dbet = L.dgamma.cpu().numpy(), L.dbeta.cpu().numpy()
        assert np.all(np.abs(dgam - dg) <= HALF_ULP * np.abs(dg) * (1 + 1e-6) + 1e-11 * Sg + 1e-45)
        assert np.all(np.abs(dbet - db) <= HALF_ULP * np.abs(db) * (1 + 1e-6) + 1e-11 * Sb + 1e-45)
        L.backward(dev(dY))                                    # nothing it reads was overwritten: the same again
        assert np.array_equal(dx, L.gather_grad("dx").cpu().numpy())
        assert np.array_equal(dgam, L.dgamma.cpu().numpy())
    # end to end against the oracle's own chain (Xn and A in FP32 here differ in the last bits from the oracle's)
    r = oracle.mixing_block_backward(ways, X, gamma, beta, W1, b1, W2, dY)
    for got, name in ((dx, "dX"), (g["dw1"], "dW1"), (g["dw2"], "dW2"), (dgam, "dgamma"), (dbet, "dbeta")):
        ref = r[name]
        assert np.all(np.abs(got - ref) <= 1e-4 * (np.abs(ref) + np.abs(ref).max())), name


@pytest.mark.timeout(900)
def test_mixing_block_backward_size(jg, capsys):
    """The channel-mixing block's backward at the 1B model's size, in the launch configuration bench.py --op
    mixing_backward times.  Per sampled token every step of the chain (whole rows of A, dH, dA, dXn, dX) against the
    oracle applied to what the GPU stored for the step before; sampled entries of dW1 and dW2 (sums over all tokens),
    the bias gradients and the norm's parameter gradients in full."""
    from paper_2507_05753_amd.layer import JigsawMixing
    cfg = inputs.MLP_CONFIGS["channel_mixing_1b"]
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    gen = lambda s, r, c, e=0: inputs.matrix_torch(s, r, c, "R", e, device="cuda")
    Xd, dYd = gen(seed, M, C) + 0.25, gen(seed + 7, M, C)
    W1d, W2d = gen(seed + 1, Hd, C, inputs.W_SCALE_EXP), gen(seed + 3, C, Hd, inputs.W_SCALE_EXP)
    b1d, b2d = gen(seed + 2, 1, Hd)[0].contiguous(), gen(seed + 4, 1, C)[0].contiguous()
    gammad, betad = (gen(seed + 5, 1, C)[0] + 1.5).contiguous(), gen(seed + 6, 1, C)[0].contiguous()
    W1, b1, W2, gamma = W1d.cpu().numpy(), b1d.cpu().numpy(), W2d.cpu().numpy(), gammad.cpu().numpy()
    X, dY = Xd.cpu().numpy(), dYd.cpu().numpy()
    k = inputs.keys(6100, np.arange(64, dtype=np.uint64))
    rows = np.unique(np.concatenate([(k[:24] % np.uint64(M)).astype(np.int64), [0, M // 2 - 1, M // 2, M - 1]]))
    cs = np.unique(np.concatenate([(k[24:44] % np.uint64(C)).astype(np.int64), [0, C // 2 - 1, C // 2, C - 1]]))
    hs = np.unique(np.concatenate([(k[44:] % np.uint64(Hd)).astype(np.int64), [0, Hd // 2 - 1, Hd // 2, Hd - 1]]))
    ri, ci, hi = (torch.from_numpy(v).cuda() for v in (rows, cs, hs))
    f64 = lambda a: a.astype(np.float64)
    HALF = 2.0 ** -24
    T = lambda a: np.ascontiguousarray(a.T)
    for ways in (1, 4):
        with JigsawMixing(M, C, Hd, ways) as L:
            L.shard(Xd, gammad, betad, W1d, b1d, W2d, b2d)
            L.forward()
            L.backward(dYd)
            torch.cuda.synchronize()
            Xn, H = L.gather_xn(), L.gather_h()
            full = {}
            for name in ("a", "dh", "da", "dxn", "dx", "dw1", "dw2"):
                t = L.gather_grad(name)
                assert torch.isfinite(t).all(), name
                full[name] = t
            g = {n: full[n][ri].cpu().numpy() for n in ("a", "dh", "da", "dxn", "dx")}
            Xn_r, H_r = Xn[ri].cpu().numpy(), H[ri].cpu().numpy()
            dA_h, Xn_c = full["da"][:, hi].cpu().numpy(), Xn[:, ci].cpu().numpy()       # columns over all tokens
            H_h, dY_c = H[:, hi].cpu().numpy(), dY[:, cs]
            dW1_s = full["dw1"][hi][:, ci].cpu().numpy()
            dW2_s = full["dw2"][ci][:, hi].cpu().numpy()
            dA_full, dXn_full = full["da"].cpu().numpy(), full["dxn"].cpu().numpy()
            db1, db2 = L.gather_grad("db1").cpu().numpy(), L.gather_grad("db2").cpu().numpy()
            dgam, dbet = L.dgamma.cpu().numpy(), L.dbeta.cpu().numpy()
            del full, Xn, H
        torch.cuda.empty_cache()
        worst = {}

        def within(name, got, want, S, tol=TOL):
            e = (np.abs(f64(got) - want) / np.maximum(S, 1e-300)).max()
            worst[name] = e
            assert e <= tol, (ways, name, e)
        # per sampled token, step by step
        within("A", g["a"], oracle.linear(Xn_r, W1, b1), oracle.magnitude(Xn_r, W1, b1))
        within("dH", g["dh"], oracle.backward(H_r, W2, dY[rows])[0], oracle.backward_magnitude(H_r, W2, dY[rows])[0])
        dA = f64(g["dh"]) * oracle.gelu_grad(f64(g["a"]))
        assert np.all(np.abs(f64(g["da"]) - dA) <= 2.0 ** -23 * np.abs(dA) + 1e-45), (ways, "dA")
        within("dXn", g["dxn"], oracle.backward(Xn_r, W1, g["da"])[0], oracle.backward_magnitude(Xn_r, W1, g["da"])[0])
        dXl, _, _, SX, _, _ = oracle.layernorm_backward(X[rows], gamma, g["dxn"], oracle.ln_groups(ways), magnitude=True)
        want = f64(dY[rows]) + dXl
        assert np.all(np.abs(f64(g["dx"]) - want) <= HALF * np.abs(want) * (1 + 1e-6) + 1e-11 * (SX + np.abs(dY[rows]))), (ways, "dX")
        # sampled entries of the weight gradients: sums over all tokens of what the GPU stored
        within("dW1", dW1_s, oracle.linear(T(dA_h), T(Xn_c)), oracle.magnitude(T(dA_h), T(Xn_c)))
        within("dW2", dW2_s, oracle.linear(T(dY_c), T(H_h)), oracle.magnitude(T(dY_c), T(H_h)))
        # sums over all tokens, in full
        for name, got, src in (("db1", db1, dA_full), ("db2", db2, dY)):
            want, S = oracle.bias_backward(src), oracle.bias_backward(src, absolute=True)
            assert np.all(np.abs(f64(got) - want) <= HALF * np.abs(want) * (1 + 1e-6) + 1e-11 * S), (ways, name)
        _, dg, db, _, Sg, Sb = oracle.layernorm_backward(X, gamma, dXn_full, oracle.ln_groups(ways), magnitude=True)
        assert np.all(np.abs(f64(dgam) - dg) <= HALF * np.abs(dg) * (1 + 1e-6) + 1e-11 * Sg), (ways, "dgamma")
        assert np.all(np.abs(f64(dbet) - db) <= HALF * np.abs(db) * (1 + 1e-6) + 1e-11 * Sb), (ways, "dbeta")
        note(capsys, f"mixing block backward ways={ways}: {rows.size} tokens, {cs.size} x {hs.size} weight entries; max err/S "
                     + ", ".join(f"{n} {e:.2e}" for n, e in worst.items()))


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("M,C,Hd", [(100, 112, 112), (130, 80, 272), (258, 272, 144), (301, 528, 1040)])
def test_mixing_block_backward_in_mixed_precision(jg, ctx, ways, dtype_name, M, C, Hd):
    """jg_mixing_backward on reduced plans: every product against the oracle's reduced routine applied to what the GPU
    stored for the step before; the norm's step in full precision; then loosely against the oracle's own chain."""
    from paper_2507_05753_amd.layer import JigsawMixing
    dtype = getattr(jg, dtype_name)
    t = 3 if dtype == jg.JG_BF16X3 else 1
    if ways == 4 and M % 2:
        M += 1
    X, W1, b1 = inputs.layer_inputs(390, M, C, Hd, "R", bias=True)
    X = (X + np.float32(0.25)).astype(np.float32)
    W2 = inputs.matrix(391, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(392, 1, C, "R")[0]
    dY = inputs.matrix(393, M, C, "R")
    gamma = (inputs.matrix(394, 1, C, "R")[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(395, 1, C, "R")[0]
    HALF_ULP = 2.0 ** -24
    with JigsawMixing(M, C, Hd, ways, ctx=ctx, dtype=dtype) as L:
        L.keep_masters = True
        L.shard(dev(X), dev(gamma), dev(beta), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        L.backward(dev(dY))
        Xn = L.gather_xn().cpu().numpy()
        g = check_mlp_backward(L, Xn, W1, b1, W2, dY, ways, xkey="dxn", t=t)
        dXl, dg, db, SX, Sg, Sb = oracle.layernorm_backward(X, gamma, g["dxn"], oracle.ln_groups(ways), magnitude=True)
        want = dY.astype(np.float64) + dXl
        dx = L.gather_grad("dx").cpu().numpy()
        assert np.all(np.abs(dx - want) <= HALF_ULP * np.abs(want) * (1 + 1e-6) + 1e-11 * (SX + np.abs(dY)) + 1e-45)
        dgam = L.dgamma.cpu().numpy()
        assert np.all(np.abs(dgam - dg) <= HALF_ULP * np.abs(dg) * (1 + 1e-6) + 1e-11 * Sg + 1e-45)
        L.backward(dev(dY))
        assert np.array_equal(dx, L.gather_grad("dx").cpu().numpy())
    # (an FP32 value that differs in its last bit between the two chains can round to the other bfloat16 neighbour:
    # in the one-term mode the chains agree to a few bfloat16 roundings of single terms, not to FP32 accuracy)
    r = oracle.mixing_block_backward_reduced(ways, X, gamma, beta, W1, b1, W2, dY, t)
    loose = 2e-3 if t == 1 else 1e-4
    for got, name in ((dx, "dX"), (g["dw1"], "dW1"), (g["dw2"], "dW2"), (dgam, "dgamma")):
        ref = r[name]
        assert np.all(np.abs(got - ref) <= loose * (np.abs(ref) + np.abs(ref).max())), name
    if t == 1:      # and it is the mixed-precision chain, not the FP32 one
        full = oracle.mixing_block_backward(ways, X, gamma, beta, W1, b1, W2, dY)
        assert (np.abs(g["dw2"] - full["dW2"]) / (np.abs(full["dW2"]) + np.abs(full["dW2"]).max())).max() > 1e-5
