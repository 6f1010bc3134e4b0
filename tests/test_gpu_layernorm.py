"""GPU parity of the layer norm over a rank's channels and of the pre-norm channel-mixing block.

Bar for the norm: the kernel evaluates sums and the normalisation in double and rounds once, so
|out - out64| <= half an FP32 unit in the last place of out64 plus 1e-12 of the magnitude
S = (|x| + |mu|) / sqrt(var + eps) * |gamma| + |beta| (for the different order of the double sums) — far inside
the 1e-6 * S asked of floating-point results, which is asserted too.  Rows whose result is known in closed
form must come out exactly.  The block: as for the MLP, with one FP32 rounding of Xn more in front of it.
"""
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2507_05753_amd import inputs

pytestmark = pytest.mark.gpu
HALF_ULP = 2.0 ** -24
TOL = 1e-6
TOL_H = 1e-6 + 2.0 ** -23


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


def affine(seed, C, mode="R"):
    gamma = (inputs.matrix(seed, 1, C, mode)[0] + np.float32(1.5)).astype(np.float32)
    beta = inputs.matrix(seed + 1, 1, C, mode)[0].astype(np.float32)
    return gamma, beta


def run_norm(jg, ctx, X, gamma, beta, ways, eps=oracle.LN_EPS, op=0, in_place=False):
    """shard X -> jg_layernorm_forward -> gather like X.  X is (rows = tokens, cols = channels)."""
    from paper_2507_05753_amd.layer import JigsawLinear
    T, C = X.shape
    M, K = (C, T) if op == jg.JG_OP_XTW else (T, C)
    with JigsawLinear(M, K, 8, ways, ctx=ctx, op=op) as L:
        Xd = dev(X)
        L.shard(Xd)
        before = [t.clone() for t in L.x]
        out = None if in_place else [torch.full_like(t, float("nan")) for t in L.x]
        res = L.layernorm(dev(gamma) if gamma is not None else None, dev(beta) if beta is not None else None,
                          eps, out)
        full = torch.empty((T, C), dtype=torch.float32, device="cuda")
        jg.jg_gather_as(L.plan, jg.JG_T_X, [t.data_ptr() for t in res], full.data_ptr(), C)
        torch.cuda.synchronize()
        if not in_place:
            assert all(torch.equal(a, b) for a, b in zip(before, L.x))       # the input is left alone
        return full.cpu().numpy()


def check(got, X, gamma, beta, ways, eps=oracle.LN_EPS):
    want, S = oracle.layernorm(X, gamma, beta, oracle.ln_groups(ways), eps, magnitude=True)
    err = np.abs(got.astype(np.float64) - want)
    bound = HALF_ULP * np.abs(want) * (1 + 1e-6) + 1e-12 * S + 1e-45
    assert np.all(err <= bound), f"max err/bound = {(err / bound).max():.3f}"
    assert np.all(err <= TOL * S)


# (tokens, channels): register-resident rows of several widths, a ragged last vector chunk, row counts
# that do not fill a workgroup, widths that are no multiple of 4 (4-way: of 8) and one past the register
# budget (plain kernel)
SHAPES = [(4, 8), (2, 2), (37, 256), (130, 520), (33, 1032), (18, 4320), (6, 8640), (50, 100), (21, 250),
          (6, 16392), (4, 33000)]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("T,C", SHAPES)
def test_layernorm_matches_oracle(jg, ctx, ways, T, C):
    if ways == 4 and T % 2:
        T += 1
    X = (inputs.matrix(71, T, C, "R") + np.float32(0.4)).astype(np.float32)
    gamma, beta = affine(72, C)
    check(run_norm(jg, ctx, X, gamma, beta, ways), X, gamma, beta, ways)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("use_gamma,use_beta", [(False, False), (True, False), (False, True)])
def test_optional_scale_and_offset(jg, ctx, ways, use_gamma, use_beta):
    T, C = 10, 520
    X = inputs.matrix(73, T, C, "R")
    gamma, beta = affine(74, C)
    gamma, beta = (gamma if use_gamma else None), (beta if use_beta else None)
    check(run_norm(jg, ctx, X, gamma, beta, ways), X, gamma, beta, ways)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("T,C", [(12, 264), (6, 250), (4, 16392)])
def test_in_place_and_eps(jg, ctx, ways, T, C):
    X = inputs.matrix(75, T, C, "R")
    gamma, beta = affine(76, C)
    out = run_norm(jg, ctx, X, gamma, beta, ways, in_place=True)
    assert np.array_equal(out, run_norm(jg, ctx, X, gamma, beta, ways))
    for eps in (0.0, 1e-3, 0.5):
        check(run_norm(jg, ctx, X, gamma, beta, ways, eps=eps), X, gamma, beta, ways, eps)


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_transposed_layer_plans_norm_the_same_axis(jg, ctx, ways):
    # X of the transposed layer is [tokens, channels] as well: rows are tokens
    T, C = 20, 264
    X = inputs.matrix(77, T, C, "R")
    gamma, beta = affine(78, C)
    got = run_norm(jg, ctx, X, gamma, beta, ways, op=jg.JG_OP_XTW)
    check(got, X, gamma, beta, ways)
    assert np.array_equal(got, run_norm(jg, ctx, X, gamma, beta, ways))


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("C", [264, 252, 250])
def test_closed_forms_are_exact(jg, ctx, ways, C):
    T = 8
    if (C // oracle.ln_groups(ways)) % 2:
        pytest.skip("a channel block of odd width has no +-1 row of mean zero")
    gamma, beta = affine(79, C, "L")
    # constant rows: x - mean is exactly zero, the result is beta
    X = np.tile(np.arange(1, T + 1, dtype=np.float32)[:, None] * np.float32(0.25), (1, C))
    assert np.array_equal(run_norm(jg, ctx, X, gamma, beta, ways), np.tile(beta, (T, 1)))
    # +-1 in every channel block, eps = 0: mean 0, variance 1, result x * gamma + beta (exact on the lattice)
    X = np.tile(np.array([1.0, -1.0], dtype=np.float32), (T, C // 2))
    want = X.astype(np.float64) * gamma + beta
    assert np.array_equal(run_norm(jg, ctx, X, gamma, beta, ways, eps=0.0).astype(np.float64), want)


def test_large_offset_rows_keep_their_accuracy(jg, ctx):
    # mean 1000 times the spread: a single-precision mean or a one-pass variance would lose the result
    T, C = 16, 4320
    X = (inputs.matrix(80, T, C, "R") + np.float32(1000.0)).astype(np.float32)
    gamma, beta = affine(81, C)
    for ways in (1, 2):
        check(run_norm(jg, ctx, X, gamma, beta, ways), X, gamma, beta, ways)


def test_argument_checks(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear
    with JigsawLinear(8, 8, 8, 2, ctx=ctx) as L:
        ptrs = [t.data_ptr() for t in L.x]
        for eps in (-1.0, float("nan")):
            with pytest.raises(jg.JigsawError) as e:
                jg.jg_layernorm_forward(L.plan, ptrs, None, None, eps, ptrs)
            assert e.value.status == jg.JG_E_DTYPE
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_layernorm_forward(L.plan, [ptrs[0], 0], None, None, 1e-5, ptrs)
        assert e.value.status == jg.JG_E_NULL
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_layernorm_forward(L.plan, ptrs, L.x[0].data_ptr() + 2, None, 1e-5, ptrs)
        assert e.value.status == jg.JG_E_ALIGN


# ---------------------------------------------------------------------------------------------
# the channel-mixing half of a mixing block
# ---------------------------------------------------------------------------------------------
def block_operands(seed, M, C, Hd):
    X = (inputs.matrix(seed, M, C, "R") + np.float32(0.25)).astype(np.float32)
    W1 = inputs.matrix(seed + 1, Hd, C, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, Hd, "R")[0]
    W2 = inputs.matrix(seed + 3, C, Hd, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 4, 1, C, "R")[0]
    gamma, beta = affine(seed + 5, C)
    return X, gamma, beta, W1, b1, W2, b2


def check_block(r, Xn, H, Y):
    want = r["Xn"]
    assert np.all(np.abs(Xn.astype(np.float64) - want) <= HALF_ULP * np.abs(want) * (1 + 1e-6) + 1e-10)
    eh = np.abs(H.astype(np.float64) - r["H"])
    assert np.all(eh <= TOL_H * r["S1"]), f"H: max err/S1 = {(eh / r['S1']).max():.3e}"
    ey = np.abs(Y.astype(np.float64) - r["Y"])
    bound = TOL * r["SY"] + TOL_H * r["PY"]
    assert np.all(ey <= bound), f"Y: max err/bound = {(ey / bound).max():.3e}"


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,C,Hd", [(100, 100, 100), (130, 72, 258), (258, 264, 136), (300, 520, 1032)])
def test_mixing_forward(jg, ctx, ways, M, C, Hd):
    from paper_2507_05753_amd.layer import JigsawMixing
    X, gamma, beta, W1, b1, W2, b2 = block_operands(90, M, C, Hd)
    with JigsawMixing(M, C, Hd, ways, ctx=ctx) as L:
        Xd = dev(X)
        L.shard(Xd, dev(gamma), dev(beta), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        Xn, H, Y = L.gather_xn().cpu().numpy(), L.gather_h().cpu().numpy(), L.gather().cpu().numpy()
        L.forward()                                   # the input shards were not overwritten: the same again
        assert np.array_equal(Y, L.gather().cpu().numpy())
    check_block(oracle.mixing_block(ways, X, gamma, beta, W1, b1, W2, b2), Xn, H, Y)
    # the norm matters: the plain MLP of the same operands is far away
    assert np.abs(Y - oracle.mlp(X, W1, b1, W2, b2)["Y"]).max() > 1e-2


def note(capsys, msg):
    with capsys.disabled():
        print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


@pytest.mark.timeout(600)
def test_channel_mixing_size(jg, capsys):
    """The channel-mixing block of the paper's 1-billion-parameter model (Sec. 6.2.1) at full size: the norm
    on every element of sampled rows and on all rows through its moments, the block on sampled rows."""
    from paper_2507_05753_amd.layer import JigsawMixing
    cfg = inputs.MLP_CONFIGS["channel_mixing_1b"]
    M, C, Hd, seed = cfg["M"], cfg["C"], cfg["Hd"], cfg["seed"]
    Xd = inputs.matrix_torch(seed, M, C, "R", device="cuda") + 0.25
    W1d = inputs.matrix_torch(seed + 1, Hd, C, "R", inputs.W_SCALE_EXP, device="cuda")
    W2d = inputs.matrix_torch(seed + 3, C, Hd, "R", inputs.W_SCALE_EXP, device="cuda")
    b1 = inputs.matrix(seed + 2, 1, Hd, "R")[0]
    b2 = inputs.matrix(seed + 4, 1, C, "R")[0]
    gamma, beta = affine(seed + 5, C)
    W1, W2 = W1d.cpu().numpy(), W2d.cpu().numpy()
    k = inputs.keys(7000, np.arange(24, dtype=np.uint64))
    rows = np.unique(np.concatenate([(k % np.uint64(M)).astype(np.int64), [0, M // 2 - 1, M // 2, M - 1]]))
    Xs = Xd[torch.from_numpy(rows).cuda()].cpu().numpy()
    note(capsys, f"channel mixing: {rows.size} sampled rows")
    for ways in (1, 2, 4):
        with JigsawMixing(M, C, Hd, ways) as L:
            L.shard(Xd, dev(gamma), dev(beta), W1d, dev(b1), W2d, dev(b2))
            L.forward()
            Xn, H, Y = L.gather_xn(), L.gather_h(), L.gather()
            torch.cuda.synchronize()
            assert torch.isfinite(Y).all()
            # all rows: with gamma = 1, beta = 0 each channel block of each token has mean 0 and
            # second moment var / (var + eps)
            jg.jg_layernorm_forward(L.first.plan, [t.data_ptr() for t in L.first.x], None, None, L.eps,
                                    [t.data_ptr() for t in L.xn])
            Z = L.gather_xn().double()
            g = oracle.ln_groups(ways)
            Zg = Z.view(M, g, C // g)
            var = Xd.double().view(M, g, C // g).var(dim=2, unbiased=False)
            assert Zg.mean(dim=2).abs().max().item() <= 1e-7
            assert ((Zg * Zg).mean(dim=2) - var / (var + L.eps)).abs().max().item() <= 1e-6
            idx = torch.from_numpy(rows).cuda()
            Xn, H, Y = Xn[idx].cpu().numpy(), H[idx].cpu().numpy(), Y[idx].cpu().numpy()
        r = oracle.mixing_block(ways, Xs, gamma, beta, W1, b1, W2, b2)
        check_block(r, Xn, H, Y)
        note(capsys, f"channel mixing ways={ways}: ok")


# ---------------------------------------------------------------------------------------------
# the token-mixing half of a mixing block
# ---------------------------------------------------------------------------------------------
def token_operands(seed, T, C, D):
    X = (inputs.matrix(seed, T, C, "R") + np.float32(0.25)).astype(np.float32)
    W1 = inputs.matrix(seed + 1, T, D, "R", inputs.W_SCALE_EXP)
    b1 = inputs.matrix(seed + 2, 1, D, "R")[0]
    W2 = inputs.matrix(seed + 3, T, D, "R", inputs.W_SCALE_EXP)
    b2 = inputs.matrix(seed + 4, 1, T, "R")[0]
    gamma, beta = affine(seed + 5, C)
    return X, gamma, beta, W1, b1, W2, b2


def check_token_block(X, gamma, beta, W1, b1, W2, b2, ways, Xn, H, Y):
    want = oracle.layernorm(X, gamma, beta, oracle.ln_groups(ways))
    assert np.all(np.abs(Xn.astype(np.float64) - want) <= HALF_ULP * np.abs(want) * (1 + 1e-6) + 1e-10)
    # first layer from the Xn the GPU stored, second from the H it stored: each at the bar of one layer
    S1 = oracle.magnitude_xtw(Xn, W1, b1)
    eh = np.abs(H.astype(np.float64) - oracle.gelu(oracle.linear_xtw(Xn, W1, b1)))
    assert np.all(eh <= TOL_H * S1), f"H: max err/S1 = {(eh / S1).max():.3e}"
    b2d = np.zeros(X.shape[0]) if b2 is None else b2.astype(np.float64)
    ref = X.astype(np.float64) + oracle.linear(W2, H) + b2d[:, None]
    SY = np.abs(X.astype(np.float64)) + oracle.magnitude(W2, H) + np.abs(b2d)[:, None]
    ey = np.abs(Y.astype(np.float64) - ref)
    assert np.all(ey <= TOL * SY), f"Y: max err/S = {(ey / SY).max():.3e}"


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("T,C,D", [(100, 100, 100), (130, 72, 258), (258, 264, 136), (520, 300, 1032)])
def test_token_mixing_forward(jg, ctx, ways, T, C, D):
    from paper_2507_05753_amd.layer import JigsawTokenMixing
    X, gamma, beta, W1, b1, W2, b2 = token_operands(95, T, C, D)
    with JigsawTokenMixing(T, C, D, ways, ctx=ctx) as L:
        L.ws.fill_(0xFF)
        L.shard(dev(X), dev(gamma), dev(beta), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        Xn, H, Y = L.gather_xn().cpu().numpy(), L.gather_h().cpu().numpy(), L.gather().cpu().numpy()
        L.forward()                                   # the inputs were not overwritten: the same again
        assert np.array_equal(Y, L.gather().cpu().numpy())
    check_token_block(X, gamma, beta, W1, b1, W2, b2, ways, Xn, H, Y)
    # end to end against the oracle's own chain (loose: H's last FP32 bits differ)
    r = oracle.token_mixing_block(ways, X, gamma, beta, W1, b1, W2, b2)
    assert np.all(np.abs(Y - r["Y"]) <= 1e-5 * r["SY"])
    # the tokens are mixed: a channel-mixing block of the same operand shapes would not even type-check, and a
    # block without the norm is far away
    assert np.abs(Y - (X + b2[:, None])).max() > 1e-2


@pytest.mark.parametrize("ways", [1, 4])
def test_token_mixing_without_the_second_bias_and_without_scale(jg, ctx, ways):
    from paper_2507_05753_amd.layer import JigsawTokenMixing
    T, C, D = 130, 72, 64
    X, gamma, beta, W1, b1, W2, b2 = token_operands(96, T, C, D)
    with JigsawTokenMixing(T, C, D, ways, ctx=ctx) as L:
        L.shard(dev(X), None, None, dev(W1), dev(b1), dev(W2), None)
        L.forward()
        Xn, H, Y = L.gather_xn().cpu().numpy(), L.gather_h().cpu().numpy(), L.gather().cpu().numpy()
    check_token_block(X, None, None, W1, b1, W2, None, ways, Xn, H, Y)


def test_token_mixing_argument_checks(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear, JigsawTokenMixing
    with JigsawTokenMixing(64, 32, 48, 2, ctx=ctx) as L, \
            JigsawLinear(64, 48, 32, 2, bias=True, ctx=ctx) as biased, \
            JigsawLinear(64, 48, 30, 2, ctx=ctx) as narrow, JigsawLinear(64, 48, 32, 4, ctx=ctx) as four:
        f, s = L.first, L.second
        p = lambda ts: [t.data_ptr() for t in ts]
        b2 = torch.zeros(64, device="cuda")
        call = lambda first, second, ws_bytes, bias=b2: jg.jg_token_mixing_forward(
            first.plan, second.plan, p(f.x), None, None, 1e-5, p(f.w), p(f.b), p(s.x), bias.data_ptr() if bias is not None else None,
            p(L.xn), p(f.y), p(s.y), L.ws.data_ptr(), ws_bytes)
        for first, second, want in ((s, s, jg.JG_E_DTYPE),            # the first layer must be the transposed one
                                    (f, f, jg.JG_E_DTYPE),
                                    (f, biased, jg.JG_E_DTYPE),       # the second layer's bias is b2, per token
                                    (f, narrow, jg.JG_E_SHAPE), (f, four, jg.JG_E_WAYS)):
            with pytest.raises(jg.JigsawError) as e:
                call(first, second, L.ws_bytes)
            assert e.value.status == want
        with pytest.raises(jg.JigsawError) as e:                      # with b2 the skip connection needs its copy of X
            call(f, s, L.ws_bytes - 256)
        assert e.value.status == jg.JG_E_WORKSPACE
        L.shard(torch.zeros(64, 32, device="cuda"), None, None, torch.zeros(64, 48, device="cuda"),
                torch.zeros(48, device="cuda"), torch.zeros(64, 48, device="cuda"), None)
        call(f, s, L.ws_bytes - 256, None)                            # without b2 it does not
        torch.cuda.synchronize()


@pytest.mark.timeout(600)
def test_token_mixing_size(jg, capsys):
    """The token-mixing block of the paper's 1-billion-parameter model at full size (16200 tokens, 4320 channels,
    8640 hidden), in the launch configuration bench.py --op token_mixing times: sampled channels of H and sampled
    tokens of Y element by element, everything finite."""
    from paper_2507_05753_amd.layer import JigsawTokenMixing
    cfg = inputs.XTW_CONFIGS["token_mixing_1b"]
    T, C, D, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    Xd = inputs.matrix_torch(seed, T, C, "R", device="cuda") + 0.25
    W1d = inputs.matrix_torch(seed + 1, T, D, "R", inputs.W_SCALE_EXP, device="cuda")
    W2d = inputs.matrix_torch(seed + 3, T, D, "R", inputs.W_SCALE_EXP, device="cuda")
    b1 = inputs.matrix(seed + 2, 1, D, "R")[0]
    b2 = inputs.matrix(seed + 4, 1, T, "R")[0]
    gamma, beta = affine(seed + 5, C)
    W1, W2 = W1d.cpu().numpy(), W2d.cpu().numpy()
    k = inputs.keys(7200, np.arange(40, dtype=np.uint64))
    chans = np.unique(np.concatenate([(k[:16] % np.uint64(C)).astype(np.int64), [0, C // 2 - 1, C // 2, C - 1]]))
    toks = np.unique(np.concatenate([(k[16:] % np.uint64(T)).astype(np.int64), [0, T // 2 - 1, T // 2, T - 1]]))
    ci, ti = torch.from_numpy(chans).cuda(), torch.from_numpy(toks).cuda()
    note(capsys, f"token mixing block: {chans.size} sampled channels of H, {toks.size} sampled tokens of Y")
    for ways in (1, 2, 4):
        with JigsawTokenMixing(T, C, D, ways) as L:
            L.shard(Xd, dev(gamma), dev(beta), W1d, dev(b1), W2d, dev(b2))
            L.forward()
            Xn, H, Y = L.gather_xn(), L.gather_h(), L.gather()
            torch.cuda.synchronize()
            assert torch.isfinite(Y).all() and torch.isfinite(H).all()
            Xn_t = Xn[ti].cpu().numpy()
            Xn_c = Xn[:, ci].cpu().numpy()                       # the sampled channels' columns of Xn: T x n
            H_c = H[ci].cpu().numpy()                            # their rows of H: n x D
            Hh = H.cpu().numpy()
            Y_t, X_t = Y[ti].cpu().numpy(), Xd[ti].cpu().numpy()
        want = oracle.layernorm(X_t, gamma, beta, oracle.ln_groups(ways))      # the norm on the sampled tokens
        assert np.all(np.abs(Xn_t.astype(np.float64) - want) <= HALF_ULP * np.abs(want) * (1 + 1e-6) + 1e-10)
        # first layer: rows of H for the sampled channels, from the Xn the GPU stored
        S1 = oracle.magnitude_xtw(Xn_c, W1, b1)
        eh = np.abs(H_c.astype(np.float64) - oracle.gelu(oracle.linear_xtw(Xn_c, W1, b1)))
        assert np.all(eh <= TOL_H * S1), f"ways={ways} H: max err/S1 = {(eh / S1).max():.3e}"
        # second layer: sampled tokens of Y from the H the GPU stored
        W2_t = np.ascontiguousarray(W2[toks])
        ref = X_t.astype(np.float64) + oracle.linear(W2_t, Hh) + b2[toks].astype(np.float64)[:, None]
        SY = np.abs(X_t.astype(np.float64)) + oracle.magnitude(W2_t, Hh) + np.abs(b2[toks]).astype(np.float64)[:, None]
        ey = np.abs(Y_t.astype(np.float64) - ref)
        assert np.all(ey <= TOL * SY), f"ways={ways} Y: max err/S = {(ey / SY).max():.3e}"
        note(capsys, f"token mixing block ways={ways}: H max err/S1 {(eh / S1).max():.2e}, Y max err/S {(ey / SY).max():.2e}")


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_whole_mixing_block(jg, ctx, ways):
    """Token-mixing half, then channel-mixing half on its output shards in place (Sec. 3): each half against the
    oracle applied to what the GPU fed it."""
    from paper_2507_05753_amd.layer import JigsawMixerBlock
    T, C, Dt, Dc = 258, 264, 136, 200
    X, g1, be1, W1, b1, W2, b2 = token_operands(97, T, C, Dt)
    _, g2, be2, V1, c1, V2, c2 = block_operands(98, T, C, Dc)
    with JigsawMixerBlock(T, C, Dt, Dc, ways, ctx=ctx) as L:
        L.shard(dev(X), token=dict(gamma=dev(g1), beta=dev(be1), W1=dev(W1), b1=dev(b1), W2=dev(W2), b2=dev(b2)),
                channel=dict(gamma=dev(g2), beta=dev(be2), W1=dev(V1), b1=dev(c1), W2=dev(V2), b2=dev(c2)))
        L.forward()
        Xn, H, U = L.token.gather_xn().cpu().numpy(), L.token.gather_h().cpu().numpy(), L.gather_token_output().cpu().numpy()
        Un, G, Y = L.channel.gather_xn().cpu().numpy(), L.channel.gather_h().cpu().numpy(), L.gather().cpu().numpy()
    check_token_block(X, g1, be1, W1, b1, W2, b2, ways, Xn, H, U)
    check_block(oracle.mixing_block(ways, U, g2, be2, V1, c1, V2, c2), Un, G, Y)
    # end to end, loosely: both halves by the oracle
    r1 = oracle.token_mixing_block(ways, X, g1, be1, W1, b1, W2, b2)
    r2 = oracle.mixing_block(ways, r1["Y"].astype(np.float32), g2, be2, V1, c1, V2, c2)
    assert np.all(np.abs(Y - r2["Y"]) <= 1e-4 * (r2["SY"] + r2["PY"]))


# ---------------------------------------------------------------------------------------------
# the layer norm's gradients
# ---------------------------------------------------------------------------------------------
def run_norm_backward(jg, ctx, X, gamma, dY, ways, op=None, want_params=True, minimal_workspace=False):
    from paper_2507_05753_amd.layer import JigsawLinear
    T, C = X.shape
    kw = dict(op=jg.JG_OP_XTW) if op == "xtw" else {}
    M, K = (C, T) if op == "xtw" else (T, C)
    with JigsawLinear(M, K, 16, ways, ctx=ctx, **kw) as L:
        L.shard(dev(X))
        dy = [torch.empty_like(t) for t in L.x]
        dx = [torch.full_like(t, float("nan")) for t in L.x]
        jg.jg_shard(L.plan, jg.JG_T_X, dev(dY).data_ptr(), C, [t.data_ptr() for t in dy])
        dg = torch.full((C,), float("nan"), device="cuda") if want_params else None
        db = torch.full((C,), float("nan"), device="cuda") if want_params else None
        need = L.query(jg.JG_Q_NORM_BACKWARD_WORKSPACE_BYTES)
        if minimal_workspace:       # the rows' statistics only: the column sums then run one workgroup per strip
            need = ways * ((16 * L.query(jg.JG_Q_X_ROWS) + 255) // 256 * 256)
        ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")
        p = lambda ts: [t.data_ptr() for t in ts]
        g = dev(gamma) if gamma is not None else None
        call = lambda: jg.jg_layernorm_backward(L.plan, p(L.x), g.data_ptr() if g is not None else None, 1e-5, p(dy), p(dx),
                                                dg.data_ptr() if dg is not None else None,
                                                db.data_ptr() if db is not None else None, ws.data_ptr(), need)
        call()
        out = torch.empty((T, C), device="cuda")
        jg.jg_gather_as(L.plan, jg.JG_T_X, p(dx), out.data_ptr(), C)
        first = (out.cpu().numpy(), dg.cpu().numpy() if want_params else None, db.cpu().numpy() if want_params else None)
        call()
        jg.jg_gather_as(L.plan, jg.JG_T_X, p(dx), out.data_ptr(), C)
        assert np.array_equal(first[0], out.cpu().numpy())
        if want_params:
            assert np.array_equal(first[1], dg.cpu().numpy()) and np.array_equal(first[2], db.cpu().numpy())
        return first


def check_norm_backward(X, gamma, dY, ways, got):
    dX, dg, db, SX, Sg, Sb = oracle.layernorm_backward(X, gamma, dY, oracle.ln_groups(ways), magnitude=True)
    # evaluated in double and rounded once; the sums' order differs from the oracle's in the last double bits
    assert np.all(np.abs(got[0] - dX) <= HALF_ULP * np.abs(dX) * (1 + 1e-6) + 1e-11 * SX + 1e-45)
    if got[1] is not None:
        assert np.all(np.abs(got[1] - dg) <= HALF_ULP * np.abs(dg) * (1 + 1e-6) + 1e-11 * Sg + 1e-45)
        assert np.all(np.abs(got[2] - db) <= HALF_ULP * np.abs(db) * (1 + 1e-6) + 1e-11 * Sb + 1e-45)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("T,C", [(2, 4), (100, 100), (130, 72), (258, 264), (64, 4320), (2200, 50)])
def test_layernorm_backward_matches_oracle(jg, ctx, ways, T, C):
    X = (inputs.matrix(130, T, C, "R") + np.float32(0.25)).astype(np.float32)
    gamma, _ = affine(131, C)
    dY = inputs.matrix(132, T, C, "R")
    check_norm_backward(X, gamma, dY, ways, run_norm_backward(jg, ctx, X, gamma, dY, ways))


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("T,C", [(4098, 200), (2 * 2049, 72), (640, 4320)])
def test_layernorm_backward_column_sums_in_row_ranges(jg, ctx, ways, T, C):
    """Enough rows for several bands / row ranges (the last one ragged), with the whole workspace (one pass: the rows'
    kernel keeps the column sums of its band) and with the statistics' share only (two kernels, one workgroup per
    strip of columns): both inside the bar of a sum taken in double and rounded once."""
    X = (inputs.matrix(136, T, C, "R") + np.float32(0.125)).astype(np.float32)
    gamma, _ = affine(137, C)
    dY = np.abs(inputs.matrix(138, T, C, "R")) + np.float32(0.25)        # same-sign: FP32 sums would not do
    full = run_norm_backward(jg, ctx, X, gamma, dY, ways)
    small = run_norm_backward(jg, ctx, X, gamma, dY, ways, minimal_workspace=True)
    check_norm_backward(X, gamma, dY, ways, full)
    check_norm_backward(X, gamma, dY, ways, small)
    # the two forms take the rows' sums in different orders: dX agrees to a unit in the last place at worst
    assert np.all(np.abs(full[0] - small[0]) <= 2.0 ** -23 * np.abs(small[0]))


@pytest.mark.parametrize("ways", [1, 4])
@pytest.mark.parametrize("T,C", [(70, 6144), (70, 6148), (38, 12288), (2, 64), (6, 772)])
def test_layernorm_backward_row_widths(jg, ctx, ways, T, C):
    """The widest rows the one-pass form takes (6144 columns per block), the first width past it, a width of one
    vector per thread, and fewer rows than workgroups."""
    X = (inputs.matrix(140, T, C, "R") + np.float32(0.25)).astype(np.float32)
    gamma, _ = affine(141, C)
    dY = inputs.matrix(142, T, C, "R")
    check_norm_backward(X, gamma, dY, ways, run_norm_backward(jg, ctx, X, gamma, dY, ways))


@pytest.mark.parametrize("minimal", [False, True])
def test_layernorm_backward_rows_far_from_zero(jg, ctx, minimal):
    """Rows whose mean is hundreds of standard deviations from zero: the one-pass form takes its sums about the row's
    first element, so nothing is lost to the mean."""
    T, C = 300, 1080
    X = (inputs.matrix(143, T, C, "R") * np.float32(0.5) + np.float32(300.0)).astype(np.float32)
    gamma, _ = affine(144, C)
    dY = inputs.matrix(145, T, C, "R")
    for ways in (1, 4):
        check_norm_backward(X, gamma, dY, ways, run_norm_backward(jg, ctx, X, gamma, dY, ways, minimal_workspace=minimal))


@pytest.mark.parametrize("ways", [1, 4])
def test_layernorm_backward_options(jg, ctx, ways):
    T, C = 130, 72
    X = (inputs.matrix(133, T, C, "R") - np.float32(0.5)).astype(np.float32)
    gamma, _ = affine(134, C)
    dY = inputs.matrix(135, T, C, "R")
    check_norm_backward(X, None, dY, ways, run_norm_backward(jg, ctx, X, None, dY, ways))                 # gamma = 1
    check_norm_backward(X, gamma, dY, ways, run_norm_backward(jg, ctx, X, gamma, dY, ways, want_params=False))
    check_norm_backward(X, gamma, dY, ways, run_norm_backward(jg, ctx, X, gamma, dY, ways, op="xtw"))      # same axis


def test_layernorm_backward_argument_checks(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear
    with JigsawLinear(16, 8, 8, 2, ctx=ctx) as L:
        p = [t.data_ptr() for t in L.x]
        need = L.query(jg.JG_Q_NORM_BACKWARD_WORKSPACE_BYTES)
        # the rows' statistics (required), then the column sums of two blocks x sixteen bands of one row x four columns
        assert need == 2 * 256 + 2 * 16 * 4 * 16
        ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
        for args, want in (((p, None, -1.0, p, p, None, None, ws.data_ptr(), need), jg.JG_E_DTYPE),
                           ((p, None, 1e-5, p, p, None, None, ws.data_ptr(), 2 * 256 - 1), jg.JG_E_WORKSPACE),
                           ((p, None, 1e-5, p, p, None, None, None, 0), jg.JG_E_WORKSPACE),
                           ((p, None, 1e-5, p, p, None, None, ws.data_ptr() + 16, need), jg.JG_E_ALIGN),
                           ((p, L.x[0].data_ptr() + 2, 1e-5, p, p, None, None, ws.data_ptr(), need), jg.JG_E_ALIGN)):
            with pytest.raises(jg.JigsawError) as e:
                jg.jg_layernorm_backward(L.plan, *args)
            assert e.value.status == want


# ---- backward of the token-mixing half -----------------------------------------------------------------------
@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("T,C,D", [(100, 100, 100), (130, 72, 258), (264, 136, 72), (520, 300, 1032)])
def test_token_mixing_backward(jg, ctx, ways, T, C, D):
    """Every step of jg_token_mixing_backward against the oracle applied to what the GPU stored for the step before
    (the products within 1e-6 * S, the elementwise steps and the sums within one rounding), then the whole chain
    loosely against the oracle's own chain."""
    from paper_2507_05753_amd.layer import JigsawTokenMixing
    X, gamma, beta, W1, b1, W2, b2 = token_operands(370, T, C, D)
    dY = inputs.matrix(371, T, C, "R")
    f64 = lambda a: a.astype(np.float64)
    within = lambda got, want, S: np.all(np.abs(f64(got) - want) <= 1e-6 * S)
    once = lambda got, want, S: np.all(np.abs(f64(got) - want) <= HALF_ULP * np.abs(want) * (1 + 1e-6) + 1e-11 * S + 1e-45)
    with JigsawTokenMixing(T, C, D, ways, ctx=ctx) as L:
        L.shard(dev(X), dev(gamma), dev(beta), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        L.backward(dev(dY))
        Xn, H = L.gather_xn().cpu().numpy(), L.gather_h().cpu().numpy()
        g = {k: L.gather_grad(k).cpu().numpy() for k in ("a", "dh", "da", "dxn", "dx", "dw1", "dw2", "db1")}
        db2, dgam, dbet = L.db2.cpu().numpy(), L.dgamma.cpu().numpy(), L.dbeta.cpu().numpy()
        L.backward(dev(dY))                                    # nothing it reads was overwritten: the same again
        for k in ("dx", "dw1", "dw2"):
            assert np.array_equal(g[k], L.gather_grad(k).cpu().numpy()), k
        assert np.array_equal(db2, L.db2.cpu().numpy()) and np.array_equal(dgam, L.dgamma.cpu().numpy())
    # A recomputed: the transposed layer once more
    assert within(g["a"], oracle.linear_xtw(Xn, W1, b1), oracle.magnitude_xtw(Xn, W1, b1)), "A"
    # second layer's backward, W2 in the activations' place and H in the weights'
    (dW2, dH), (SW2, SH) = oracle.backward(W2, H, dY), oracle.backward_magnitude(W2, H, dY)
    assert within(g["dw2"], dW2, SW2), "dW2"
    assert within(g["dh"], dH, SH), "dH"
    want = oracle.bias_backward(np.ascontiguousarray(dY.T))
    assert once(db2, want, oracle.bias_backward(np.ascontiguousarray(dY.T), absolute=True)), "db2"
    # dA from the A and dH the GPU stored: evaluated in double, rounded once
    dA = f64(g["dh"]) * oracle.gelu_grad(f64(g["a"]))
    assert np.all(np.abs(f64(g["da"]) - dA) <= 2.0 ** -23 * np.abs(dA) + 1e-45), "dA"
    # the transposed layer's backward from the dA the GPU stored
    (dXn, dW1), (SXn, SW1) = oracle.backward_xtw(Xn, W1, g["da"]), oracle.backward_xtw(Xn, W1, g["da"], absolute=True)
    assert within(g["dxn"], dXn, SXn), "dXn"
    assert within(g["dw1"], dW1, SW1), "dW1"
    assert once(g["db1"], oracle.bias_backward(g["da"]), oracle.bias_backward(g["da"], absolute=True)), "db1"
    # the norm's backward from the dXn the GPU stored, the skip connection added before the rounding
    dXl, dg, db, SX, Sg, Sb = oracle.layernorm_backward(X, gamma, g["dxn"], oracle.ln_groups(ways), magnitude=True)
    assert once(g["dx"], f64(dY) + dXl, SX + np.abs(dY)), "dX"
    assert once(dgam, dg, Sg) and once(dbet, db, Sb)
    # end to end (Xn, H and A in FP32 here differ in the last bits from the oracle's)
    r = oracle.token_mixing_block_backward(ways, X, gamma, beta, W1, b1, W2, dY)
    for got, name in ((g["dx"], "dX"), (g["dw1"], "dW1"), (g["dw2"], "dW2"), (g["db1"], "db1"), (db2, "db2"),
                      (dgam, "dgamma"), (dbet, "dbeta")):
        ref = r[name]
        assert got.shape == ref.shape and np.all(np.abs(got - ref) <= 1e-4 * (np.abs(ref) + np.abs(ref).max())), name


@pytest.mark.timeout(900)
def test_token_mixing_backward_size(jg, capsys):
    """The token-mixing block's backward at the 1B model's size, in the launch configuration bench.py --op
    token_mixing_backward times.  Per sampled channel every step of the MLP's chain (whole rows of A, dH, dA, whole
    columns of dXn), per sampled token the norm's step (whole rows of dX), each against the oracle applied to what
    the GPU stored for the step before; sampled entries of dW1 and dW2 (sums over all channels); db1, db2, dgamma and
    dbeta in full."""
    from paper_2507_05753_amd.layer import JigsawTokenMixing
    cfg = inputs.XTW_CONFIGS["token_mixing_1b"]
    T, C, D, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    gen = lambda s, r, c, e=0: inputs.matrix_torch(s, r, c, "R", e, device="cuda")
    Xd, dYd = gen(seed, T, C) + 0.25, gen(seed + 7, T, C)
    W1d, W2d = gen(seed + 1, T, D, inputs.W_SCALE_EXP), gen(seed + 3, T, D, inputs.W_SCALE_EXP)
    b1d, b2d = gen(seed + 2, 1, D)[0].contiguous(), gen(seed + 4, 1, T)[0].contiguous()
    gamma, beta = affine(seed + 5, C)
    W1, b1, W2 = W1d.cpu().numpy(), b1d.cpu().numpy(), W2d.cpu().numpy()
    X, dY = Xd.cpu().numpy(), dYd.cpu().numpy()
    k = inputs.keys(7300, np.arange(48, dtype=np.uint64))
    cs = np.unique(np.concatenate([(k[:12] % np.uint64(C)).astype(np.int64), [0, C // 2 - 1, C // 2, C - 1]]))
    ts = np.unique(np.concatenate([(k[12:32] % np.uint64(T)).astype(np.int64), [0, T // 2 - 1, T // 2, T - 1]]))
    ds = np.unique(np.concatenate([(k[32:] % np.uint64(D)).astype(np.int64), [0, D // 2 - 1, D // 2, D - 1]]))
    ci, ti, di = (torch.from_numpy(v).cuda() for v in (cs, ts, ds))
    f64 = lambda a: a.astype(np.float64)
    tr = lambda a: np.ascontiguousarray(a.T)
    for ways in (1, 4):
        with JigsawTokenMixing(T, C, D, ways) as L:
            L.shard(Xd, dev(gamma), dev(beta), W1d, b1d, W2d, b2d)
            L.forward()
            L.backward(dYd)
            torch.cuda.synchronize()
            Xn, H = L.gather_xn(), L.gather_h()
            full = {}
            for name in ("a", "dh", "da", "dxn", "dx", "dw1", "dw2"):
                t = L.gather_grad(name)
                assert torch.isfinite(t).all(), name
                full[name] = t
            a_c, dh_c, da_c = (full[n][ci].cpu().numpy() for n in ("a", "dh", "da"))      # rows of the C x D matrices
            dxn_c = full["dxn"][:, ci].cpu().numpy()                                    # columns of dXn: T x n
            dxn_t, dx_t = full["dxn"][ti].cpu().numpy(), full["dx"][ti].cpu().numpy()
            Xn_c, Xn_t = Xn[:, ci].cpu().numpy(), Xn[ti].cpu().numpy()
            da_d, H_d = full["da"][:, di].cpu().numpy(), H[:, di].cpu().numpy()          # columns over all channels
            dW1_s, dW2_s = full["dw1"][ti][:, di].cpu().numpy(), full["dw2"][ti][:, di].cpu().numpy()
            dA_full, dXn_full = full["da"].cpu().numpy(), full["dxn"].cpu().numpy()
            db1 = L.gather_grad("db1").cpu().numpy()
            db2, dgam, dbet = L.db2.cpu().numpy(), L.dgamma.cpu().numpy(), L.dbeta.cpu().numpy()
            del full, Xn, H
        torch.cuda.empty_cache()
        worst = {}

        def within(name, got, want, S):
            e = (np.abs(f64(got) - want) / np.maximum(S, 1e-300)).max()
            worst[name] = e
            assert e <= 1e-6, (ways, name, e)

        def once(name, got, want, S):
            assert np.all(np.abs(f64(got) - want) <= HALF_ULP * np.abs(want) * (1 + 1e-6) + 1e-11 * S), (ways, name)
        # per sampled channel
        within("A", a_c, oracle.linear_xtw(Xn_c, W1, b1), oracle.magnitude_xtw(Xn_c, W1, b1))
        dY_c = np.ascontiguousarray(dY[:, cs])
        within("dH", dh_c, oracle.linear_xtw(dY_c, W2), oracle.magnitude_xtw(dY_c, W2))
        dA = f64(dh_c) * oracle.gelu_grad(f64(a_c))
        assert np.all(np.abs(f64(da_c) - dA) <= 2.0 ** -23 * np.abs(dA) + 1e-45), (ways, "dA")
        within("dXn", dxn_c, oracle.linear(W1, da_c), oracle.magnitude(W1, da_c))
        # per sampled token: the norm's step with the skip connection
        dXl, _, _, SX, _, _ = oracle.layernorm_backward(X[ts], gamma, dxn_t, oracle.ln_groups(ways), magnitude=True)
        once("dX", dx_t, f64(dY[ts]) + dXl, SX + np.abs(dY[ts]))
        # sampled entries of the weight gradients: sums over all channels of what the GPU stored
        within("dW1", dW1_s, oracle.linear(Xn_t, tr(da_d)), oracle.magnitude(Xn_t, tr(da_d)))
        within("dW2", dW2_s, oracle.linear(dY[ts], tr(H_d)), oracle.magnitude(dY[ts], tr(H_d)))
        # in full
        once("db1", db1, oracle.bias_backward(dA_full), oracle.bias_backward(dA_full, absolute=True))
        once("db2", db2, oracle.bias_backward(tr(dY)), oracle.bias_backward(tr(dY), absolute=True))
        _, dg, db, _, Sg, Sb = oracle.layernorm_backward(X, gamma, dXn_full, oracle.ln_groups(ways), magnitude=True)
        once("dgamma", dgam, dg, Sg)
        once("dbeta", dbet, db, Sb)
        note(capsys, f"token mixing backward ways={ways}: {cs.size} channels, {ts.size} tokens, {ts.size} x {ds.size} weight "
                     f"entries; max err/S " + ", ".join(f"{n} {e:.2e}" for n, e in worst.items()))


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_whole_mixing_block_backward(jg, ctx, ways):
    """Backward of a whole mixing block: the channel half's backward, then the token half's on its dX shards in place.
    The halves are checked step by step in their own tests; here the hand-over on shards must give the bits of the
    hand-over through a gathered matrix, and the whole chain must follow the oracle's chain."""
    from paper_2507_05753_amd.layer import JigsawMixerBlock
    T, C, Dt, Dc = 258, 264, 136, 200
    X, g1, be1, W1, b1, W2, b2 = token_operands(380, T, C, Dt)
    _, g2, be2, V1, c1, V2, c2 = block_operands(381, T, C, Dc)
    dY = inputs.matrix(382, T, C, "R")
    with JigsawMixerBlock(T, C, Dt, Dc, ways, ctx=ctx) as L:
        L.shard(dev(X), token=dict(gamma=dev(g1), beta=dev(be1), W1=dev(W1), b1=dev(b1), W2=dev(W2), b2=dev(b2)),
                channel=dict(gamma=dev(g2), beta=dev(be2), W1=dev(V1), b1=dev(c1), W2=dev(V2), b2=dev(c2)))
        L.forward()
        L.backward(dev(dY))
        mid = L.channel.gather_grad("dx")
        got = {k: L.token.gather_grad(k).cpu().numpy() for k in ("dx", "dw1", "dw2", "db1")}
        got.update(db2=L.token.db2.cpu().numpy(), dgamma=L.token.dgamma.cpu().numpy())
        chan = {k: L.channel.gather_grad(k).cpu().numpy() for k in ("dw1", "dw2")}
        assert np.array_equal(got["dx"], L.gather_dx().cpu().numpy())
        L.token.backward(mid)                                   # the same gradient, sharded from the gathered matrix
        for k in ("dx", "dw1", "dw2", "db1"):
            assert np.array_equal(got[k], L.token.gather_grad(k).cpu().numpy()), k
        assert np.array_equal(got["db2"], L.token.db2.cpu().numpy())
        mid = mid.cpu().numpy()
    r1 = oracle.token_mixing_block(ways, X, g1, be1, W1, b1, W2, b2)
    U = r1["Y"].astype(np.float32)
    rc = oracle.mixing_block_backward(ways, U, g2, be2, V1, c1, V2, dY)
    rt = oracle.token_mixing_block_backward(ways, X, g1, be1, W1, b1, W2, rc["dX"].astype(np.float32))
    loose = lambda a, ref: np.all(np.abs(a - ref) <= 1e-4 * (np.abs(ref) + np.abs(ref).max()))
    assert loose(mid, rc["dX"]) and loose(chan["dw1"], rc["dW1"]) and loose(chan["dw2"], rc["dW2"])
    for k, name in (("dx", "dX"), ("dw1", "dW1"), ("dw2", "dW2"), ("db1", "db1"), ("db2", "db2"), ("dgamma", "dgamma")):
        assert loose(got[k], rt[name]), k


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("dtype_name", ["JG_BF16", "JG_BF16X3"])
@pytest.mark.parametrize("T,C,D", [(100, 112, 112), (130, 80, 272), (264, 144, 80), (521, 304, 1040)])
def test_token_mixing_backward_in_mixed_precision(jg, ctx, ways, dtype_name, T, C, D):
    """jg_token_mixing_backward on reduced plans: every product against the oracle's reduced routine applied to what
    the GPU stored for the step before (1e-6 * S), the FP32 steps within one rounding, the chain loosely."""
    from paper_2507_05753_amd.layer import JigsawTokenMixing
    dtype = getattr(jg, dtype_name)
    t = 3 if dtype == jg.JG_BF16X3 else 1
    if ways == 4 and T % 2:
        T += 1
    X, gamma, beta, W1, b1, W2, b2 = token_operands(510, T, C, D)
    dY = inputs.matrix(511, T, C, "R")
    f64 = lambda a: a.astype(np.float64)
    within = lambda got, want, S: np.all(np.abs(f64(got) - want) <= 1e-6 * S)
    once = lambda got, want, S: np.all(np.abs(f64(got) - want) <= HALF_ULP * np.abs(want) * (1 + 1e-6) + 1e-11 * S + 1e-45)
    with JigsawTokenMixing(T, C, D, ways, ctx=ctx, dtype=dtype) as L:
        L.keep_masters = True
        L.shard(dev(X), dev(gamma), dev(beta), dev(W1), dev(b1), dev(W2), dev(b2))
        L.forward()
        L.backward(dev(dY))
        Xn, H = L.gather_xn().cpu().numpy(), L.gather_h().cpu().numpy()
        g = {k: L.gather_grad(k).cpu().numpy() for k in ("a", "dh", "da", "dxn", "dx", "dw1", "dw2", "db1")}
        db2, dgam = L.db2.cpu().numpy(), L.dgamma.cpu().numpy()
        L.backward(dev(dY))
        for k in ("dx", "dw1", "dw2"):
            assert np.array_equal(g[k], L.gather_grad(k).cpu().numpy()), k
    assert within(g["a"], oracle.linear_xtw_reduced(Xn, W1, b1, t), oracle.linear_xtw_reduced(Xn, W1, b1, t, absolute=True)), "A"
    (dW2, dH), (SW2, SH) = oracle.backward_reduced(W2, H, dY, t), oracle.backward_reduced(W2, H, dY, t, absolute=True)
    assert within(g["dw2"], dW2, SW2), "dW2"
    assert within(g["dh"], dH, SH), "dH"
    assert once(db2, oracle.bias_backward(np.ascontiguousarray(dY.T)), oracle.bias_backward(np.ascontiguousarray(dY.T), absolute=True))
    dA = f64(g["dh"]) * oracle.gelu_grad(f64(g["a"]))
    assert np.all(np.abs(f64(g["da"]) - dA) <= 2.0 ** -23 * np.abs(dA) + 1e-45), "dA"
    (dXn, dW1) = oracle.backward_xtw_reduced(Xn, W1, g["da"], t)
    (SXn, SW1) = oracle.backward_xtw_reduced(Xn, W1, g["da"], t, absolute=True)
    assert within(g["dxn"], dXn, SXn), "dXn"
    assert within(g["dw1"], dW1, SW1), "dW1"
    assert once(g["db1"], oracle.bias_backward(g["da"]), oracle.bias_backward(g["da"], absolute=True)), "db1"
    dXl, dg, db, SX, Sg, Sb = oracle.layernorm_backward(X, gamma, g["dxn"], oracle.ln_groups(ways), magnitude=True)
    assert once(g["dx"], f64(dY) + dXl, SX + np.abs(dY)), "dX"
    assert once(dgam, dg, Sg)
    r = oracle.token_mixing_block_backward_reduced(ways, X, gamma, beta, W1, b1, W2, dY, t)
    loose = 2e-3 if t == 1 else 1e-4        # (a last-bit difference in an FP32 intermediate can flip a bfloat16 rounding)
    for got, name in ((g["dx"], "dX"), (g["dw1"], "dW1"), (g["dw2"], "dW2"), (db2, "db2"), (dgam, "dgamma")):
        ref = r[name]
        assert got.shape == ref.shape and np.all(np.abs(got - ref) <= loose * (np.abs(ref) + np.abs(ref).max())), name
