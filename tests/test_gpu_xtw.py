"""GPU parity of the transposed linear layer Y = X^T W + b (JG_OP_XTW) against the CPU oracle.

Same bars as for the X W^T layer: |Y_gpu - Y64| <= 1e-6 * S with S = |b| + |X|^T |W|, bit-exact
layout steps, bit-exact products on lattice inputs.  X is [tokens, channels] = K x M, W is K x N.
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


def operands(seed, K, M, N, mode="R", bias=True):
    X = inputs.matrix(seed, K, M, mode)
    W = inputs.matrix(seed + inputs.W_STREAM, K, N, mode, inputs.W_SCALE_EXP)
    b = inputs.matrix(seed + inputs.B_STREAM, 1, N, mode)[0] if bias else None
    return X, W, b


def run_layer(jg, ctx, X, W, b, ways, combine=0, weights=0):
    from paper_2507_05753_amd.layer import JigsawLinear
    K, M = X.shape
    N = W.shape[1]
    with JigsawLinear(M, K, N, ways, bias=b is not None, combine=combine, weights=weights, ctx=ctx,
                      op=jg.JG_OP_XTW) as L:
        nf = L.ws.numel() // 4      # stale workspace / output contents must not matter
        if nf:
            L.ws[: nf * 4].view(torch.float32).fill_(float("nan"))
        for y in L.y:
            y.fill_(float("nan"))
        Xd, Wd = dev(X), dev(W)
        L.shard(Xd, Wd, dev(b) if b is not None else None)
        L.forward()
        Y = L.gather()
        torch.cuda.synchronize()
        assert torch.equal(Xd.cpu(), torch.from_numpy(X)) and torch.equal(Wd.cpu(), torch.from_numpy(W))
        shards = dict(x=[t.cpu().numpy() for t in L.x], w=[t.cpu().numpy() for t in L.w],
                      y=[t.cpu().numpy() for t in L.y],
                      b=[t.cpu().numpy() for t in L.b] if b is not None else None)
        return Y.cpu().numpy(), shards


# (K tokens, M channels, N)
SHAPES = [
    (100, 100, 100),     # block extents of 50: not multiples of 4 (guarded kernel)
    (2, 2, 2),           # smallest 4-way instance
    (72, 130, 258),      # ragged edges in M and N, K of two slabs and a bit
    (200, 264, 136),     # several tiles in M, stream kernel (all extents multiples of 8)
    (520, 64, 640),      # several tiles in N, ragged K tail
    (1032, 520, 264),    # multi-tile in both, long K
]


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("K,M,N", SHAPES)
def test_shard_and_gather_are_bit_exact(jg, ctx, ways, K, M, N):
    X, W, b = operands(7, K, M, N)
    Y, sh = run_layer(jg, ctx, X, W, b, ways)
    for got, want in zip(sh["x"], oracle.shard_blocks(X, ways)):
        assert np.array_equal(got, want)
    for got, want in zip(sh["w"], oracle.shard_blocks(W, ways)):
        assert np.array_equal(got, want)
    for got, want in zip(sh["b"], oracle.shard_b(b, ways)):
        assert np.array_equal(got, want)
    assert np.array_equal(Y, oracle.gather_y(sh["y"], ways))


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("bias", [False, True])
@pytest.mark.parametrize("K,M,N", SHAPES)
def test_forward_matches_oracle_within_tolerance(jg, ctx, ways, bias, K, M, N):
    X, W, b = operands(11, K, M, N, bias=bias)
    Y, _ = run_layer(jg, ctx, X, W, b, ways)
    Y64 = oracle.linear_xtw(X, W, b)
    S = oracle.magnitude_xtw(X, W, b)
    err = np.abs(Y.astype(np.float64) - Y64)
    assert np.all(err <= TOL * S), f"max err/S = {(err / S).max():.3e}"
    # and against the block-wise oracle, which sums in the method's order
    err = np.abs(Y.astype(np.float64) - oracle.jigsaw_xtw(ways, X, W, b))
    assert np.all(err <= TOL * S)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("K,M,N", SHAPES)
def test_lattice_inputs_are_bit_exact(jg, ctx, ways, K, M, N):
    X, W, b = operands(13, K, M, N, "L")
    Y, _ = run_layer(jg, ctx, X, W, b, ways)
    want = oracle.linear_xtw(X, W, b)
    assert np.array_equal(want.astype(np.float32).astype(np.float64), want)   # representable: a fair demand
    assert np.array_equal(Y.astype(np.float64), want)


@pytest.mark.parametrize("ways", [2, 4])
@pytest.mark.parametrize("combine,weights", [(1, 0), (0, 1), (1, 1)])
def test_option_variants_agree_bit_for_bit_on_lattice_inputs(jg, ctx, ways, combine, weights):
    K, M, N = 200, 264, 136
    X, W, b = operands(17, K, M, N, "L")
    base, _ = run_layer(jg, ctx, X, W, b, ways)
    other, _ = run_layer(jg, ctx, X, W, b, ways, combine=combine, weights=weights)
    assert np.array_equal(base, other)
    X, W, b = operands(18, K, M, N, "R")
    got, _ = run_layer(jg, ctx, X, W, b, ways, combine=combine, weights=weights)
    S = oracle.magnitude_xtw(X, W, b)
    assert np.all(np.abs(got.astype(np.float64) - oracle.linear_xtw(X, W, b)) <= TOL * S)


def test_same_sign_operands_stay_within_tolerance(jg, ctx):
    # all-positive data: the running sum is the magnitude itself (two-level accumulation at work)
    K, M, N = 4096, 136, 264
    X = np.abs(inputs.matrix(19, K, M, "R"))
    W = np.abs(inputs.matrix(20, K, N, "R"))
    for ways in (1, 4):
        Y, _ = run_layer(jg, ctx, X, W, None, ways)
        S = oracle.magnitude_xtw(X, W)
        err = np.abs(Y.astype(np.float64) - oracle.linear_xtw(X, W))
        assert np.all(err <= TOL * S), f"ways={ways}: {(err / S).max():.3e}"


def run_backward(jg, ctx, X, W, dY, ways):
    from paper_2507_05753_amd.layer import JigsawLinear
    K, M = X.shape
    N = W.shape[1]
    with JigsawLinear(M, K, N, ways, ctx=ctx, op=jg.JG_OP_XTW) as L:
        L.shard(dev(X), dev(W))
        L.shard_dy(dev(dY))
        L.backward()
        dX, dW = L.gather_dx().cpu().numpy(), L.gather_dw().cpu().numpy()
        L.backward()        # the inputs are untouched: the same again
        assert np.array_equal(dX, L.gather_dx().cpu().numpy()) and np.array_equal(dW, L.gather_dw().cpu().numpy())
    return dX, dW


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("K,M,N", [(2, 2, 2), (100, 100, 100), (130, 72, 258), (258, 264, 136), (520, 300, 1032),
                                   (64, 1030, 36)])
def test_backward_matches_oracle_within_tolerance(jg, ctx, ways, K, M, N):
    """dX = W dY^T and dW = X dY of the transposed layer: |got - want64| <= 1e-6 * (|W| |dY|^T resp. |X| |dY|)."""
    X, W, _ = operands(640, K, M, N, "R", bias=False)
    dY = inputs.matrix(641, M, N, "R")
    dX, dW = run_backward(jg, ctx, X, W, dY, ways)
    wX, wW = oracle.backward_xtw(X, W, dY)
    SX, SW = oracle.backward_xtw(X, W, dY, absolute=True)
    ex, ew = np.abs(dX - wX), np.abs(dW - wW)
    assert np.all(ex <= TOL * SX), f"dX: {(ex / np.maximum(SX, 1e-300)).max():.3e}"
    assert np.all(ew <= TOL * SW), f"dW: {(ew / np.maximum(SW, 1e-300)).max():.3e}"


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_backward_is_bit_exact_on_lattice_inputs(jg, ctx, ways):
    K, M, N = 132, 200, 72
    X, W, _ = operands(642, K, M, N, "L", bias=False)
    dY = inputs.matrix(643, M, N, "L")
    dX, dW = run_backward(jg, ctx, X, W, dY, ways)
    wX, wW = oracle.backward_xtw(X, W, dY)
    assert np.array_equal(dX.astype(np.float64), wX) and np.array_equal(dW.astype(np.float64), wW)


def test_backward_checks_its_workspace(jg, ctx):
    from paper_2507_05753_amd.layer import JigsawLinear
    with JigsawLinear(8, 8, 8, 2, ctx=ctx, op=jg.JG_OP_XTW) as L:
        ptrs = [t.data_ptr() for t in L.x]
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_linear_backward(L.plan, ptrs, ptrs, ptrs, ptrs, ptrs, None, 0)
        assert e.value.status == jg.JG_E_WORKSPACE


# --------------------------------------------------------------------------------------------
# full size: first token-mixing linear of the paper's 1-billion-parameter model (Sec. 6.2.1:
# embedding dimension 4320, token-mixing hidden dimension 8640; 16200 tokens = the 721 x 1440
# grid in 8 x 8 patches)
# --------------------------------------------------------------------------------------------
def note(capsys, msg):
    with capsys.disabled():
        print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def pm1(seed, n, cols):
    bits = inputs.keys(seed, np.arange(n * cols, dtype=np.uint64)) >> np.uint64(63)
    return np.where(bits.reshape(n, cols) == 1, 1.0, -1.0)


@pytest.mark.timeout(600)
def test_token_mixing_size(jg, capsys):
    from paper_2507_05753_amd.layer import JigsawLinear
    cfg = inputs.XTW_CONFIGS["token_mixing_1b"]
    K, M, N, seed = cfg["K"], cfg["M"], cfg["N"], cfg["seed"]
    Xd = inputs.matrix_torch(seed, K, M, "R", device="cuda")
    Wd = inputs.matrix_torch(seed + inputs.W_STREAM, K, N, "R", inputs.W_SCALE_EXP, device="cuda")
    X, W = Xd.cpu().numpy(), Wd.cpu().numpy()
    rows = [0, 1, K // 2, K - 1]
    assert np.array_equal(X[rows], inputs.matrix_rows(seed, M, rows, "R"))      # host generator agrees
    # Freivalds: Y v = X^T (W v), in double, with the bound |X|^T (|W| |v|)
    V = pm1(5000, N, 3)
    Xd64, Wd64 = X.astype(np.float64), W.astype(np.float64)
    want = Xd64.T @ (Wd64 @ V)
    bound = np.abs(Xd64).T @ (np.abs(Wd64) @ np.abs(V))
    del Xd64, Wd64
    # sampled entries, one by one, from the oracle: rows of X^T against rows of W^T
    k = inputs.keys(5001, np.arange(600, dtype=np.uint64))
    I = np.unique(np.concatenate([(k[:300] % np.uint64(M)).astype(np.int64), [0, M // 2 - 1, M // 2, M - 1]]))
    J = np.unique(np.concatenate([(k[300:] % np.uint64(N)).astype(np.int64), [0, N // 2 - 1, N // 2, N - 1]]))
    gi, gj = np.meshgrid(np.arange(I.size), np.arange(J.size), indexing="ij")
    ent, mag = oracle.entries(np.ascontiguousarray(X[:, I].T), np.ascontiguousarray(W[:, J].T), gi.ravel(), gj.ravel())
    note(capsys, "token mixing: references ready")
    for ways in (1, 2, 4):
        with JigsawLinear(M, K, N, ways, op=jg.JG_OP_XTW) as L:
            L.ws.fill_(0xFF)
            L.shard(Xd, Wd)
            L.forward()
            Y = L.gather()
            torch.cuda.synchronize()
            Y = Y.cpu().numpy()
        assert np.isfinite(Y).all()
        err = np.abs(Y.astype(np.float64) @ V - want)
        assert np.all(err <= TOL * bound), f"ways={ways}: Freivalds worst {(err / bound).max():.3e}"
        e = np.abs(Y[np.ix_(I, J)].ravel() - ent) / mag
        assert e.max() <= TOL, (ways, e.max())
        note(capsys, f"token mixing ways={ways}: Freivalds {(err / bound).max():.2e}, {e.size} entries max err/S {e.max():.2e}")
