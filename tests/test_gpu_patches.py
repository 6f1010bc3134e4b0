"""GPU parity of the patch encoder / decoder data movement and of the encoder end to end.

jg_shard_patches must produce, bit for bit, the shards of the patch matrix the oracle builds with
plain loops; jg_gather_patches must invert it; the encoder (patch shards + Jigsaw linear) must match
the strided convolution written out by its definition (tiny shapes) and the forward oracle on the
patch matrix (larger ones).
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


def field_of(seed, C, H, W, mode="R"):
    return inputs.matrix(seed, C * H, W, mode).reshape(C, H, W)


# (C, H, W, p): 16-byte path (p = 4, 8), element path (p = 2, 3, 1, and W not a multiple of 4)
GEOMETRIES = [(2, 8, 16, 4), (6, 16, 24, 8), (4, 12, 18, 3), (2, 6, 8, 2), (8, 4, 6, 1), (3, 8, 16, 8), (2, 16, 12, 4),
              (2, 32, 48, 16), (4, 24, 40, 8), (2, 24, 24, 12)]   # tiled kernel: p = 4, 8, 16 with whole channels per block


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("C,H,W,p", GEOMETRIES)
def test_patch_shards_and_their_inverse_are_bit_exact(jg, ctx, ways, C, H, W, p):
    from paper_2507_05753_amd.layer import JigsawLinear
    M, K, N = (H // p) * (W // p), C * p * p, 6
    if (ways >= 2 and K % 2) or (ways == 4 and M % 2):
        pytest.skip("not divisible for this number of ranks")
    f = field_of(71, C, H, W)
    P = oracle.patchify(f, p)
    with JigsawLinear(M, K, N, ways, ctx=ctx) as L:
        for t in L.x:
            t.fill_(float("nan"))
        fd = torch.from_numpy(f).cuda()
        L.shard_patches(fd, p)
        torch.cuda.synchronize()
        for got, want in zip(L.x, oracle.shard_x(P, ways)):
            assert np.array_equal(got.cpu().numpy(), want)
        assert torch.equal(fd.cpu(), torch.from_numpy(f))
    # decoder direction: a plan whose output rows are patches
    with JigsawLinear(M, 6, K, ways, ctx=ctx) as L:
        for t, blk in zip(L.y, oracle.shard_y(P, ways)):
            t.copy_(torch.from_numpy(blk))
        out = torch.full((C, H, W), float("nan"), device="cuda")
        L.gather_patches(C, H, W, p, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), f)
        assert np.array_equal(oracle.unpatchify(P, C, H, W, p), f)


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_encoder_equals_the_strided_convolution(jg, ctx, ways):
    from paper_2507_05753_amd.layer import JigsawLinear
    C, H, W, p, N = 2, 8, 8, 4, 6
    f = field_of(72, C, H, W, "L")
    kern = inputs.matrix(73, N * C * p, p, "L").reshape(N, C, p, p)
    b = inputs.matrix(74, 1, N, "L")[0]
    want = oracle.patch_conv(f, kern, b)                     # six nested loops; lattice values: exact
    M, K = (H // p) * (W // p), C * p * p
    with JigsawLinear(M, K, N, ways, bias=True, ctx=ctx) as L:
        L.shard(None, torch.from_numpy(kern.reshape(N, K)).cuda(), torch.from_numpy(b).cuda())
        L.shard_patches(torch.from_numpy(f).cuda(), p)
        L.forward()
        Y = L.gather().cpu().numpy()
    assert np.array_equal(Y.astype(np.float64), want)


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_encoder_and_decoder_at_a_medium_size(jg, ctx, ways):
    from paper_2507_05753_amd.layer import JigsawLinear
    C, H, W, p, N = 6, 64, 96, 8, 136          # 96 patches of 384 features
    f = field_of(75, C, H, W)
    M, K = (H // p) * (W // p), C * p * p
    Wt = inputs.matrix(76, N, K, "R", inputs.W_SCALE_EXP)
    b = inputs.matrix(77, 1, N, "R")[0]
    P = oracle.patchify(f, p)
    with JigsawLinear(M, K, N, ways, bias=True, ctx=ctx) as L:
        L.shard(None, torch.from_numpy(Wt).cuda(), torch.from_numpy(b).cuda())
        L.shard_patches(torch.from_numpy(f).cuda(), p)
        L.forward()
        Y = L.gather().cpu().numpy()
    S = oracle.magnitude(P, Wt, b)
    assert np.all(np.abs(Y.astype(np.float64) - oracle.linear(P, Wt, b)) <= TOL * S)
    # decoder: tokens x (C p^2) -> field
    Wd = inputs.matrix(78, K, N, "R", inputs.W_SCALE_EXP)
    T = inputs.matrix(79, M, N, "R")
    with JigsawLinear(M, N, K, ways, ctx=ctx) as L:
        L.shard(torch.from_numpy(T).cuda(), torch.from_numpy(Wd).cuda())
        L.forward()
        out = L.gather_patches(C, H, W, p).cpu().numpy()
    want = oracle.unpatchify(oracle.linear(T, Wd), C, H, W, p)
    Sf = oracle.unpatchify(oracle.magnitude(T, Wd), C, H, W, p)
    assert np.all(np.abs(out.astype(np.float64) - want) <= TOL * Sf)


def note(capsys, msg):
    with capsys.disabled():
        print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


@pytest.mark.timeout(600)
def test_encoder_size(jg, capsys):
    """The encoder of the 1B model: 72 variables on a 720 x 1440 grid, 8 x 8 patches, embedding 4320."""
    from paper_2507_05753_amd.layer import JigsawLinear
    cfg = inputs.ENCODER_CONFIGS["encoder_1b"]
    C, H, W, p, N, seed = cfg["C"], cfg["H"], cfg["W"], cfg["p"], cfg["N"], cfg["seed"]
    M, K = (H // p) * (W // p), C * p * p
    fd = inputs.matrix_torch(seed, C * H, W, "R", device="cuda").reshape(C, H, W)
    Wt = inputs.matrix(seed + inputs.W_STREAM, N, K, "R", inputs.W_SCALE_EXP)
    Wd = torch.from_numpy(Wt).cuda()
    # sampled patches, rebuilt on the host from the rows of the field they cover
    k = inputs.keys(7000, np.arange(60, dtype=np.uint64))
    toks = np.unique(np.concatenate([(k % np.uint64(M)).astype(np.int64), [0, M // 2 - 1, M // 2, M - 1]]))
    wp = W // p
    rows = np.empty((toks.size, K), dtype=np.float32)
    for i, t in enumerate(toks):
        py, px = divmod(int(t), wp)
        for c in range(C):
            ids = [c * H + py * p + dy for dy in range(p)]
            blk = inputs.matrix_rows(seed, W, ids, "R")[:, px * p:(px + 1) * p]
            rows[i, c * p * p:(c + 1) * p * p] = blk.reshape(-1)
    want = oracle.linear(rows, Wt)
    S = oracle.magnitude(rows, Wt)
    note(capsys, f"encoder: oracle rows ready ({toks.size} patches)")
    idx = torch.from_numpy(toks).cuda()
    for ways in (1, 2, 4):
        with JigsawLinear(M, K, N, ways) as L:
            L.ws.fill_(0xFF)
            L.shard(None, Wd)
            L.shard_patches(fd, p)
            L.forward()
            Y = L.gather()
            torch.cuda.synchronize()
            assert torch.isfinite(Y).all()
            Ys = Y[idx].cpu().numpy().astype(np.float64)
            del Y
        torch.cuda.empty_cache()
        e = np.abs(Ys - want) / S
        assert e.max() <= TOL, (ways, e.max())
        note(capsys, f"encoder ways={ways}: {e.size} entries max err/S {e.max():.2e}")
