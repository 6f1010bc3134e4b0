"""Host-side checks of the C-ABI library: it loads, exports what the header declares,
validates descriptors and does its accounting.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_2507_05753_amd import binding as jg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "jigsaw.h")).read()
    declared = set(re.findall(r"^\s*(?:const\s+char\s*\*|int|void)\s+(jg_\w+)\s*\(", header, re.M))
    assert declared == set(jg.EXPORTS)
    lib = ctypes.CDLL(jg.LIB_PATH)
    for name in sorted(declared):
        assert getattr(lib, name) is not None, name


def test_strerror_is_total():
    for s in range(-12, 2):
        assert isinstance(jg.jg_strerror(s), str) and jg.jg_strerror(s)
    assert jg.jg_strerror(jg.JG_OK) == "ok"
    assert "gfx950" in jg.jg_strerror(jg.JG_E_ARCH)


def status_of(**kw):
    base = dict(M=8, K=8, N=8, ways=2)
    base.update(kw)
    try:
        p = jg.jg_plan_create(None, **base)
    except jg.JigsawError as e:
        return e.status
    jg.jg_plan_destroy(p)
    return jg.JG_OK


def test_plan_validation():
    assert status_of() == jg.JG_OK
    assert status_of(ways=3) == jg.JG_E_WAYS
    assert status_of(ways=0) == jg.JG_E_WAYS
    assert status_of(ways=8) == jg.JG_E_WAYS
    assert status_of(M=0) == jg.JG_E_SHAPE
    assert status_of(K=-2) == jg.JG_E_SHAPE
    assert status_of(N=2 ** 31) == jg.JG_E_SHAPE
    # tile counts beyond the 32-bit block index are refused, just below the limit is accepted
    assert status_of(M=128 * 23171, N=128 * 23171, K=128) == jg.JG_E_SHAPE      # 23171^2 * 4 > 2^31
    assert status_of(M=128 * 23169, N=128 * 23169, K=128) == jg.JG_OK
    assert status_of(M=128, N=128 * 23171, K=128 * 23171) == jg.JG_E_SHAPE      # backward dW tiles
    assert status_of(K=7) == jg.JG_E_SHAPE            # 2-way needs even K
    assert status_of(N=7) == jg.JG_E_SHAPE            # ... and even N
    assert status_of(M=7) == jg.JG_OK                 # ... but any M
    assert status_of(M=7, ways=4) == jg.JG_E_SHAPE    # 4-way needs even M too
    assert status_of(M=7, K=7, N=7, ways=1) == jg.JG_OK
    assert status_of(dtype=3) == jg.JG_E_DTYPE
    # reduced precision: forward only, and every rank's share of K in whole 8-element chunks
    for dt in (jg.JG_BF16, jg.JG_BF16X3):
        assert status_of(dtype=dt) == jg.JG_E_SHAPE                 # K / 2 = 4
        assert status_of(dtype=dt, K=16) == jg.JG_OK
        assert status_of(dtype=dt, K=8, ways=1) == jg.JG_OK
        assert status_of(dtype=dt, K=24, ways=4) == jg.JG_E_SHAPE   # K / 2 = 12
        # the transposed layer's shard step pads the contracted dimension itself: any K that `ways` divides
        assert status_of(dtype=dt, K=8, op=jg.JG_OP_XTW) == jg.JG_OK
        assert status_of(dtype=dt, K=12, op=jg.JG_OP_XTW, ways=4) == jg.JG_OK
        assert status_of(dtype=dt, K=7, op=jg.JG_OP_XTW, ways=1) == jg.JG_OK
        assert status_of(dtype=dt, K=7, op=jg.JG_OP_XTW, ways=4) == jg.JG_E_SHAPE
    assert status_of(op=3) == jg.JG_E_DTYPE
    # the X W permutation: FP32 only, split like X W^T (K and N halved, 4-way M as well)
    assert status_of(op=jg.JG_OP_XW) == jg.JG_OK
    assert status_of(op=jg.JG_OP_XW, dtype=jg.JG_BF16, K=16) == jg.JG_E_DTYPE
    assert status_of(op=jg.JG_OP_XW, K=7) == jg.JG_E_SHAPE
    assert status_of(op=jg.JG_OP_XW, N=7) == jg.JG_E_SHAPE
    assert status_of(op=jg.JG_OP_XW, M=7) == jg.JG_OK
    assert status_of(op=jg.JG_OP_XW, M=7, ways=4) == jg.JG_E_SHAPE
    # the transposed layer splits M and N (2-way), and K as well (4-way)
    assert status_of(op=jg.JG_OP_XTW) == jg.JG_OK
    assert status_of(op=jg.JG_OP_XTW, K=7) == jg.JG_OK
    assert status_of(op=jg.JG_OP_XTW, M=7) == jg.JG_E_SHAPE
    assert status_of(op=jg.JG_OP_XTW, N=7) == jg.JG_E_SHAPE
    assert status_of(op=jg.JG_OP_XTW, K=7, ways=4) == jg.JG_E_SHAPE
    assert status_of(op=jg.JG_OP_XTW, M=7, K=7, N=7, ways=1) == jg.JG_OK
    assert status_of(combine=2) == jg.JG_E_DTYPE
    assert status_of(weights=5) == jg.JG_E_DTYPE
    lib = jg.raw()
    out = ctypes.c_void_p()
    assert lib.jg_plan_create(None, None, ctypes.byref(out)) == jg.JG_E_NULL
    d = jg.jg_linear_desc(8, 8, 8, 2, 0, 0, 0, 0, 0)
    assert lib.jg_plan_create(None, ctypes.byref(d), None) == jg.JG_E_NULL
    jg.jg_plan_destroy(None)
    jg.jg_free(None)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", [(100, 100, 100), (25000, 4000, 4000), (200000, 10000, 10000), (6, 4, 2)])
def test_accounting(ways, M, K, N):
    p = jg.jg_plan_create(None, M, K, N, ways)
    q = lambda what, r=0: jg.jg_plan_query(p, what, r)
    try:
        assert q(jg.JG_Q_FLOPS_TOTAL) == 2 * M * K * N
        assert sum(q(jg.JG_Q_FLOPS_RANK, r) for r in range(ways)) == 2 * M * K * N
        # zero memory redundancy (Sec. 4): the shards tile X, W and Y exactly
        assert sum(q(jg.JG_Q_RESIDENT_BYTES_RANK, r) for r in range(ways)) == 4 * (M * K + N * K + M * N)
        assert sum(q(jg.JG_Q_X_ROWS, r) * q(jg.JG_Q_X_COLS, r) for r in range(ways)) == M * K
        assert sum(q(jg.JG_Q_W_ROWS, r) * q(jg.JG_Q_W_COLS, r) for r in range(ways)) == N * K
        assert sum(q(jg.JG_Q_Y_ROWS, r) * q(jg.JG_Q_Y_COLS, r) for r in range(ways)) == M * N
        for r in range(ways):
            assert q(jg.JG_Q_B_LEN, r) == q(jg.JG_Q_Y_COLS, r)
            # Y is partitioned like X (Sec. 4.1: the scheme is maintained after the product)
            assert q(jg.JG_Q_Y_ROWS, r) == q(jg.JG_Q_X_ROWS, r)
        # the scratch of the split tail comes on top of what the method itself needs
        tail = q(jg.JG_Q_TAIL_SCRATCH_BYTES)
        assert 0 <= tail <= 512 * 2 * 128 * 128 * 4 and tail % (128 * 128 * 4) == 0
        if ways == 1:
            assert q(jg.JG_Q_WORKSPACE_BYTES) == tail and q(jg.JG_Q_EXCHANGE_BYTES_RANK) == 0
            assert q(jg.JG_Q_HBM_BYTES_ALGO) == 4 * (M * K + N * K + M * N)
            assert q(jg.JG_Q_GEMM_LAUNCHES) == 1
        else:
            assert q(jg.JG_Q_HBM_BYTES_ALGO) == 4 * (M * K + N * K + M * N) + 8 * M * N
            assert q(jg.JG_Q_GEMM_LAUNCHES) == 2
            # one partial per output element, plus (4-way, copy mode) one weight block per rank
            ws = q(jg.JG_Q_WORKSPACE_BYTES) - tail
            need = 4 * M * N + (4 * N * K if ways == 4 else 0)
            assert need <= ws <= need + 2 * ways * 256
            if ways == 2:
                assert q(jg.JG_Q_EXCHANGE_BYTES_RANK, 1) == 4 * M * N // 2
            else:
                assert q(jg.JG_Q_EXCHANGE_BYTES_RANK, 3) == 4 * (M * N // 4 + N * K // 4)
        # backward: twice the forward work (Sec. 6.3); one partial per dX element, and per dW element in 4-way
        assert q(jg.JG_Q_BACKWARD_FLOPS_TOTAL) == 4 * M * K * N
        assert q(jg.JG_Q_BACKWARD_GEMM_LAUNCHES) == {1: 2, 2: 3, 4: 4}[ways]
        bw = q(jg.JG_Q_BACKWARD_WORKSPACE_BYTES) - q(jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES)
        need = 0 if ways == 1 else 4 * M * K + (4 * N * K if ways == 4 else 0)
        assert need <= bw <= need + 2 * ways * 256
        with pytest.raises(jg.JigsawError) as e:
            q(jg.JG_Q_X_ROWS, ways)
        assert e.value.status == jg.JG_E_WAYS
        with pytest.raises(jg.JigsawError) as e:
            q(99)
        assert e.value.status == jg.JG_E_DTYPE
    finally:
        jg.jg_plan_destroy(p)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", [(100, 100, 100), (4320, 16200, 8640), (6, 4, 2), (130, 72, 258)])
def test_accounting_of_the_transposed_layer(ways, M, K, N):
    p = jg.jg_plan_create(None, M, K, N, ways, op=jg.JG_OP_XTW)
    q = lambda what, r=0: jg.jg_plan_query(p, what, r)
    try:
        assert q(jg.JG_Q_FLOPS_TOTAL) == 2 * M * K * N
        assert sum(q(jg.JG_Q_FLOPS_RANK, r) for r in range(ways)) == 2 * M * K * N
        # nothing is duplicated: the shards tile X (K x M), W (K x N) and Y (M x N) exactly
        assert sum(q(jg.JG_Q_RESIDENT_BYTES_RANK, r) for r in range(ways)) == 4 * (M * K + N * K + M * N)
        assert sum(q(jg.JG_Q_X_ROWS, r) * q(jg.JG_Q_X_COLS, r) for r in range(ways)) == M * K
        assert sum(q(jg.JG_Q_W_ROWS, r) * q(jg.JG_Q_W_COLS, r) for r in range(ways)) == N * K
        assert sum(q(jg.JG_Q_Y_ROWS, r) * q(jg.JG_Q_Y_COLS, r) for r in range(ways)) == M * N
        rows, cols = (2 if ways == 4 else 1), (2 if ways >= 2 else 1)
        for r in range(ways):
            assert (q(jg.JG_Q_X_ROWS, r), q(jg.JG_Q_X_COLS, r)) == (K // rows, M // cols)
            assert (q(jg.JG_Q_W_ROWS, r), q(jg.JG_Q_W_COLS, r)) == (K // rows, N // cols)
            assert (q(jg.JG_Q_Y_ROWS, r), q(jg.JG_Q_Y_COLS, r)) == (M // rows, N // cols)
            assert q(jg.JG_Q_B_LEN, r) == N // cols
        ws = q(jg.JG_Q_WORKSPACE_BYTES) - q(jg.JG_Q_TAIL_SCRATCH_BYTES)
        if ways == 1:
            assert ws == 0 and q(jg.JG_Q_EXCHANGE_BYTES_RANK) == 0 and q(jg.JG_Q_GEMM_LAUNCHES) == 1
            assert q(jg.JG_Q_HBM_BYTES_ALGO) == 4 * (M * K + N * K + M * N)
        elif ways == 2:
            # only an activation block changes hands; no partial products
            assert q(jg.JG_Q_EXCHANGE_BYTES_RANK, 1) == 4 * K * M // 2 and q(jg.JG_Q_GEMM_LAUNCHES) == 1
            assert q(jg.JG_Q_HBM_BYTES_ALGO) == 4 * (M * K + N * K + M * N)
            assert 4 * K * M <= ws <= 4 * K * M + 2 * ways * 256
        else:
            assert q(jg.JG_Q_EXCHANGE_BYTES_RANK, 3) == 4 * (M * N // 4 + K * M // 4) and q(jg.JG_Q_GEMM_LAUNCHES) == 2
            assert q(jg.JG_Q_HBM_BYTES_ALGO) == 4 * (M * K + N * K + M * N) + 8 * M * N
            assert 4 * (M * N + K * M) <= ws <= 4 * (M * N + K * M) + 2 * ways * 256
        # backward: dX and dW cost a forward each; with more than one rank both sum two terms through a partial
        assert q(jg.JG_Q_BACKWARD_FLOPS_TOTAL) == 4 * M * K * N
        assert q(jg.JG_Q_BACKWARD_GEMM_LAUNCHES) == (2 if ways == 1 else 4)
        bw = q(jg.JG_Q_BACKWARD_WORKSPACE_BYTES) - q(jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES)
        if ways == 1:
            assert bw == 0
        else:
            assert 4 * (K * M + K * N) <= bw <= 4 * (K * M + K * N) + 2 * ways * 256
    finally:
        jg.jg_plan_destroy(p)


def test_backward_of_a_transposed_plan_needs_a_context():
    p = jg.jg_plan_create(None, 8, 8, 8, 2, op=jg.JG_OP_XTW)
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    assert lib.jg_linear_backward(p, pp, pp, pp, pp, pp, 256, 1 << 20) == jg.JG_E_NULL   # no context comes first
    jg.jg_plan_destroy(p)


def test_tail_split_accounting():
    q = lambda p, what: jg.jg_plan_query(p, what)
    tile = 128 * 128 * 4
    # token-mixing size of the transposed layer: 34 x 68 = 2312 tiles = 4 rounds of 512 slots + 264
    # tiles of 507 slabs: the tail goes to 512 runs (two scratch tiles each)
    p = jg.jg_plan_create(None, 4320, 16200, 8640, 1, op=jg.JG_OP_XTW)
    assert q(p, jg.JG_Q_TAIL_SCRATCH_BYTES) == 512 * 2 * tile
    assert q(p, jg.JG_Q_WORKSPACE_BYTES) == 512 * 2 * tile
    jg.jg_plan_destroy(p)
    p = jg.jg_plan_create(None, 4320, 16200, 8640, 1, op=jg.JG_OP_XTW, tail=jg.JG_TAIL_WHOLE)
    assert q(p, jg.JG_Q_TAIL_SCRATCH_BYTES) == 0 and q(p, jg.JG_Q_WORKSPACE_BYTES) == 0
    jg.jg_plan_destroy(p)
    # config 3: 12 whole rounds and a quarter: the estimated saving is below the threshold
    p = jg.jg_plan_create(None, 25000, 4000, 4000, 4)
    assert q(p, jg.JG_Q_TAIL_SCRATCH_BYTES) == 0 and q(p, jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES) == 0
    jg.jg_plan_destroy(p)
    # a whole number of rounds: nothing to split (64 x 64 tiles = 8 rounds)
    p = jg.jg_plan_create(None, 8192, 4096, 8192, 1)
    assert q(p, jg.JG_Q_TAIL_SCRATCH_BYTES) == 0
    jg.jg_plan_destroy(p)
    # a single short tile: runs would be shorter than the minimum, stays whole
    p = jg.jg_plan_create(None, 100, 100, 100, 1)
    assert q(p, jg.JG_Q_TAIL_SCRATCH_BYTES) == 0
    jg.jg_plan_destroy(p)
    # a problem smaller than the chip (less than half a round of tiles): runs of four slabs fill it.
    # 1000^3, one rank: 8 x 8 tiles of 32 slabs -> one run per compute unit; 4-way: 4 x 16 tiles of 16 slabs -> 256 runs
    p = jg.jg_plan_create(None, 1000, 1000, 1000, 1)
    assert q(p, jg.JG_Q_TAIL_SCRATCH_BYTES) == 256 * 2 * tile
    jg.jg_plan_destroy(p)
    p = jg.jg_plan_create(None, 1000, 1000, 1000, 4)
    assert q(p, jg.JG_Q_TAIL_SCRATCH_BYTES) == 256 * 2 * tile
    jg.jg_plan_destroy(p)
    # few long tiles: 3 x 3 tiles of 65 slabs -> 585 / 4 = 146 runs
    p = jg.jg_plan_create(None, 300, 2080, 260, 1)
    assert q(p, jg.JG_Q_TAIL_SCRATCH_BYTES) == 146 * 2 * tile
    # ... and in the backward pass: dX 3 x 17 tiles of 9 slabs (whole), dW 3 x 17 tiles of 10 slabs (whole)
    assert q(p, jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES) == 0
    jg.jg_plan_destroy(p)
    with pytest.raises(jg.JigsawError) as e:
        jg.jg_plan_create(None, 8, 8, 8, 2, tail=2)
    assert e.value.status == jg.JG_E_DTYPE


def test_workspace_grows_with_options():
    M, K, N = 64, 32, 48
    base = jg.jg_plan_create(None, M, K, N, 4)
    sep = jg.jg_plan_create(None, M, K, N, 4, combine=jg.JG_COMBINE_SEPARATE)
    direct = jg.jg_plan_create(None, M, K, N, 4, weights=jg.JG_WEIGHTS_DIRECT)
    ws = lambda p: jg.jg_plan_query(p, jg.JG_Q_WORKSPACE_BYTES) - jg.jg_plan_query(p, jg.JG_Q_TAIL_SCRATCH_BYTES)
    assert ws(sep) == ws(base) + 4 * M * N
    assert ws(direct) == ws(base) - 4 * N * K
    for p in (base, sep, direct):
        jg.jg_plan_destroy(p)


def test_data_calls_refuse_a_plan_without_context():
    p = jg.jg_plan_create(None, 8, 8, 8, 2)
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    assert lib.jg_linear_forward(p, pp, pp, None, pp, 256, 1 << 20) == jg.JG_E_NULL
    assert lib.jg_shard(p, jg.JG_T_X, 256, 8, pp) == jg.JG_E_NULL
    assert lib.jg_gather(p, pp, 256, 8) == jg.JG_E_NULL
    assert lib.jg_gather_as(p, jg.JG_T_W, pp, 256, 8) == jg.JG_E_NULL
    assert lib.jg_linear_backward(p, pp, pp, pp, pp, pp, 256, 1 << 20) == jg.JG_E_NULL
    assert lib.jg_linear_forward(None, pp, pp, None, pp, 256, 1 << 20) == jg.JG_E_NULL
    jg.jg_plan_destroy(p)


def test_init_without_a_gpu_fails_cleanly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(jg.JigsawError) as e:
        jg.jg_init(0, None)
    assert e.value.status == jg.JG_E_HIP


def test_mlp_entry_point_checks_that_the_plans_chain():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    call = lambda a, b: lib.jg_mlp_forward(a, b, pp, pp, pp, pp, pp, pp, pp, 256, 1 << 20)
    a = jg.jg_plan_create(None, 64, 32, 48, 2, True)
    assert call(None, a) == jg.JG_E_NULL
    for (M, K, N), ways, want in (((64, 48, 30), 2, jg.JG_E_SHAPE), ((62, 48, 32), 2, jg.JG_E_SHAPE),
                                  ((64, 40, 32), 2, jg.JG_E_SHAPE), ((64, 48, 32), 4, jg.JG_E_WAYS),
                                  ((64, 48, 32), 2, jg.JG_E_NULL)):      # chains, but no context
        b = jg.jg_plan_create(None, M, K, N, ways, True)
        assert call(a, b) == want
        jg.jg_plan_destroy(b)
    t = jg.jg_plan_create(None, 48, 64, 32, 2, True, op=jg.JG_OP_XTW)
    assert call(a, t) == jg.JG_E_DTYPE
    assert lib.jg_linear_forward_ex(a, pp, pp, pp, None, 7, pp, 256, 1 << 20) == jg.JG_E_NULL   # no context comes first
    jg.jg_plan_destroy(t)
    jg.jg_plan_destroy(a)


def test_mixing_and_layernorm_entry_points_check_their_arguments():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    mix = lambda a, b: lib.jg_mixing_forward(a, b, pp, None, None, 1e-5, pp, pp, pp, pp, pp, pp, pp, 256, 1 << 20)
    a = jg.jg_plan_create(None, 64, 32, 48, 2, True)
    assert mix(None, a) == jg.JG_E_NULL
    for (M, K, N), ways, want in (((64, 48, 30), 2, jg.JG_E_SHAPE), ((64, 48, 32), 4, jg.JG_E_WAYS),
                                  ((64, 48, 32), 2, jg.JG_E_NULL)):      # chains, but no context
        b = jg.jg_plan_create(None, M, K, N, ways, True)
        assert mix(a, b) == want
        jg.jg_plan_destroy(b)
    assert lib.jg_layernorm_forward(None, pp, None, None, 1e-5, pp) == jg.JG_E_NULL
    assert lib.jg_layernorm_forward(a, pp, None, None, 1e-5, pp) == jg.JG_E_NULL     # a plan without a context
    jg.jg_plan_destroy(a)


def test_reduced_precision_plans_account_for_their_shards():
    M, K, N = 64, 272, 32        # K / 2 = 136: padded to 192 per plane
    for ways in (1, 2, 4):
        f = jg.jg_plan_create(None, M, K, N, ways)
        h = jg.jg_plan_create(None, M, K, N, ways, dtype=jg.JG_BF16)
        s = jg.jg_plan_create(None, M, K, N, ways, dtype=jg.JG_BF16X3)
        q = jg.jg_plan_query
        for r in range(ways):
            xe = q(f, jg.JG_Q_X_ROWS, r) * q(f, jg.JG_Q_X_COLS, r)
            we = q(f, jg.JG_Q_W_ROWS, r) * q(f, jg.JG_Q_W_COLS, r)
            assert q(f, jg.JG_Q_X_SHARD_BYTES, r) == 4 * xe and q(f, jg.JG_Q_W_SHARD_BYTES, r) == 4 * we
            # bfloat16 shard rows are padded to whole 128-byte lines (64 values) per plane
            xrows, wrows = q(f, jg.JG_Q_X_ROWS, r), q(f, jg.JG_Q_W_ROWS, r)
            plane = (q(f, jg.JG_Q_X_COLS, r) + 63) // 64 * 64
            assert q(h, jg.JG_Q_X_SHARD_BYTES, r) == 2 * xrows * plane and q(h, jg.JG_Q_W_SHARD_BYTES, r) == 2 * wrows * plane
            assert q(s, jg.JG_Q_X_SHARD_BYTES, r) == 4 * xrows * plane and q(s, jg.JG_Q_W_SHARD_BYTES, r) == 4 * wrows * plane
            assert q(h, jg.JG_Q_X_COLS, r) == q(f, jg.JG_Q_X_COLS, r)          # logical sizes do not change
        assert q(h, jg.JG_Q_FLOPS_TOTAL) == q(f, jg.JG_Q_FLOPS_TOTAL) == 2 * M * K * N
        extra = 8 * M * N if ways >= 2 else 0
        assert q(f, jg.JG_Q_HBM_BYTES_ALGO) == 4 * (M * K + N * K + M * N) + extra
        assert q(h, jg.JG_Q_HBM_BYTES_ALGO) == 2 * (M * K + N * K) + 4 * M * N + extra
        assert q(s, jg.JG_Q_HBM_BYTES_ALGO) == 4 * (M * K + N * K + M * N) + extra
        # split tail of the bfloat16 kernel: one 256 x 256 scratch tile of floats per CU (256 CUs without a context)
        assert q(h, jg.JG_Q_TAIL_SCRATCH_BYTES) == q(s, jg.JG_Q_TAIL_SCRATCH_BYTES) == 256 * 256 * 256 * 4
        w = jg.jg_plan_create(None, M, K, N, ways, dtype=jg.JG_BF16, tail=jg.JG_TAIL_WHOLE)
        assert q(w, jg.JG_Q_TAIL_SCRATCH_BYTES) == 0
        assert q(w, jg.JG_Q_WORKSPACE_BYTES) == q(h, jg.JG_Q_WORKSPACE_BYTES) - q(h, jg.JG_Q_TAIL_SCRATCH_BYTES)
        jg.jg_plan_destroy(w)
        # backward: the FP32 partials of the FP32 plan, plus every operand rounded into the workspace - dY_r twice
        # (rows as they are; contraction-major over the tokens), the weight blocks and X_r contraction-major
        up = lambda n: (n + 255) // 256 * 256
        mr, kh, nh = q(f, jg.JG_Q_X_ROWS), q(f, jg.JG_Q_X_COLS), q(f, jg.JG_Q_Y_COLS)
        pn, pm = (nh + 63) // 64 * 64, (mr + 63) // 64 * 64
        wblocks = 2 if ways == 2 else 1
        for p, eb in ((h, 2), (s, 4)):
            partials = q(f, jg.JG_Q_BACKWARD_WORKSPACE_BYTES) - q(f, jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES)
            cvt = ways * (up(eb * mr * pn) + up(eb * nh * pm) + wblocks * up(eb * kh * pn) + up(eb * kh * pm))
            assert q(p, jg.JG_Q_BACKWARD_WORKSPACE_BYTES) - q(p, jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES) == partials + cvt
            assert q(p, jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES) == q(p, jg.JG_Q_TAIL_SCRATCH_BYTES)
            assert q(p, jg.JG_Q_BACKWARD_FLOPS_TOTAL) == 4 * M * K * N
        if ways == 4:   # the received weight block is bfloat16 too
            assert (q(h, jg.JG_Q_WORKSPACE_BYTES) - q(h, jg.JG_Q_TAIL_SCRATCH_BYTES)
                    < q(f, jg.JG_Q_WORKSPACE_BYTES) - q(f, jg.JG_Q_TAIL_SCRATCH_BYTES))
        # as a layer of an MLP chain a reduced-precision plan also holds its input, rounded: ways shards, 256-byte pieces
        up = lambda n: (n + 255) // 256 * 256
        assert q(f, jg.JG_Q_CHAIN_WORKSPACE_BYTES) == q(f, jg.JG_Q_WORKSPACE_BYTES)
        for p in (h, s):
            assert (q(p, jg.JG_Q_CHAIN_WORKSPACE_BYTES)
                    == q(p, jg.JG_Q_WORKSPACE_BYTES) + ways * up(q(p, jg.JG_Q_X_SHARD_BYTES, 0)))
        for p in (f, h, s):
            jg.jg_plan_destroy(p)


def test_chain_refuses_plans_of_different_precision():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    call = lambda a, b: lib.jg_mlp_forward(a, b, pp, pp, pp, pp, pp, pp, pp, 256, 1 << 30)
    kinds = {d: (jg.jg_plan_create(None, 64, 32, 48, 2, True, dtype=d), jg.jg_plan_create(None, 64, 48, 32, 2, True, dtype=d))
             for d in (jg.JG_F32, jg.JG_BF16, jg.JG_BF16X3)}
    for d1, (a, _) in kinds.items():
        for d2, (_, b) in kinds.items():
            assert call(a, b) == (jg.JG_E_NULL if d1 == d2 else jg.JG_E_DTYPE)      # same precision: chains, but no context
    for a, b in kinds.values():
        jg.jg_plan_destroy(a)
        jg.jg_plan_destroy(b)
    # the FP32 selector is a valid tensor name for data calls (which then miss the context)
    a = jg.jg_plan_create(None, 64, 32, 48, 2, True, dtype=jg.JG_BF16)
    assert lib.jg_shard(a, jg.JG_T_X_F32, 256, 32, pp) == jg.JG_E_NULL
    assert lib.jg_shard(a, jg.JG_T_W_F32, 256, 32, pp) == jg.JG_E_NULL
    assert lib.jg_shard(a, 6, 256, 32, pp) == jg.JG_E_DTYPE
    jg.jg_plan_destroy(a)


def test_patch_calls_check_sizes_against_the_plan():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    # 2 channels, 8 x 16 field, 4 x 4 patches: 8 patches of 32 features
    p = jg.jg_plan_create(None, 8, 32, 6, 2)
    call = lambda C, H, W, ps: lib.jg_shard_patches(p, 256, C, H, W, ps, pp)
    assert call(2, 8, 16, 4) == jg.JG_E_NULL          # sizes fit; the plan has no context
    assert call(2, 8, 16, 3) == jg.JG_E_SHAPE         # patch size does not divide the field
    assert call(2, 8, 8, 4) == jg.JG_E_SHAPE          # 4 patches, the plan has 8 rows
    assert call(1, 8, 16, 4) == jg.JG_E_SHAPE         # 16 features, the plan has 32
    assert call(2, 8, 16, 0) == jg.JG_E_SHAPE
    assert lib.jg_shard_patches(p, None, 2, 8, 16, 4, pp) == jg.JG_E_NULL
    assert lib.jg_shard_patches(p, 258, 2, 8, 16, 4, pp) == jg.JG_E_ALIGN
    # decoder side: the features are the plan's N
    q = jg.jg_plan_create(None, 8, 6, 32, 2)
    assert lib.jg_gather_patches(q, pp, 256, 2, 8, 16, 4) == jg.JG_E_NULL
    assert lib.jg_gather_patches(p, pp, 256, 2, 8, 16, 4) == jg.JG_E_SHAPE
    t = jg.jg_plan_create(None, 32, 8, 6, 2, op=jg.JG_OP_XTW)
    assert lib.jg_shard_patches(t, 256, 2, 8, 16, 4, pp) == jg.JG_E_DTYPE
    for h in (p, q, t):
        jg.jg_plan_destroy(h)


def test_token_mixing_entry_point_checks_that_the_plans_chain():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    call = lambda a, b: lib.jg_token_mixing_forward(a, b, pp, None, None, 1e-5, pp, pp, pp, None, pp, pp, pp, 256, 1 << 20)
    T, C, D = 64, 32, 48
    first = jg.jg_plan_create(None, C, T, D, 2, True, op=jg.JG_OP_XTW)      # K = T tokens, M = C channels, N = D hidden
    assert call(None, first) == jg.JG_E_NULL
    for (M, K, N), ways, bias, want in (((T, D, C), 2, False, jg.JG_E_NULL),          # chains, but no context
                                        ((T, D, C), 2, True, jg.JG_E_DTYPE),          # the second bias goes with the token
                                        ((T, D, C), 4, False, jg.JG_E_WAYS),
                                        ((T, D, C + 2), 2, False, jg.JG_E_SHAPE),
                                        ((T + 2, D, C), 2, False, jg.JG_E_SHAPE),
                                        ((T, D + 2, C), 2, False, jg.JG_E_SHAPE)):
        second = jg.jg_plan_create(None, M, K, N, ways, bias)
        assert call(first, second) == want
        jg.jg_plan_destroy(second)
    plain = jg.jg_plan_create(None, T, D, C, 2, False)
    assert call(plain, plain) == jg.JG_E_DTYPE                                          # the first layer is the transposed one
    assert call(first, first) == jg.JG_E_DTYPE
    half = jg.jg_plan_create(None, C, T, D, 2, True, op=jg.JG_OP_XTW)
    q = jg.jg_plan_query
    assert q(first, jg.JG_Q_X_F32_SHARDS_BYTES) == 2 * ((4 * q(first, jg.JG_Q_X_ROWS) * q(first, jg.JG_Q_X_COLS) + 255) // 256 * 256)
    for p in (plain, half, first):
        jg.jg_plan_destroy(p)


def test_bias_backward_checks_its_arguments():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    assert lib.jg_bias_backward(None, pp, pp, None, 0) == jg.JG_E_NULL
    a = jg.jg_plan_create(None, 64, 32, 48, 2, True)
    assert lib.jg_bias_backward(a, pp, pp, None, 0) == jg.JG_E_NULL          # a plan without a context
    jg.jg_plan_destroy(a)


def test_layernorm_backward_checks_its_arguments():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    call = lambda plan: lib.jg_layernorm_backward(plan, pp, None, 1e-5, pp, pp, None, None, 256, 1 << 20)
    assert call(None) == jg.JG_E_NULL
    a = jg.jg_plan_create(None, 64, 32, 48, 2, True)
    assert call(a) == jg.JG_E_NULL                                      # a plan without a context
    # two doubles per row of a rank's block, in 256-byte pieces; then the one-pass form's column sums: a rank's
    # 64 rows x 16 columns go to 64 bands of one row, two doubles per column and band
    assert jg.jg_plan_query(a, jg.JG_Q_NORM_BACKWARD_WORKSPACE_BYTES) == 2 * ((16 * 64 + 255) // 256 * 256) + 2 * 64 * 16 * 16
    jg.jg_plan_destroy(a)
    # the 1B model's channel mixing: one band of rows per compute unit and workgroup slot
    for ways, blocks, rows, cols, bands in ((1, 1, 16200, 4320, 256), (2, 2, 16200, 2160, 256), (4, 4, 8100, 2160, 128)):
        b = jg.jg_plan_create(None, 16200, 4320, 4320, ways)
        per = -(-rows // bands)
        nbands = -(-rows // per)
        stats = ways * ((16 * rows + 255) // 256 * 256)
        assert jg.jg_plan_query(b, jg.JG_Q_NORM_BACKWARD_WORKSPACE_BYTES) == stats + blocks * nbands * cols * 16
        jg.jg_plan_destroy(b)


def test_mlp_and_mixing_backward_check_that_the_plans_chain():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    mlp = lambda a, b: lib.jg_mlp_backward(a, b, *([pp] * 14), 256, 1 << 20)
    mix = lambda a, b: lib.jg_mixing_backward(a, b, pp, None, 1e-5, *([pp] * 15), None, None, 256, 1 << 20)
    a = jg.jg_plan_create(None, 64, 32, 48, 2, True)
    for call in (mlp, mix):
        assert call(None, a) == jg.JG_E_NULL and call(a, None) == jg.JG_E_NULL
        for (M, K, N), ways, want in (((64, 48, 30), 2, jg.JG_E_SHAPE), ((62, 48, 32), 2, jg.JG_E_SHAPE),
                                      ((64, 48, 32), 4, jg.JG_E_WAYS), ((64, 48, 32), 2, jg.JG_E_NULL)):
            b = jg.jg_plan_create(None, M, K, N, ways, True)
            assert call(a, b) == want
            jg.jg_plan_destroy(b)
        t = jg.jg_plan_create(None, 48, 64, 32, 2, True, op=jg.JG_OP_XTW)
        assert call(a, t) == jg.JG_E_DTYPE
        jg.jg_plan_destroy(t)
    jg.jg_plan_destroy(a)


def test_token_mixing_backward_checks_that_the_plans_chain():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    call = lambda a, b: lib.jg_token_mixing_backward(a, b, pp, None, 1e-5, *([pp] * 14), None, None, None, 256, 1 << 20)
    first = jg.jg_plan_create(None, 32, 64, 48, 2, True, op=jg.JG_OP_XTW)        # T = 64, C = 32, D = 48
    assert call(None, first) == jg.JG_E_NULL
    for (M, K, N), ways, bias, want in (((64, 48, 32), 2, True, jg.JG_E_DTYPE),   # the second layer carries no bias
                                        ((64, 48, 30), 2, False, jg.JG_E_SHAPE),
                                        ((64, 48, 32), 4, False, jg.JG_E_WAYS),
                                        ((64, 48, 32), 2, False, jg.JG_E_NULL)):  # chains, but no context
        second = jg.jg_plan_create(None, M, K, N, ways, bias)
        assert call(first, second) == want
        jg.jg_plan_destroy(second)
    plain = jg.jg_plan_create(None, 64, 48, 32, 2, False)
    assert call(plain, plain) == jg.JG_E_DTYPE                                    # the first layer must be the transposed one
    jg.jg_plan_destroy(plain)
    jg.jg_plan_destroy(first)


def test_reduced_precision_transposed_plans_account_for_their_shards():
    M, K, N = 36, 272, 20        # X is K x M, W is K x N; the shards are stored contraction-major
    for ways in (1, 2, 4):
        f = jg.jg_plan_create(None, M, K, N, ways, op=jg.JG_OP_XTW)
        h = jg.jg_plan_create(None, M, K, N, ways, op=jg.JG_OP_XTW, dtype=jg.JG_BF16)
        s = jg.jg_plan_create(None, M, K, N, ways, op=jg.JG_OP_XTW, dtype=jg.JG_BF16X3)
        q = jg.jg_plan_query
        for r in range(ways):
            kr = q(f, jg.JG_Q_X_ROWS, r)                       # the rank's share of the contracted dimension
            plane = (kr + 63) // 64 * 64
            xc, wc = q(f, jg.JG_Q_X_COLS, r), q(f, jg.JG_Q_W_COLS, r)
            assert q(h, jg.JG_Q_X_SHARD_BYTES, r) == 2 * xc * plane and q(h, jg.JG_Q_W_SHARD_BYTES, r) == 2 * wc * plane
            assert q(s, jg.JG_Q_X_SHARD_BYTES, r) == 4 * xc * plane and q(s, jg.JG_Q_W_SHARD_BYTES, r) == 4 * wc * plane
            assert (q(h, jg.JG_Q_X_ROWS, r), q(h, jg.JG_Q_X_COLS, r)) == (kr, xc)      # logical sizes do not change
        assert q(h, jg.JG_Q_FLOPS_TOTAL) == 2 * M * K * N
        extra = 8 * M * N if ways == 4 else 0
        assert q(h, jg.JG_Q_HBM_BYTES_ALGO) == 2 * (M * K + N * K) + 4 * M * N + extra
        if ways >= 2:   # the activation block a rank receives is bfloat16 too
            assert (q(h, jg.JG_Q_WORKSPACE_BYTES) - q(h, jg.JG_Q_TAIL_SCRATCH_BYTES)
                    < q(f, jg.JG_Q_WORKSPACE_BYTES) - q(f, jg.JG_Q_TAIL_SCRATCH_BYTES))
        # backward: the FP32 plan's partials, plus W_r, dY_r and X_r rounded as they are and every block of dY_r
        # contraction-major
        up = lambda n: (n + 255) // 256 * 256
        tr, ch, dh, yr = q(f, jg.JG_Q_X_ROWS), q(f, jg.JG_Q_X_COLS), q(f, jg.JG_Q_W_COLS), q(f, jg.JG_Q_Y_ROWS)
        pd, pc = (dh + 63) // 64 * 64, (ch + 63) // 64 * 64
        yblocks = 2 if ways == 2 else 1
        for p, eb in ((h, 2), (s, 4)):
            partials = q(f, jg.JG_Q_BACKWARD_WORKSPACE_BYTES) - q(f, jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES)
            cvt = ways * (up(eb * tr * pd) + up(eb * yr * pd) + up(eb * tr * pc) + yblocks * up(eb * dh * pc))
            assert q(p, jg.JG_Q_BACKWARD_WORKSPACE_BYTES) - q(p, jg.JG_Q_BACKWARD_TAIL_SCRATCH_BYTES) == partials + cvt
        for p in (f, h, s):
            jg.jg_plan_destroy(p)


def test_token_mixing_chain_takes_two_plans_of_one_precision():
    lib = jg.raw()
    arr = (ctypes.c_void_p * 2)(256, 512)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
    # (a workspace size that passes the size check: nothing is touched, the plans have no context)
    fwd = lambda a, b: lib.jg_token_mixing_forward(a, b, pp, None, None, 1e-5, pp, pp, pp, None, pp, pp, pp, 256, 1 << 30)
    bwd = lambda a, b: lib.jg_token_mixing_backward(a, b, pp, None, 1e-5, *([pp] * 14), None, None, None, 256, 1 << 30)
    T, C, D = 64, 32, 48
    plans = {}
    for dt in (jg.JG_F32, jg.JG_BF16, jg.JG_BF16X3):
        plans[dt] = (jg.jg_plan_create(None, C, T, D, 2, True, op=jg.JG_OP_XTW, dtype=dt),
                     jg.jg_plan_create(None, T, D, C, 2, False, dtype=dt))
    for dt, (f, s) in plans.items():
        assert fwd(f, s) == jg.JG_E_NULL                                   # chains; the plans have no context
        assert bwd(f, s) == jg.JG_E_NULL
        for other, (f2, s2) in plans.items():
            if other != dt:
                assert fwd(f, s2) == jg.JG_E_DTYPE
    for f, s in plans.values():
        jg.jg_plan_destroy(f)
        jg.jg_plan_destroy(s)


@pytest.mark.parametrize("ways", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", [(100, 60, 40), (16200, 4320, 4320), (6, 4, 2)])
def test_accounting_of_the_xw_permutation(ways, M, K, N):
    p = jg.jg_plan_create(None, M, K, N, ways, op=jg.JG_OP_XW)
    q = lambda what, r=0: jg.jg_plan_query(p, what, r)
    try:
        assert q(jg.JG_Q_FLOPS_TOTAL) == 2 * M * K * N and q(jg.JG_Q_BACKWARD_FLOPS_TOTAL) == 4 * M * K * N
        # zero memory redundancy (Sec. 4): the shards tile X [M x K], W [K x N] and Y [M x N] exactly
        assert sum(q(jg.JG_Q_RESIDENT_BYTES_RANK, r) for r in range(ways)) == 4 * (M * K + K * N + M * N)
        assert sum(q(jg.JG_Q_X_ROWS, r) * q(jg.JG_Q_X_COLS, r) for r in range(ways)) == M * K
        assert sum(q(jg.JG_Q_W_ROWS, r) * q(jg.JG_Q_W_COLS, r) for r in range(ways)) == K * N
        assert sum(q(jg.JG_Q_Y_ROWS, r) * q(jg.JG_Q_Y_COLS, r) for r in range(ways)) == M * N
        for r in range(ways):
            assert q(jg.JG_Q_W_SHARD_BYTES, r) == 4 * q(jg.JG_Q_W_ROWS, r) * q(jg.JG_Q_W_COLS, r)
            assert q(jg.JG_Q_W_COLS, r) == q(jg.JG_Q_Y_COLS, r)         # W is split along N like Y
            assert q(jg.JG_Q_W_ROWS, r) == (K // 2 if ways == 4 else K)   # 2-way: all K rows of the column half
        # what a rank gets from its peers: the row neighbour's activation block, 4-way also a weight block
        want = {1: 0, 2: 4 * M * (K // 2), 4: 4 * ((M // 2) * (K // 2) + (K // 2) * (N // 2))}[ways]
        assert q(jg.JG_Q_EXCHANGE_BYTES_RANK) == want
        assert q(jg.JG_Q_GEMM_LAUNCHES) == (1 if ways == 1 else 2)
        ws, tail = q(jg.JG_Q_WORKSPACE_BYTES), q(jg.JG_Q_TAIL_SCRATCH_BYTES)
        if ways == 1:
            assert ws == tail
        else:
            assert ws >= tail + 4 * M * N + ways * want      # partials of every block + the copies of the received blocks
        # the gradients are the other two permutations: their workspaces bound the backward's
        dx = jg.jg_plan_create(None, M, N, K, ways)
        dw = jg.jg_plan_create(None, K, M, N, ways, op=jg.JG_OP_XTW)
        assert q(jg.JG_Q_BACKWARD_WORKSPACE_BYTES) == max(jg.jg_plan_query(dx, jg.JG_Q_WORKSPACE_BYTES),
                                                         jg.jg_plan_query(dw, jg.JG_Q_WORKSPACE_BYTES))
        jg.jg_plan_destroy(dx)
        jg.jg_plan_destroy(dw)
    finally:
        jg.jg_plan_destroy(p)
