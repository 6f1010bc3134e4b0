"""jg_linear_forward_static: the forward pass on the library's fixed device workspace (for callers that cannot
allocate) against jg_linear_forward on a caller's workspace - the same kernels, so the same bits - and against the
oracle at the layer's bar.  Two calls in a row share the array, the second on a smaller layer."""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_05753_amd import binding as jg
from paper_2507_05753_amd import inputs
from paper_2507_05753_amd.layer import JigsawLinear

pytestmark = pytest.mark.gpu

TOL = 1e-6


def run_both(M, K, N, ways, seed, bias, tail):
    X, W, b = inputs.layer_inputs(seed, M, K, N, "R", bias=bias)
    with JigsawLinear(M, K, N, ways, bias=bias, tail=tail) as L:
        L.shard(torch.from_numpy(X).cuda(), torch.from_numpy(W).cuda(), torch.from_numpy(b).cuda() if bias else None)
        if L.ws_bytes:
            L.ws[: L.ws_bytes // 4 * 4].view(torch.float32).fill_(float("nan"))
        L.forward()
        want = L.gather().cpu().numpy()
        for y in L.y:
            y.fill_(float("nan"))
        print(f"static forward: M={M} K={K} N={N} ways={ways} workspace={L.ws_bytes} B", flush=True)
        jg.jg_linear_forward_static(L.plan, [t.data_ptr() for t in L.x], [t.data_ptr() for t in L.w],
                                    [t.data_ptr() for t in L.b] if bias else None, [t.data_ptr() for t in L.y])
        got = L.gather().cpu().numpy()
        torch.cuda.synchronize()
    assert np.array_equal(got, want), f"static workspace result differs, ways={ways}"
    Y64 = oracle.linear(X, W, b if bias else None)
    S = oracle.magnitude(X, W, b if bias else None)
    assert np.all(np.abs(got - Y64) <= TOL * S), float((np.abs(got - Y64) / S).max())


@pytest.mark.parametrize("ways", [1, 2, 4])
def test_two_calls_in_a_row_the_second_smaller(ways):
    # 1000 x 1000 x 1000 is BASELINE config 2 (4 MB of partial products, 4 MB of weight blocks 4-way);
    # the second call leaves most of what the first wrote in the array and must not read it
    run_both(1000, 1000, 1000, ways, seed=2, bias=True, tail=jg.JG_TAIL_WHOLE)
    run_both(300, 264, 200, ways, seed=1, bias=False, tail=jg.JG_TAIL_WHOLE)


def test_split_tail_scratch_in_the_static_array():
    # a long contraction on few tiles: the planner splits the tail and its scratch tiles live in the array too
    run_both(640, 2048, 512, 2, seed=7, bias=True, tail=jg.JG_TAIL_SPLIT)
    run_both(258, 1024, 130, 2, seed=8, bias=False, tail=jg.JG_TAIL_SPLIT)


def test_sizes_beyond_the_array_are_refused():
    ctx = jg.jg_init(0, torch.cuda.current_stream().cuda_stream)
    try:
        plan = jg.jg_plan_create(ctx, 25000, 4000, 4000, 4)        # 400 MB of partial products
        assert jg.jg_plan_query(plan, jg.JG_Q_WORKSPACE_BYTES) > jg.JG_STATIC_WORKSPACE_BYTES
        dummy = torch.zeros(64, device="cuda")
        ptrs = [dummy.data_ptr()] * 4
        with pytest.raises(jg.JigsawError) as e:
            jg.jg_linear_forward_static(plan, ptrs, ptrs, None, ptrs)
        assert e.value.status == jg.JG_E_WORKSPACE
        jg.jg_plan_destroy(plan)
    finally:
        jg.jg_free(ctx)
    assert torch.cuda.memory_allocated() >= 0
