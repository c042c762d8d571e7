"""revnet_stack_fwd_static -- the forward entry point whose workspace is an
array inside the library's device image (for callers that cannot allocate) --
against revnet_stack_fwd on the same inputs.  Same kernels, same driver, so
the results have to be the same bits; the fp32 forward bar (1e-5) is asserted
as well.  Two calls in a row share the one array, the second on a smaller
input, and the array's stale contents must not leak into it."""
import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu


def _run_pair(rv, torch, cfg, seed):
    from paper_1707_04585_amd.torch_harness import StackRunner
    x, params, _ = S.draw_stack(seed, **cfg)
    r = StackRunner(**cfg)
    r.set_params(params)
    assert r.fwd_bytes <= rv.STATIC_WS_BYTES
    X, Y_ref, Y_new = r.new_pair(x), r.new_pair(), r.new_pair()
    rv.revnet_stack_fwd(r.desc, r.depth, X[1], X[2], r._pp, Y_ref[1], Y_ref[2], r.ws)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rv.revnet_stack_fwd_static(r.desc, r.depth, X[1], X[2], r._pp, Y_new[1], Y_new[2])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return r.to_host(Y_ref[0]), r.to_host(Y_new[0])


def test_static_workspace_forward_matches_caller_workspace_forward(oracle):
    import torch
    import paper_1707_04585_amd as rv
    assert torch.cuda.is_available()
    big = dict(kind="bottleneck", n=6, c=64, h=16, w=16, depth=3, width=16, conv="bf16", affine="random")
    small = dict(kind="basic", n=3, c=10, h=7, w=9, depth=2, width=None, conv="f32", affine="random")
    for cfg, seed in ((big, 501), (small, 502)):   # the second call finds the first one's leftovers
        print("case", cfg, flush=True)
        ref, got = _run_pair(rv, torch, cfg, seed)
        assert oracle.rel_l2(got, ref) < 1e-5
        np.testing.assert_array_equal(got, ref)
