"""revnet_stack_cost walks the same driver as the real calls: its launch count
must equal the launches the event profiler records for the same stack."""
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,shrink", [("c2_stack9", {}), ("c4_bneck12", dict(n=8, depth=3)),
                                         ("c5_stage3", dict(depth=2)), ("c3_stage2", dict(depth=2))])
def test_cost_query_counts_what_is_launched(name, shrink):
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import StackRunner
    cfg = dict(S.STACKS[name], **shrink)
    x, params, dy = S.draw_stack(7, **cfg)
    r = StackRunner(**cfg)
    r.set_params(params)
    X, DY = r.new_pair(x), r.new_pair(dy)
    fwd, bwd = rv.revnet_stack_cost(r.desc, cfg["depth"], cfg["n"], cfg["h"], cfg["w"])
    rv.revnet_profile_begin()
    r.forward(X, X)
    torch.cuda.synchronize()
    f_stats = rv.revnet_profile_end()
    rv.revnet_profile_begin()
    r.backward(X, DY, X, DY)
    torch.cuda.synchronize()
    b_stats = rv.revnet_profile_end()
    for cost, stats, what in ((fwd, f_stats, "forward"), (bwd, b_stats, "backward")):
        launched = sum(s["launches"] for s in stats.values())
        nbytes = sum(s["algorithmic_bytes"] for s in stats.values())
        print(name, what, "cost query:", cost["kernel_launches"], "launched:", launched, flush=True)
        assert cost["kernel_launches"] == launched, (what, cost, stats)
        assert abs(cost["algorithmic_bytes"] - nbytes) <= 1e-9 * nbytes
