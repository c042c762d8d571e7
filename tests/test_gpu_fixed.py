"""GPU parity of the fixed-point residual stream (Section 3.2, "Numerical
error": the x's and y's in fixed point, F and G in floating point) against
the CPU oracle's version of it, and the property it exists for: the backward
pass returns the stack's input bit for bit."""
import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu

FB = 16  # fraction bits: codes of 2^-16, range +-32768


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def split(t):
    c = t.shape[1] // 2
    return np.ascontiguousarray(t[:, :c]), np.ascontiguousarray(t[:, c:])


def run_fixed(cfg, x, params, dy, frac_bits=FB):
    import torch
    from paper_1707_04585_amd.torch_harness import StackRunner, download_grads
    r = StackRunner(frac_bits=frac_bits, **cfg)
    r.set_params(params)
    X = r.new_stream_pair(x)
    codes_in = X[0].clone()
    r.forward(X, X)
    torch.cuda.synchronize()
    codes_y = X[0].clone()
    y = r.stream_to_host(X[0])
    DY = r.new_pair(dy)
    r.backward(X, DY, X, DY)
    torch.cuda.synchronize()
    return dict(codes_in=codes_in, codes_y=codes_y, codes_rec=X[0].clone(), y=y, dx=r.to_host(DY[0]),
                grads=download_grads(r.grads), runner=r)


@pytest.mark.parametrize("name,cfg", [
    ("basic_f32_24_blocks", dict(kind="basic", n=8, c=32, h=16, w=16, depth=24, width=None, conv="f32", affine="random")),
    ("basic_bf16_24_blocks", dict(kind="basic", n=8, c=32, h=16, w=16, depth=24, width=None, conv="bf16", affine="random")),
    # 150 basic blocks = 600 convolution layers, the depth of the network the paper's appendix on memory savings mentions
    ("basic_bf16_150_blocks", dict(kind="basic", n=4, c=16, h=8, w=8, depth=150, width=None, conv="bf16", affine="random")),
    ("bottleneck_bf16_12_blocks_ragged", dict(kind="bottleneck", n=3, c=96, h=9, w=7, depth=12, width=24, conv="bf16", affine="random")),
    # whole 128-pixel tiles: inside F and G the 1x1 convolutions hand their outputs' statistics to the next BN
    # layer, in the forward pass and in the recomputation alike
    ("bottleneck_bf16_12_blocks_tiles", dict(kind="bottleneck", n=8, c=64, h=16, w=16, depth=12, width=16, conv="bf16", affine="random")),
    ("bottleneck_bf16_6_blocks_shares", dict(kind="bottleneck", n=16, c=512, h=8, w=8, depth=6, width=128, conv="bf16", affine="random")),
])
def test_fixed_stream_reconstructs_bit_for_bit(oracle, torch_cuda, name, cfg):
    """The reconstructed input codes equal the input codes exactly, at depths
    where the floating-point stream has drifted by 1e-5 (fp32 operands) or by
    tens of per cent (bf16 operands)."""
    import torch
    from paper_1707_04585_amd.torch_harness import StackRunner
    x, params, dy = S.draw_stack(555, **cfg)
    out = run_fixed(cfg, x, params, dy)
    assert not torch.equal(out["codes_y"], out["codes_in"])
    assert torch.equal(out["codes_rec"], out["codes_in"]), "fixed-point reconstruction is not exact"
    assert np.isfinite(out["dx"]).all()
    # for comparison: the same stack with the floating-point stream
    r = StackRunner(**cfg)
    r.set_params(params)
    X, DY = r.new_pair(x), r.new_pair(dy)
    r.forward(X, X)
    r.backward(X, DY, X, DY)
    torch.cuda.synchronize()
    print(f"{name}: fixed-point stream reconstructs exactly; floating-point stream: rel. error "
          f"{oracle.rel_l2(r.to_host(X[0]), x):.2e}", flush=True)


@pytest.mark.parametrize("kind,width", [("basic", None), ("bottleneck", 8)])
def test_fixed_stream_matches_oracle_fp32(oracle, torch_cuda, kind, width):
    """Forward codes and all derivatives against the oracle's fixed-point
    stack (F, G in float64, stored-activation backprop).  After one function
    from identical input codes (y1 of a single block) a code may differ by one
    unit, where the function value times 2^frac_bits lies within fp32 rounding
    distance of a half-integer, and by no more; deeper in, such differences
    travel through the functions like any other rounding difference, so whole
    stacks are held to the fp32 bars on the decoded values."""
    cfg = dict(kind=kind, n=4, c=32, h=12, w=12, depth=3, width=width, conv="f32", affine="random")
    x, params, dy = S.draw_stack(556, **cfg)
    x = x.astype(np.float32).astype(np.float64)   # the GPU is handed fp32 values; encode the same ones
    q1, q2 = (oracle.fixed_encode(t, FB) for t in split(x))
    y1, y2, stored = oracle.stack_fwd_fixed(q1, q2, params, FB, keep=True)
    dx1, dx2, grads = oracle.stack_bwd_stored(stored, params, *split(dy))
    out = run_fixed(cfg, x, params, dy)
    assert np.array_equal(out["codes_in"].cpu().numpy(), np.concatenate([q1, q2], 1)), "encoding differs"
    diff = np.abs(out["codes_y"].cpu().numpy().astype(np.int64) - np.concatenate([y1, y2], 1))
    print("output codes: %.3f%% differ from the oracle's, largest difference %d code(s)" %
          (100.0 * (diff > 0).mean(), diff.max()), flush=True)
    one = run_fixed(dict(cfg, depth=1), x, params[:1], dy)
    o1, _, _ = oracle.stack_fwd_fixed(q1, q2, params[:1], FB, keep=True)
    d1 = np.abs(one["codes_y"].cpu().numpy().astype(np.int64)[:, :cfg["c"] // 2] - o1)
    print("y1 of one block: %.3f%% of the codes differ, by at most %d" % (100.0 * (d1 > 0).mean(), d1.max()), flush=True)
    assert d1.max() <= 1 and (d1 > 0).mean() < 0.02
    y_ref = np.concatenate([oracle.fixed_decode(y1, FB), oracle.fixed_decode(y2, FB)], 1)
    assert oracle.rel_l2(out["y"], y_ref) < 1e-5
    e_dx = oracle.rel_l2(out["dx"], np.concatenate([dx1, dx2], 1))
    worst = 0.0
    for k in range(cfg["depth"]):
        for fn in ("F", "G"):
            for l in range(len(params[k][fn])):
                for key in ("w", "gamma", "beta"):
                    worst = max(worst, oracle.rel_l2(out["grads"][k][fn][l][key], grads[k][fn][l][key]))
    print("rel. errors: dx %.2e, worst parameter gradient %.2e" % (e_dx, worst), flush=True)
    assert e_dx < 1e-4 and worst < 1e-4


def test_fixed_stream_bf16_block_matches_oracle(oracle, torch_cuda):
    """bf16 operands, one block from the oracle's inputs, 2e-2 on gradients."""
    cfg = dict(kind="bottleneck", n=8, c=64, h=14, w=14, depth=1, width=16, conv="bf16", affine="random")
    x, params, dy = S.draw_stack(557, **cfg)
    x = x.astype(np.float32).astype(np.float64)
    q1, q2 = (oracle.fixed_encode(t, FB) for t in split(x))
    with oracle.conv_operands("bf16"):
        y1, y2, stored = oracle.stack_fwd_fixed(q1, q2, params, FB, keep=True)
        dx1, dx2, grads = oracle.stack_bwd_stored(stored, params, *split(dy))
    out = run_fixed(cfg, x, params, dy)
    y_ref = np.concatenate([oracle.fixed_decode(y1, FB), oracle.fixed_decode(y2, FB)], 1)
    e_y, e_dx = oracle.rel_l2(out["y"], y_ref), oracle.rel_l2(out["dx"], np.concatenate([dx1, dx2], 1))
    worst = max(oracle.rel_l2(out["grads"][0][fn][l][key], grads[0][fn][l][key])
                for fn in ("F", "G") for l in range(3) for key in ("w", "gamma", "beta"))
    print("rel. errors: y %.2e dx %.2e worst parameter gradient %.2e" % (e_y, e_dx, worst), flush=True)
    assert e_y < 1e-2 and e_dx < 2e-2 and worst < 2e-2


def test_fixed_stream_workspace_and_errors(torch_cuda):
    import paper_1707_04585_amd as rv
    d = rv.BlockDesc("basic", 16)
    f0, b0 = rv.revnet_workspace_bytes(d, 8, 16, 16)
    f1, b1 = rv.revnet_fixed_workspace_bytes(d, 8, 16, 16)
    assert f1 > f0 and b1 > b0    # two more half-stream tensors
    assert f1 - f0 >= 2 * 8 * 16 * 256 * 4


@pytest.mark.parametrize("conv", ["f32", "bf16"])
def test_fixed_point_body_reconstructs_every_stage_and_matches_oracle(oracle, torch_cuda, conv):
    """Three stages joined by two subsampling blocks with the stage tensors in
    fixed point: after the backward pass every top holds the codes the stage
    received (stage 0: the encoded input; later stages: what the subsampling
    block below wrote), bit for bit; tops and derivatives against the oracle's
    fixed-point body (fp32 / bf16 bars; a tensor above its bar must be within
    1.5x its own float32-to-float64 oracle distance, of both oracle runs)."""
    import torch
    from paper_1707_04585_amd.torch_harness import BodyRunner, download_grads, download_down, _dev
    from test_gpu_body import body_errors, cast_down
    cfg = dict(kind="basic", n=4, h=16, w=16, channels=(8, 12, 16), depths=(3, 2, 3), widths=(None, None, None), conv=conv)
    x, stages, downs, dy = S.draw_body(2026, **cfg)
    x = x.astype(np.float32).astype(np.float64)
    with oracle.conv_operands(conv):
        tops_ref, kept = oracle.body_fwd_fixed(x, stages, downs, FB)
        dx_ref, sg_ref, dg_ref = oracle.body_bwd_stored(kept, stages, downs, dy)
        st32 = [S.cast_params(st, np.float32) for st in stages]
        dn32 = [cast_down(P, np.float32) for P in downs]
        t32, k32 = oracle.body_fwd_fixed(x, st32, dn32, FB, np.float32(1e-5), np.float32)
        dx32, sg32, dg32 = oracle.body_bwd_stored(k32, st32, dn32, dy.astype(np.float32), np.float32(1e-5))
    dec = lambda tops: [oracle.fixed_decode(t, FB) for t in tops]
    o32 = dict(tops=dec(t32), x_rec=x, dx=dx32, stage_grads=sg32, down_grads=dg32)
    f_fwd, _, f_dx, f_g = body_errors(oracle, o32, dec(tops_ref), dx_ref, sg_ref, dg_ref, x)
    base = dict(f32=dict(fwd=1e-5, grad=1e-4), bf16=dict(fwd=1e-2, grad=2e-2))[conv]
    tol = dict(fwd=max(base["fwd"], 1.5 * f_fwd), grad=base["grad"])

    r = BodyRunner(frac_bits=FB, **cfg)
    r.set_params(stages, downs)
    r.forward(_dev(x, "cuda:0"))
    torch.cuda.synchronize()
    tops = [r.top_to_host(s) for s in range(3)]
    # what each stage received: the encoded input, and the codes each subsampling block wrote
    received = [torch.empty_like(t) for t in r.tops]
    import paper_1707_04585_amd as rv
    rv.revnet_fixed_from_float(_dev(x, "cuda:0"), FB, received[0])
    codes_top = [t.clone() for t in r.tops]
    r.dtops[-1].copy_(_dev(dy, "cuda:0"))
    r.backward()
    torch.cuda.synchronize()
    assert torch.equal(r.tops[0].view(torch.int32), received[0].view(torch.int32)), "stage 0 input not reconstructed exactly"
    # a second forward + backward leaves the same codes everywhere (the pass is reproducible)
    after_first = [t.clone() for t in r.tops]
    r.forward(_dev(x, "cuda:0"))
    torch.cuda.synchronize()
    for s in range(3):
        assert torch.equal(r.tops[s].view(torch.int32), codes_top[s].view(torch.int32))
    r.dtops[-1].copy_(_dev(dy, "cuda:0"))
    r.backward()
    torch.cuda.synchronize()
    for s in range(3):
        assert torch.equal(r.tops[s].view(torch.int32), after_first[s].view(torch.int32))
    out = dict(tops=tops, x_rec=x, dx=r.dtops[0].cpu().numpy().astype(np.float64),
               stage_grads=[download_grads(g) for g in r.stage_grads], down_grads=[download_down(g) for g in r.down_grads])
    fwd, _, dx, g = body_errors(oracle, out, dec(tops_ref), dx_ref, sg_ref, dg_ref, x)
    worst = max(g, key=g.get)
    print(f"fixed-point body conv={conv}: tops {fwd:.2e} dx {dx:.2e} worst gradient {worst} {g[worst]:.2e} (tolerances {tol})", flush=True)
    assert fwd < tol["fwd"]
    _, _, v_dx, v_g = body_errors(oracle, out, dec(t32), dx32, sg32, dg32, x)
    from parity_checks import check_with_floors, record
    used = check_with_floors(dict(g, dx=dx), dict(f_g, dx=f_dx), dict(v_g, dx=v_dx), tol["grad"], pooled=conv == "f32")
    record(f"fixed_point_body/{conv}", conv=conv, y=fwd, dx=dx, worst_param=g[worst], worst_param_name=worst, bar=tol["grad"],
           dx_floor=f_dx, worst_param_floor=f_g[worst], dx_vs_f32_oracle=v_dx, worst_fraction_of_allowance=used)
    # stage 1's reconstructed input equals the codes of the subsampling block's output: recompute that output
    rec1 = r.tops[1].view(torch.int32).cpu().numpy().astype(np.int64)
    with oracle.conv_operands(conv):
        y0, _ = oracle.down_fwd(oracle.fixed_decode(codes_top[0].view(torch.int32).cpu().numpy().astype(np.int64), FB), downs[0])
    diff = np.abs(rec1 - oracle.fixed_encode(y0, FB))
    print("  stage 1 input codes against the oracle's subsampling block on the GPU's stage-0 top: largest difference %d code(s), %.2f%% differ" %
          (diff.max(), 100.0 * (diff > 0).mean()), flush=True)
    assert diff.max() <= (2 if conv == "f32" else 600)
