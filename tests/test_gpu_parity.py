"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.

Tolerances (per-tensor relative L2 error, float64 oracle as reference):
  fp32 path : forward 1e-5, gradients 1e-4
  bf16 convolution operands : gradients 2e-2 (forward and reconstruction 1e-2)
The reference gradient is the ordinary stored-activation one, so the tolerance
covers both fp32 rounding and reconstruction drift.

For the bf16 path the oracle rounds the operands of its convolutions to bf16
as well (and still sums in float64): rounding moves a fraction ~1e-3 of the
pre-activations across zero, each flipped ReLU derivative changes its gradient
element by O(1), and that alone is a 5-10% relative L2 difference from the
unrounded gradient at any size.  The 0/1 decisions are therefore taken in the
kernel's operand precision on both sides; the distance to the unrounded
float64 gradient is printed for information.
"""
import numpy as np
import pytest

import synth_inputs as S
from bf16_floor import bf16_grad_floor
from parity_checks import assert_structure, record, PAIR_FACTOR

pytestmark = pytest.mark.gpu

# bf16 operands make a residual function ill-conditioned with respect to
# summation order: a relative difference d entering a rounding step (fp32 sums on
# the GPU, float64 sums in the oracle: d ~ 1e-7) moves a fraction d / 2^-8 of the
# values to the neighbouring bf16 number, i.e. leaves a relative difference
# sqrt(d * 2^-8); three layers take 1e-7 to 2e-5, 3e-4 and 1e-3, and at 1e-3 about
# one ReLU decision in a thousand differs, each an O(1) change of its gradient
# element: sqrt(1e-3) = 3e-2.  No kernel can be closer to a float64-summing oracle
# than another correct summation order is.  That floor is measured, on the CPU
# and with the oracle alone, as the distance between the oracle run in float32
# and in float64 (both with bf16 operands); the GPU must stay within the 2e-2 bar
# or, where the floor is above it, within 1.5x the floor of both oracle runs.
FLOOR_FACTOR = 1.5


def bf16_grad_tol(oracle, cfg, x, params, dy, ref):
    """(floor of dx, the float32 oracle's outputs): see check_against_oracle."""
    floor, r32 = bf16_grad_floor(oracle, cfg, x, params, dy, ref, want32=True)
    print("  bf16 floor (oracle float32 vs float64, dx): %.2e" % floor, flush=True)
    return floor, r32


TOL = {"f32": dict(fwd=1e-5, grad=1e-4, recon=1e-5), "bf16": dict(fwd=1e-2, grad=2e-2, recon=1e-2)}


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def split(t):
    c = t.shape[1] // 2
    return np.ascontiguousarray(t[:, :c]), np.ascontiguousarray(t[:, c:])


def oracle_reference(oracle, cfg, x, params, dy):
    x1, x2 = split(x)
    dy1, dy2 = split(dy)
    with oracle.conv_operands(cfg.get("conv", "f32")):
        y1, y2, inputs, stored = oracle.stack_fwd(x1, x2, params, eps=cfg.get("eps", 1e-5), keep=True)
        dx1, dx2, grads = oracle.stack_bwd_stored(stored, params, dy1, dy2, eps=cfg.get("eps", 1e-5))
    return dict(y=np.concatenate([y1, y2], 1), dx=np.concatenate([dx1, dx2], 1), grads=grads, inputs=inputs)


def gpu_run(cfg, x, params, dy, inplace=True, split_buffers=False, accumulate=False, repeat_bwd=1):
    from paper_1707_04585_amd.torch_harness import StackRunner, download_grads
    import torch
    r = StackRunner(split_buffers=split_buffers, **cfg)
    r.set_params(params)
    X = r.new_pair(x)
    Y = X if inplace else r.new_pair()
    r.forward(X, Y)
    torch.cuda.synchronize()
    y = r.to_host(Y[0])
    DY = r.new_pair(dy)
    if inplace:
        XR, DX = Y, DY
    else:
        XR, DX = r.new_pair(), r.new_pair()
    for i in range(repeat_bwd):
        if i:   # run backward again from fresh copies of (y, dy)
            Y = r.new_pair(y)
            DY = r.new_pair(dy)
            XR, DX = (Y, DY) if inplace else (XR, DX)
        r.backward(Y, DY, XR, DX, accumulate=accumulate)
    torch.cuda.synchronize()
    return dict(y=y, x_rec=r.to_host(XR[0]), dx=r.to_host(DX[0]), grads=download_grads(r.grads), runner=r)


def error_table(oracle, out, ref, x, scale_grads=1.0):
    """Relative L2 error of every output tensor; parameter gradients keyed
    'k.F.l.w' etc.  A gradient whose reference is zero up to rounding is
    reported as an absolute error over its scale."""
    err = dict(y=oracle.rel_l2(out["y"], ref["y"]), x_rec=oracle.rel_l2(out["x_rec"], x),
               dx=oracle.rel_l2(out["dx"], ref["dx"]))
    for k, (gb, rb) in enumerate(zip(out["grads"], ref["grads"])):
        for fn in ("F", "G"):
            for l, (gl, rl) in enumerate(zip(gb[fn], rb[fn])):
                for key in ("w", "gamma", "beta"):
                    want = scale_grads * rl[key]
                    floor = 1e-6 * max(1.0, float(np.abs(want).max()))
                    if np.linalg.norm(want) < floor:
                        err[f"{k}.{fn}.{l}.{key}"] = float(np.abs(gl[key] - want).max()) / (1e4 * floor)
                    else:
                        err[f"{k}.{fn}.{l}.{key}"] = oracle.rel_l2(gl[key], want)
    return err


def check_against_oracle(oracle, out, ref, x, conv, scale_grads=1.0, tol=None, case=None, floor=None, ref32=None):
    """Every output tensor against the float64 oracle at the bars of `tol`.
    With `ref32` (the float32 oracle's outputs, bf16 cases) a gradient tensor
    that misses the fixed bar may still pass at FLOOR_FACTOR x its own floor
    -- the distance between the two oracle runs for that same tensor -- if the
    GPU is also within PAIR_FACTOR floors of the float32 oracle."""
    tol = tol or TOL[conv]
    err = error_table(oracle, out, ref, x, scale_grads)
    gerr = {k: v for k, v in err.items() if "." in k}
    worst = max(gerr, key=gerr.get)
    print("rel. errors: y %.2e  x_rec %.2e  dx %.2e  worst parameter gradient %s %.2e" %
          (err["y"], err["x_rec"], err["dx"], worst, gerr[worst]), flush=True)
    assert err["y"] < tol["fwd"], ("y", err["y"])
    assert err["x_rec"] < tol["recon"], ("x_rec", err["x_rec"])
    bar = TOL[conv]["grad"] if ref32 is not None else tol["grad"]
    floors, vs32 = {}, {}
    if ref32 is not None:
        as_out = lambda r: dict(y=r["y"], x_rec=x, dx=r["dx"], grads=r["grads"])
        floors = error_table(oracle, as_out(ref32), ref, x, scale_grads)
        vs32 = error_table(oracle, out, dict(y=ref32["y"], dx=ref32["dx"], grads=ref32["grads"]), x, scale_grads)
    worst_ratio = 0.0
    for key in ["dx"] + sorted(gerr):
        e = err[key]
        if e < bar:
            worst_ratio = max(worst_ratio, e / bar)
            continue
        fl = floors.get(key)
        assert fl is not None, (key, e, "above the bar", bar)
        print("  %s: %.2e is above the %.0e bar; floor of this tensor %.2e, GPU against the float32 oracle %.2e" %
              (key, e, bar, fl, vs32[key]), flush=True)
        assert e < FLOOR_FACTOR * fl, (key, e, "floor", fl)
        assert vs32[key] < PAIR_FACTOR * fl, (key, "against the float32 oracle", vs32[key], "floor", fl)
        worst_ratio = max(worst_ratio, e / (FLOOR_FACTOR * fl))
    # inside the tensors: images, channels, border slices, single elements
    dx_bar = max(bar, FLOOR_FACTOR * floors.get("dx", 0.0))
    st = dict(y=assert_structure("y", out["y"], ref["y"], tol["fwd"], smooth=True),
              x_rec=assert_structure("x_rec", out["x_rec"], x, tol["recon"], smooth=True),
              dx=assert_structure("dx", out["dx"], ref["dx"], dx_bar, smooth=False))
    if case:
        record(case, conv=conv, y=err["y"], x_rec=err["x_rec"], dx=err["dx"], worst_param=gerr[worst],
               worst_param_name=worst, bar=bar, dx_floor=floors.get("dx"), worst_param_floor=floors.get(worst),
               dx_vs_f32_oracle=vs32.get("dx"), worst_fraction_of_allowance=worst_ratio,
               dx_per_image=st["dx"]["per_image"], dx_per_channel=st["dx"]["per_channel"], dx_border=st["dx"]["border"],
               y_max_abs_over_rms=st["y"]["max_abs_over_rms"], dx_outliers=st["dx"]["outliers"])
    return err


SMALL_CASES = {
    # name: (cfg, note)
    "c1_single_basic_block": dict(S.STACKS["c1_block"]),
    "basic_ragged_odd_channels": dict(kind="basic", n=3, c=10, h=7, w=9, depth=2, width=None, conv="f32", affine="random"),
    "basic_several_tiles": dict(kind="basic", n=6, c=32, h=32, w=32, depth=2, width=None, conv="f32", affine="random"),
    "basic_c56_8x8": dict(kind="basic", n=8, c=112, h=8, w=8, depth=1, width=None, conv="f32", affine="random"),
    "bottleneck_ragged": dict(kind="bottleneck", n=2, c=24, h=6, w=10, depth=2, width=5, conv="f32", affine="random"),
    "bottleneck_56x56": dict(kind="bottleneck", n=2, c=64, h=56, w=56, depth=1, width=16, conv="f32", affine="random"),
    "bottleneck_7x7_wide": dict(kind="bottleneck", n=4, c=256, h=7, w=7, depth=1, width=64, conv="f32", affine="random"),
    "degenerate_one_pixel": dict(kind="basic", n=1, c=2, h=1, w=1, depth=1, width=None, conv="f32", affine="random"),
    "degenerate_one_row": dict(kind="basic", n=2, c=4, h=1, w=5, depth=1, width=None, conv="f32", affine="random"),
}


@pytest.mark.parametrize("conv", ["f32", "bf16"])
@pytest.mark.parametrize("name", list(SMALL_CASES))
def test_stack_matches_oracle(oracle, torch_cuda, name, conv):
    cfg = dict(SMALL_CASES[name], conv=conv)
    print(f"case {name} conv={conv} cfg={cfg}", flush=True)
    x, params, dy = S.draw_stack(1234, **cfg)
    ref = oracle_reference(oracle, cfg, x, params, dy)
    out = gpu_run(cfg, x, params, dy)
    r32 = bf16_grad_tol(oracle, cfg, x, params, dy, ref)[1] if conv == "bf16" else None
    check_against_oracle(oracle, out, ref, x, conv, case=f"small/{name}/{conv}", ref32=r32)


@pytest.mark.parametrize("kind,c,width,h,w,n", [
    ("basic", 32, None, 16, 16, 8), ("bottleneck", 64, 16, 14, 14, 8),
    # whole 128-pixel tiles: the 1x1 convolutions leave the statistics of their outputs for the next BN layer
    ("bottleneck", 64, 16, 16, 16, 8),
    # ragged shapes for the bf16 kernels: H*W and W not multiples of 4 (unaligned 16-byte loads,
    # quads that run over row ends), channel counts that fill matrix-instruction tiles only partly
    ("bottleneck", 96, 24, 9, 7, 5), ("basic", 48, None, 10, 6, 5), ("bottleneck", 64, 32, 5, 5, 5),
    # the three stages of the 32x32 bf16 workload at their full batch, i.e. in the launch
    # configuration the benchmark times
    ("basic", 32, None, 32, 32, 128), ("basic", 64, None, 16, 16, 128), ("basic", 112, None, 8, 8, 128)])
def test_bf16_every_block_of_a_stack_from_oracle_inputs(oracle, torch_cuda, kind, c, width, h, w, n):
    """bf16 operands, 2e-2 bar, block by block: block k of a 4-block stack gets
    the oracle's (x, y, ybar) of that block, so every block is checked at its
    real statistics without the divergence between two precisions compounding
    through the rounding steps of the blocks above and below it."""
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import StackRunner, download_grads
    cfg = dict(kind=kind, n=n, c=c, h=h, w=w, depth=4, width=width, conv="bf16", affine="random")
    x, params, dy = S.draw_stack(4321, **cfg)
    with oracle.conv_operands("bf16"):
        x1, x2 = split(x)
        y1, y2, inputs, stored = oracle.stack_fwd(x1, x2, params, keep=True)
        outs = inputs[1:] + [(y1, y2)]
        g1, g2 = split(dy)
        ups, downs, grads = [None] * 4, [None] * 4, [None] * 4
        for k in range(3, -1, -1):
            ups[k] = (g1, g2)
            g1, g2, grads[k] = oracle.block_bwd_stored(stored[k], params[k], g1, g2)
            downs[k] = (g1, g2)
    r = StackRunner(**cfg)
    r.set_params(params)
    cat = lambda pr: np.concatenate(pr, axis=1)
    for k in range(4):
        X, Y = r.new_pair(cat(inputs[k])), r.new_pair()
        rv.revnet_block_fwd(r.desc, X[1], X[2], r.params[k], Y[1], Y[2], r.ws)
        torch.cuda.synchronize()
        y_gpu = r.to_host(Y[0])
        Y, DY = r.new_pair(cat(outs[k])), r.new_pair(cat(ups[k]))
        rv.revnet_block_bwd_reconstruct(r.desc, Y[1], Y[2], DY[1], DY[2], r.params[k], Y[1], Y[2], DY[1], DY[2],
                                        r.grads[k], 0, r.ws)
        torch.cuda.synchronize()
        out = dict(y=y_gpu, x_rec=r.to_host(Y[0]), dx=r.to_host(DY[0]), grads=[download_grads(r.grads)[k]])
        ref = dict(y=cat(outs[k]), dx=cat(downs[k]), grads=[grads[k]])
        print(f"block {k}:", end=" ")
        check_against_oracle(oracle, out, ref, cat(inputs[k]), "bf16", case=f"block_by_block/{kind}_c{c}_{h}x{w}_n{n}/block{k}")


def test_block_entry_points_c1(oracle, torch_cuda):
    """revnet_block_fwd / revnet_block_bwd_reconstruct on the single-block
    workload, out of place, against the oracle and against Algorithm 1 run in
    float32 on the CPU."""
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import StackRunner, download_grads
    cfg, x, params, dy = S.draw_named("c1_block")
    ref = oracle_reference(oracle, cfg, x, params, dy)
    r = StackRunner(**cfg)
    r.set_params(params)
    X, Y, DY, XR, DX = r.new_pair(x), r.new_pair(), r.new_pair(dy), r.new_pair(), r.new_pair()
    rv.revnet_block_fwd(r.desc, X[1], X[2], r.params[0], Y[1], Y[2], r.ws)
    rv.revnet_block_bwd_reconstruct(r.desc, Y[1], Y[2], DY[1], DY[2], r.params[0], XR[1], XR[2], DX[1], DX[2],
                                    r.grads[0], 0, r.ws)
    torch.cuda.synchronize()
    out = dict(y=r.to_host(Y[0]), x_rec=r.to_host(XR[0]), dx=r.to_host(DX[0]), grads=download_grads(r.grads))
    check_against_oracle(oracle, out, ref, x, "f32")
    # inputs are untouched by an out-of-place call
    np.testing.assert_array_equal(r.to_host(X[0]), x.astype(np.float32).astype(np.float64))
    np.testing.assert_array_equal(r.to_host(DY[0]), dy.astype(np.float32).astype(np.float64))


def test_in_place_out_of_place_and_split_buffers_agree_bitwise(oracle, torch_cuda):
    cfg = dict(kind="basic", n=4, c=16, h=12, w=12, depth=3, width=None, conv="f32", affine="random")
    x, params, dy = S.draw_stack(77, **cfg)
    a = gpu_run(cfg, x, params, dy, inplace=True)
    b = gpu_run(cfg, x, params, dy, inplace=False)
    c = gpu_run(cfg, x, params, dy, inplace=False, split_buffers=True)
    for other in (b, c):
        for key in ("y", "x_rec", "dx"):
            np.testing.assert_array_equal(a[key], other[key])
        np.testing.assert_array_equal(oracle.flatten_grads(a["grads"]), oracle.flatten_grads(other["grads"]))


def test_runs_are_bitwise_reproducible(oracle, torch_cuda):
    """No floating-point atomics anywhere: two runs give identical bits, which
    is also what makes the recomputed G(y1) equal the forward one."""
    cfg = dict(kind="bottleneck", n=4, c=32, h=14, w=14, depth=2, width=8, conv="bf16", affine="random")
    x, params, dy = S.draw_stack(78, **cfg)
    a = gpu_run(cfg, x, params, dy)
    b = gpu_run(cfg, x, params, dy)
    for key in ("y", "x_rec", "dx"):
        np.testing.assert_array_equal(a[key], b[key])
    np.testing.assert_array_equal(oracle.flatten_grads(a["grads"]), oracle.flatten_grads(b["grads"]))


def test_fresh_buffers_reproduce_bitwise_at_full_size(oracle, torch_cuda):
    """A full-size bf16 stack run from freshly allocated buffers (new addresses,
    stale workspace contents) gives the same bits every time.  The per-channel
    reductions cross workgroups through published partial results and a
    ticket; the ticket must not overtake the partial result it announces, or
    the finishing workgroup reads what an earlier launch left in the scratch
    area -- a plausible value, so only a comparison of bits shows it."""
    cfg, x, params, dy = S.draw_named("c5_stage3")
    ref = None
    for rep in range(4):
        out = gpu_run(cfg, x, params, dy)
        got = (out["y"], out["x_rec"], out["dx"], oracle.flatten_grads(out["grads"]))
        del out
        if ref is None:
            ref = got
            continue
        for name, a, b in zip(("y", "x_rec", "dx", "parameter gradients"), ref, got):
            assert np.array_equal(a, b), f"run {rep}: {name} differ from the first run"


def test_accumulate_wgrads(oracle, torch_cuda):
    """accumulate_wgrads adds to the gradient buffers (weight sharing, footnote
    to Algorithm 1): two backward passes give twice the gradient."""
    cfg = dict(kind="basic", n=3, c=8, h=6, w=6, depth=2, width=None, conv="f32", affine="random")
    x, params, dy = S.draw_stack(79, **cfg)
    ref = oracle_reference(oracle, cfg, x, params, dy)
    out = gpu_run(cfg, x, params, dy, accumulate=True, repeat_bwd=2)
    check_against_oracle(oracle, out, ref, x, "f32", scale_grads=2.0)


@pytest.mark.parametrize("kind,width", [("basic", None), ("bottleneck", 6)])
def test_weight_shared_stack(oracle, torch_cuda, kind, width):
    """Footnote to Algorithm 1 (Section 3.2): when blocks share weights, their
    contributions to the weight derivative are summed.  A 'recurrent' stack --
    the same block applied five times -- through revnet_stack_bwd with every
    block pointing at the same parameter and gradient buffers and
    accumulate_wgrads set, against the sum over blocks of the oracle's
    per-block stored-activation gradients."""
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import StackRunner, download_grads, zeros_like_params
    depth = 5
    cfg = dict(kind=kind, n=4, c=16, h=10, w=10, depth=1, width=width, conv="f32", affine="random")
    x, one, dy = S.draw_stack(83, **cfg)
    one[0]["F"] = [dict(L, w=0.5 * L["w"]) for L in one[0]["F"]]   # keep the five-fold composition tame
    one[0]["G"] = [dict(L, w=0.5 * L["w"]) for L in one[0]["G"]]
    params = one * depth
    cfg["depth"] = depth
    ref = oracle_reference(oracle, cfg, x, params, dy)
    summed = {fn: [{k: sum(ref["grads"][d][fn][l][k] for d in range(depth)) for k in ("w", "gamma", "beta")}
                   for l in range(len(one[0][fn]))] for fn in ("F", "G")}
    r = StackRunner(**cfg)
    r.set_params(one)                       # one block's parameters on the device ...
    shared_p = rv.pack_params([r.params[0]] * depth)    # ... named by every block of the stack
    shared_g = rv.pack_grads([r.grads[0]] * depth)      # gradients start at zero
    X, DY = r.new_pair(x), r.new_pair(dy)
    rv.revnet_stack_fwd(r.desc, depth, X[1], X[2], shared_p, X[1], X[2], r.ws)
    torch.cuda.synchronize()
    y = r.to_host(X[0])
    rv.revnet_stack_bwd(r.desc, depth, X[1], X[2], DY[1], DY[2], shared_p, X[1], X[2], DY[1], DY[2], shared_g, 1, r.ws)
    torch.cuda.synchronize()
    out = dict(y=y, x_rec=r.to_host(X[0]), dx=r.to_host(DY[0]), grads=download_grads(r.grads))
    check_against_oracle(oracle, out, dict(y=ref["y"], dx=ref["dx"], grads=[summed]), x, "f32")


def test_deep_stack_activation_memory_flat_and_drift_small(oracle, torch_cuda):
    """Section 4, Table 1: the activation storage of a reversible stack does not
    depend on its depth; Section 3.2 'Numerical error': the reconstruction error
    grows with depth but stays small.  A 72-block stack against a 2-block one:
    same workspace and same peak device memory around forward + backward (the
    library allocates nothing).  The drift bar comes from the oracle alone: its
    float32 run of Algorithm 1 on the same inputs, against its float64
    stored-activation gradients; the GPU has to stay within 1.5x of that for the
    reconstructed input, the input gradient and the parameter-gradient angle."""
    import torch
    from paper_1707_04585_amd.torch_harness import StackRunner, download_grads
    peaks, ws = {}, {}
    for depth in (2, 72):
        cfg = dict(kind="basic", n=8, c=32, h=16, w=16, depth=depth, width=None, conv="f32", affine="random")
        x, params, dy = S.draw_stack(900 + depth, **cfg)
        r = StackRunner(**cfg)
        r.set_params(params)
        X, DY = r.new_pair(x), r.new_pair(dy)
        torch.cuda.synchronize()
        torch.cuda.reset_peak_memory_stats()
        before = torch.cuda.memory_allocated()
        r.forward(X, X)
        r.backward(X, DY, X, DY)
        torch.cuda.synchronize()
        peaks[depth] = torch.cuda.max_memory_allocated() - before
        ws[depth] = (r.fwd_bytes, r.bwd_bytes, r.activation_bytes()["total"])
        if depth == 72:
            ref = oracle_reference(oracle, cfg, x, params, dy)
            out = dict(x_rec=r.to_host(X[0]), dx=r.to_host(DY[0]), grads=download_grads(r.grads))
            e_rec, e_dx = oracle.rel_l2(out["x_rec"], x), oracle.rel_l2(out["dx"], ref["dx"])
            ang = oracle.angle_deg(oracle.flatten_grads(out["grads"]), oracle.flatten_grads(ref["grads"]))
            c = cfg["c"] // 2
            sp32 = lambda t: (np.ascontiguousarray(t[:, :c], dtype=np.float32),
                              np.ascontiguousarray(t[:, c:], dtype=np.float32))
            p32 = S.cast_params(params, np.float32)
            y1, y2 = oracle.stack_fwd(*sp32(x), p32, eps=np.float32(1e-5))[:2]
            (x1r, x2r), (d1, d2), g32, _ = oracle.stack_reverse(y1, y2, *sp32(dy), p32, eps=np.float32(1e-5))
            o_rec = oracle.rel_l2(np.concatenate([x1r, x2r], 1), x)
            o_dx = oracle.rel_l2(np.concatenate([d1, d2], 1), ref["dx"])
            o_ang = oracle.angle_deg(oracle.flatten_grads(g32), oracle.flatten_grads(ref["grads"]))
            print("depth 72: x_rec %.2e  dx %.2e  gradient angle %.3f deg  (oracle float32 Algorithm 1: %.2e %.2e %.3f)" %
                  (e_rec, e_dx, ang, o_rec, o_dx, o_ang), flush=True)
            assert e_rec < 1.5 * o_rec and e_dx < 1.5 * o_dx and ang < 1.5 * o_ang
            record("deep_stack_72_blocks/f32", conv="f32", x_rec=e_rec, dx=e_dx, angle_deg=ang, oracle_f32_x_rec=o_rec,
                   oracle_f32_dx=o_dx, oracle_f32_angle_deg=o_ang)
    assert ws[2] == ws[72], ws
    assert peaks[2] == 0 and peaks[72] == 0, peaks


def expected_relu_flips(params, stored64, sigmas=4.0):
    """From the float64 oracle alone: how many of the stack's ReLU decisions a
    correct float32 evaluation can take differently, per image.

    A pre-activation u = scale * h + shift inherits the rounding of the
    convolution sum h behind it: K = c_in * k * k products accumulated in
    float32 leave a relative error of about eps * sqrt(K) of the result's scale
    (eps = 2^-24; random-walk growth of the rounding errors), so the float32
    value is u + d with d ~ N(0, sigma^2), sigma = eps * sqrt(K) * rms(u) per
    channel.  (The stream tensors that layer 0 reads carry the error of the
    previous function's last convolution, hence that layer's K.)  Such a value
    decides differently from u with probability Phi(-|u| / sigma); the sum over
    an image's elements is the expected number of differing decisions there.
    Returns (expected count per image, per-image flag: some |u| < sigmas * sigma)."""
    from scipy.special import ndtr
    eps = 2.0 ** -24
    n = stored64[0]["F"][0]["u"].shape[0]
    expected = np.zeros(n)
    flagged = np.zeros(n, dtype=bool)
    for k, st in enumerate(stored64):
        for fn in ("F", "G"):
            layers = params[k][fn]
            for l, s64 in enumerate(st[fn]):
                w = layers[l - 1]["w"] if l > 0 else layers[-1]["w"]   # the convolution that produced this layer's input
                K = w.shape[1] * w.shape[2] * w.shape[3]
                u = s64["u"]
                sigma = eps * np.sqrt(K) * np.sqrt((u ** 2).mean(axis=(0, 2, 3), keepdims=True))
                t = np.abs(u) / np.maximum(sigma, 1e-300)
                expected += ndtr(-t).sum(axis=(1, 2, 3))
                flagged |= (t < sigmas).any(axis=(1, 2, 3))
    return expected, flagged


def test_c2_full_size_with_drift_report(oracle, torch_cuda):
    """The 9-block stack at N=128, C=32, 32x32, fp32, every output against the
    float64 oracle, plus reconstruction error per depth (Section 3.2
    'Numerical error': it accumulates but stays small).

    Tolerance at this size.  The stack takes 9*4*N*c*H*W = 7.5e7 ReLU
    decisions u > 0.  Float32 sums put u a few 1e-7 (more after several blocks
    of reconstruction drift) away from the float64 value, so a handful of
    decisions differ whatever the kernel.  Each one changes its gradient
    element by O(1), and that error stays inside its own image:
      * an image either meets the 1e-4 bar, or it holds a pre-activation within
        4 sigma of zero in the float64 oracle (sigma: the rounding error of a
        float32 convolution sum, see expected_relu_flips);
      * the number of images above the bar is at most E + 4 sqrt(E) + 2, E the
        expected number of differing decisions computed from the oracle alone;
      * whole tensors: dx within 5e-3, parameter gradients within 1e-2, and the
        angle between the parameter-gradient vectors (the quantity of the
        paper's figure on stored versus reconstructed activations) < 0.2 deg.
    """
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import StackRunner
    cfg, x, params, dy = S.draw_named("c2_stack9")
    print("oracle reference for c2_stack9 ...", flush=True)
    x1, x2 = split(x)
    y1, y2, inputs, stored = oracle.stack_fwd(x1, x2, params, keep=True)
    dx1, dx2, grads = oracle.stack_bwd_stored(stored, params, *split(dy))
    ref = dict(y=np.concatenate([y1, y2], 1), dx=np.concatenate([dx1, dx2], 1), grads=grads, inputs=inputs)
    expected, flagged = expected_relu_flips(params, stored)
    del stored
    print("gpu run ...", flush=True)
    out = gpu_run(cfg, x, params, dy)
    err = error_table(oracle, out, ref, x)
    gerr = {k: v for k, v in err.items() if "." in k}
    worst = max(gerr, key=gerr.get)
    print("rel. errors: y %.2e  x_rec %.2e  dx %.2e  worst parameter gradient %s %.2e" %
          (err["y"], err["x_rec"], err["dx"], worst, gerr[worst]), flush=True)
    assert err["y"] < 1e-5 and err["x_rec"] < 1e-5
    assert err["dx"] < 5e-3 and gerr[worst] < 1e-2
    assert_structure("y", out["y"], ref["y"], 1e-5, smooth=True)
    assert_structure("x_rec", out["x_rec"], x, 1e-5, smooth=True)
    per_image = np.array([oracle.rel_l2(out["dx"][i], ref["dx"][i]) for i in range(cfg["n"])])
    above = per_image >= 1e-4
    E = float(expected.sum())
    print("images whose dx meets 1e-4: %d of %d; median per-image error %.2e; expected differing decisions %.1f; "
          "images with a pre-activation within 4 sigma of zero: %d" %
          (int((~above).sum()), cfg["n"], np.median(per_image), E, int(flagged.sum())), flush=True)
    assert not (above & ~flagged).any(), ("images above 1e-4 without a near-zero pre-activation", np.nonzero(above & ~flagged)[0])
    assert above.sum() <= E + 4.0 * np.sqrt(E) + 2.0, (int(above.sum()), E)
    ang = oracle.angle_deg(oracle.flatten_grads(out["grads"]), oracle.flatten_grads(ref["grads"]))
    print("angle between GPU and stored-activation parameter gradients: %.3e degrees" % ang, flush=True)
    assert ang < 0.2
    record("c2_stack9/full", conv="f32", y=err["y"], x_rec=err["x_rec"], dx=err["dx"], worst_param=gerr[worst],
           worst_param_name=worst, images_above_bar=int(above.sum()), expected_flips=E, flagged_images=int(flagged.sum()),
           median_per_image_dx=float(np.median(per_image)), angle_deg=ang)
    # drift per depth: peel the stack one block at a time with the block entry point
    r = StackRunner(**cfg)
    r.set_params(params)
    Y, DY = r.new_pair(ref["y"]), r.new_pair(dy)
    drift = []
    for k in range(cfg["depth"] - 1, -1, -1):
        rv.revnet_block_bwd_reconstruct(r.desc, Y[1], Y[2], DY[1], DY[2], r.params[k], Y[1], Y[2], DY[1], DY[2],
                                        r.grads[k], 0, r.ws)
        torch.cuda.synchronize()
        xin = np.concatenate(ref["inputs"][k], axis=1)
        drift.append(oracle.rel_l2(r.to_host(Y[0]), xin))
    print("reconstruction rel. error, top block first:", ["%.2e" % d for d in drift], flush=True)
    assert max(drift) < 1e-5


def test_large_bottleneck_properties(oracle, torch_cuda):
    """Bottleneck stack at the real channel counts and resolution (C=256,
    width 64, 56x56) with a batch too large for the oracle to finish quickly:
    properties that hold at any size.  (i) reconstruction returns the input;
    (ii) F and G start with a BN, so the gradient that arrives through them
    sums to zero over each channel."""
    cfg = dict(S.STACKS["c4_bneck12"], n=8, depth=2)
    x, params, dy = S.draw_stack(80, **cfg)
    out = gpu_run(cfg, x, params, dy)
    assert oracle.rel_l2(out["x_rec"], x) < TOL["bf16"]["recon"]
    through = (out["dx"] - dy.astype(np.float32)).sum(axis=(0, 2, 3))
    scale = np.abs(out["dx"]).sum(axis=(0, 2, 3))
    c = cfg["c"] // 2
    # x2-half: dx2 - dy2 came through F of the bottom block; sums to ~0 per channel
    assert np.abs(through[c:]).max() < 1e-4 * scale[c:].max()


def test_reduced_batch_real_shapes_bf16(oracle, torch_cuda):
    """Real channel counts and resolutions of the bf16 workloads at a batch the
    oracle finishes in seconds."""
    for name, n in (("c3_stage2", 8), ("c3_stage3", 16), ("c5_stage2", 2), ("c5_stage4", 8)):
        cfg = dict(S.STACKS[name], n=n, depth=1)
        print(f"case {name} n={n}", flush=True)
        x, params, dy = S.draw_stack(81, **cfg)
        ref = oracle_reference(oracle, cfg, x, params, dy)
        out = gpu_run(cfg, x, params, dy)
        _, r32 = bf16_grad_tol(oracle, cfg, x, params, dy, ref)
        check_against_oracle(oracle, out, ref, x, "bf16", case=f"reduced_batch/{name}_n{n}", ref32=r32)
        with oracle.conv_operands("exact"):
            exact = oracle_reference(oracle, dict(cfg, conv="f32"), x, params, dy)
        print("  for information, against unrounded float64: dx %.2e" % oracle.rel_l2(out["dx"], exact["dx"]), flush=True)
