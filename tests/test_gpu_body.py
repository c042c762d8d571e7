"""GPU parity of the non-reversible subsampling block and of the multi-stage
body (reversible stages joined by such blocks), called through the C ABI,
against the CPU oracle on the same seeded inputs.

Tolerances as for the stacks: fp32 forward 1e-5, gradients 1e-4; bf16
convolution operands 2e-2 on gradients (1e-2 forward).  A tensor that misses
its bar passes only within 1.5x its own floor -- the distance between the
oracle's float32 and float64 runs for that tensor (see test_gpu_parity.py for
why bf16 operands make that the floor) -- and then the GPU must be as close to
the float32 oracle as well."""
import numpy as np
import pytest

import synth_inputs as S
from parity_checks import check_with_floors, record, assert_structure

pytestmark = pytest.mark.gpu

TOL = {"f32": dict(fwd=1e-5, grad=1e-4), "bf16": dict(fwd=1e-2, grad=2e-2)}


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def grad_err(oracle, got, want):
    floor = 1e-6 * max(1.0, float(np.abs(want).max()))
    if np.linalg.norm(want) < floor:
        return float(np.abs(got - want).max()) / (1e4 * floor)
    return oracle.rel_l2(got, want)


def down_errors(oracle, got, want, prefix=""):
    err = {prefix + "S.w": grad_err(oracle, got["S"]["w"], want["S"]["w"])}
    for l, (gl, wl) in enumerate(zip(got["R"], want["R"])):
        for key in ("w", "gamma", "beta"):
            err[f"{prefix}R.{l}.{key}"] = grad_err(oracle, gl[key], wl[key])
    return err


def cast_down(P, dt):
    return dict(R=[{k: (np.ascontiguousarray(v, dtype=dt) if k != "stride" else v) for k, v in L.items()} for L in P["R"]],
                S=dict(w=np.ascontiguousarray(P["S"]["w"], dtype=dt)))


DOWN_CASES = [
    # kind, n, c_in, c_out, h, w
    ("basic", 3, 12, 20, 12, 8),
    ("bottleneck", 2, 24, 32, 8, 12),
    ("basic", 8, 32, 64, 32, 32),        # the first subsampling block of the three-stage basic body
    ("bottleneck", 2, 64, 128, 28, 28),
    ("bottleneck", 4, 48, 40, 10, 6),     # ragged: half resolution 5x3, inner width 10
    # shapes the stride-2 3x3 kernel of the bf16 path takes (input channels a multiple of 8) with ragged geometry:
    # rows that are not whole 4-pixel groups, several bands per image with a short last one, odd half resolution
    ("basic", 3, 16, 24, 12, 10),
    ("bottleneck", 5, 64, 96, 20, 12),    # inner width 24
    ("basic", 2, 40, 72, 36, 44),         # several bands per image
    ("bottleneck", 3, 32, 64, 18, 14),    # inner width 16, half resolution 9x7
    # the other subsampling blocks of the two multi-stage workloads, at their real shapes
    ("basic", 8, 64, 112, 16, 16),
    ("bottleneck", 2, 256, 512, 56, 56),
    ("bottleneck", 2, 512, 1024, 28, 28),
    ("bottleneck", 4, 1024, 2048, 14, 14),
]


@pytest.mark.parametrize("conv", ["f32", "bf16"])
@pytest.mark.parametrize("kind,n,c_in,c_out,h,w", DOWN_CASES)
def test_down_block_matches_oracle(oracle, torch_cuda, kind, n, c_in, c_out, h, w, conv):
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import upload_down, zeros_like_down, download_down, _dev
    print(f"down block {kind} n={n} {c_in}->{c_out} {h}x{w} conv={conv}", flush=True)
    rng = np.random.default_rng(77)
    x = rng.standard_normal((n, c_in, h, w))
    P = S.draw_down(rng, kind, c_in, c_out, "random")
    dy = rng.standard_normal((n, c_out, h // 2, w // 2))
    with oracle.conv_operands(conv):
        y_ref, stored = oracle.down_fwd(x, P)
        dx_ref, g_ref = oracle.down_bwd(stored, P, dy)
    tol = dict(TOL[conv])
    floors = {}
    if conv == "bf16":   # the same block in float32: its distance from float64, per tensor
        with oracle.conv_operands("bf16"):
            P32 = cast_down(P, np.float32)
            _, st32 = oracle.down_fwd(x.astype(np.float32), P32, np.float32(1e-5))
            dx32, g32 = oracle.down_bwd(st32, P32, dy.astype(np.float32), np.float32(1e-5))
        floors = dict(down_errors(oracle, g32, g_ref), dx=oracle.rel_l2(dx32, dx_ref))

    desc = rv.DownDesc(kind, c_in, c_out, 0, 1e-5, conv)
    fwd_b, bwd_b = rv.revnet_down_workspace_bytes(desc, n, h, w)
    ws = torch.empty(max(fwd_b, bwd_b), dtype=torch.uint8, device="cuda:0")
    dp = upload_down(P)
    dg = zeros_like_down(dp)
    X, DY = _dev(x, "cuda:0"), _dev(dy, "cuda:0")
    Y = torch.empty((n, c_out, h // 2, w // 2), dtype=torch.float32, device="cuda:0")
    DX = torch.empty_like(X)
    rv.revnet_down_fwd(desc, X, dp, Y, ws)
    rv.revnet_down_bwd(desc, X, DY, dp, DX, dg, 0, ws)
    torch.cuda.synchronize()
    e_y = oracle.rel_l2(Y.cpu().numpy(), y_ref)
    e_dx = oracle.rel_l2(DX.cpu().numpy(), dx_ref)
    errs = down_errors(oracle, download_down(dg), g_ref)
    worst = max(errs, key=errs.get)
    print("  rel. errors: y %.2e  dx %.2e  worst parameter gradient %s %.2e" % (e_y, e_dx, worst, errs[worst]), flush=True)
    assert torch.equal(X.cpu(), torch.as_tensor(x.astype(np.float32))), "the stored input must not be modified"
    assert e_y < tol["fwd"]
    vs32 = dict(down_errors(oracle, download_down(dg), g32), dx=oracle.rel_l2(DX.cpu().numpy(), dx32)) if floors else {}
    used = check_with_floors(dict(errs, dx=e_dx), floors, vs32, tol["grad"])
    st_y = assert_structure("y", Y.cpu().numpy(), y_ref, tol["fwd"], smooth=True)
    st = assert_structure("dx", DX.cpu().numpy(), dx_ref, max(tol["grad"], 1.5 * floors.get("dx", 0.0)), smooth=False)
    record(f"down_block/{kind}_{c_in}to{c_out}_{h}x{w}_n{n}/{conv}", conv=conv, y=e_y, dx=e_dx, worst_param=errs[worst],
           worst_param_name=worst, bar=tol["grad"], dx_floor=floors.get("dx"), worst_param_floor=floors.get(worst),
           dx_vs_f32_oracle=vs32.get("dx"), worst_fraction_of_allowance=used, dx_per_image=st["per_image"],
           dx_per_channel=st["per_channel"], dx_border=st["border"], y_max_abs_over_rms=st_y["max_abs_over_rms"],
           dx_outliers=st["outliers"])

    # accumulate_wgrads adds to what is there: a second backward doubles every gradient (the kernels are
    # deterministic, so up to the rounding of the one addition)
    first = download_down(dg)
    rv.revnet_down_bwd(desc, X, DY, dp, DX, dg, 1, ws)
    torch.cuda.synchronize()
    doubled = dict(R=[{k: 2.0 * v for k, v in L.items()} for L in first["R"]], S=dict(w=2.0 * first["S"]["w"]))
    errs2 = down_errors(oracle, download_down(dg), doubled)
    assert max(errs2.values()) < 1e-6, errs2


def small_body_cfg(kind, conv):
    if kind == "basic":
        return dict(kind=kind, n=4, h=16, w=16, channels=(8, 12, 16), depths=(2, 1, 2), widths=(None, None, None), conv=conv)
    return dict(kind=kind, n=3, h=16, w=8, channels=(16, 32, 32), depths=(1, 2, 1), widths=(4, 8, 6), conv=conv)


def run_body(cfg, x, stages, downs, dy):
    import torch
    from paper_1707_04585_amd.torch_harness import BodyRunner, download_grads, download_down, _dev
    r = BodyRunner(**cfg)
    r.set_params(stages, downs)
    X = _dev(x, "cuda:0")
    r.forward(X)
    torch.cuda.synchronize()
    tops = [t.cpu().numpy().astype(np.float64) for t in r.tops]
    assert torch.equal(X.cpu(), torch.as_tensor(x.astype(np.float32))), "the body's input must not be modified"
    r.dtops[-1].copy_(_dev(dy, "cuda:0"))
    r.backward()
    torch.cuda.synchronize()
    return dict(runner=r, tops=tops, x_rec=r.tops[0].cpu().numpy().astype(np.float64),
                dx=r.dtops[0].cpu().numpy().astype(np.float64),
                stage_grads=[download_grads(g) for g in r.stage_grads],
                down_grads=[download_down(g) for g in r.down_grads])


def body_errors(oracle, out, tops_ref, dx_ref, sg_ref, dg_ref, x):
    err = {f"top{s}": oracle.rel_l2(t, tr) for s, (t, tr) in enumerate(zip(out["tops"], tops_ref))}
    fwd = max(err.values())
    g = {}
    for s, (gs, rs) in enumerate(zip(out["stage_grads"], sg_ref)):
        for k, (gb, rb) in enumerate(zip(gs, rs)):
            for fn in ("F", "G"):
                for l, (gl, rl) in enumerate(zip(gb[fn], rb[fn])):
                    for key in ("w", "gamma", "beta"):
                        g[f"s{s}.{k}.{fn}.{l}.{key}"] = grad_err(oracle, gl[key], rl[key])
    for s, (gd, rd) in enumerate(zip(out["down_grads"], dg_ref)):
        g.update(down_errors(oracle, gd, rd, prefix=f"down{s}."))
    return fwd, oracle.rel_l2(out["x_rec"], x), oracle.rel_l2(out["dx"], dx_ref), g


@pytest.mark.parametrize("conv", ["f32", "bf16"])
@pytest.mark.parametrize("kind", ["basic", "bottleneck"])
def test_body_matches_oracle(oracle, torch_cuda, kind, conv):
    """Three stages joined by two subsampling blocks: every stage top, the
    reconstructed input, the input gradient and every parameter gradient
    against ordinary stored-activation backprop in float64."""
    cfg = small_body_cfg(kind, conv)
    print(f"body {cfg}", flush=True)
    x, stages, downs, dy = S.draw_body(2025, **cfg)
    with oracle.conv_operands(conv):
        tops_ref, kept = oracle.body_fwd(x, stages, downs, keep=True)
        dx_ref, sg_ref, dg_ref = oracle.body_bwd_stored(kept, stages, downs, dy)
    tol = dict(TOL[conv])
    out = run_body(cfg, x, stages, downs, dy)
    fwd, rec, dx, g = body_errors(oracle, out, tops_ref, dx_ref, sg_ref, dg_ref, x)
    worst = max(g, key=g.get)
    print("  rel. errors: tops %.2e  x_rec %.2e  dx %.2e  worst parameter gradient %s %.2e" % (fwd, rec, dx, worst, g[worst]), flush=True)
    floors, vs32, f_fwd = body_floors(oracle, out, x, stages, downs, dy, tops_ref, dx_ref, sg_ref, dg_ref) if conv == "bf16" else ({}, {}, 0.0)
    assert fwd < max(tol["fwd"], 1.5 * f_fwd)
    assert rec < max(tol["fwd"], 1.5 * f_fwd)
    used = check_with_floors(dict(g, dx=dx), floors, vs32, tol["grad"])
    record(f"body_small/{kind}/{conv}", conv=conv, y=fwd, x_rec=rec, dx=dx, worst_param=g[worst], worst_param_name=worst,
           bar=tol["grad"], dx_floor=floors.get("dx"), worst_param_floor=floors.get(worst), dx_vs_f32_oracle=vs32.get("dx"),
           worst_fraction_of_allowance=used)


def body_floors(oracle, out, x, stages, downs, dy, tops_ref, dx_ref, sg_ref, dg_ref):
    """Per tensor: the distance of the oracle's memory-saving backward pass in
    float32 (Algorithm 1 inside the stages, bf16 operands) from the float64
    stored-activation reference, and of the GPU from that float32 run.  Also
    the float32 oracle's largest forward (stage top) distance."""
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    with oracle.conv_operands("bf16"):
        st32 = [S.cast_params(st, np.float32) for st in stages]
        dn32 = [cast_down(P, np.float32) for P in downs]
        t32 = oracle.body_fwd(f32(x), st32, dn32, np.float32(1e-5))
        dx32, sg32, dg32, _ = oracle.body_reverse(t32, st32, dn32, f32(dy), np.float32(1e-5))
    o32 = dict(tops=t32, x_rec=x, dx=dx32, stage_grads=sg32, down_grads=dg32)
    f_fwd, _, f_dx, f_g = body_errors(oracle, o32, tops_ref, dx_ref, sg_ref, dg_ref, x)
    _, _, v_dx, v_g = body_errors(oracle, out, t32, dx32, sg32, dg32, x)
    print("  floor (oracle float32 vs float64): tops %.2e, dx %.2e, worst gradient %.2e" % (f_fwd, f_dx, max(f_g.values())), flush=True)
    return dict(f_g, dx=f_dx), dict(v_g, dx=v_dx), f_fwd


def test_body_activation_memory_does_not_depend_on_depth(torch_cuda):
    """Section 3.2: only the stage tops (the stored inputs of the subsampling
    blocks) and a workspace are alive between forward and backward, whatever the
    stages' depths."""
    from paper_1707_04585_amd.torch_harness import BodyRunner
    base = dict(kind="basic", n=8, h=32, w=32, channels=(32, 64, 112), widths=(None, None, None), conv="bf16")
    a = BodyRunner(depths=(1, 1, 1), **base).activation_bytes()
    b = BodyRunner(depths=(9, 9, 9), **base).activation_bytes()
    assert a == b
    tops = 4 * 8 * (32 * 32 * 32 + 64 * 16 * 16 + 112 * 8 * 8)
    assert a["stream"] == tops


@pytest.mark.parametrize("conv", ["f32", "bf16"])
@pytest.mark.parametrize("name,n", [("c3_body", 4), ("c5_body", 2)])
def test_body_real_shapes_reduced_batch(oracle, torch_cuda, name, n, conv):
    """The two multi-stage workloads at their real channel counts and
    resolutions (32/64/112 channels from 32x32; 256..2048 channels from 56x56
    down to 7x7), one reversible block per stage and a batch the oracle
    finishes in seconds.

    Bars: the fp32 / bf16 ones; a tensor above its bar must be within 1.5x its
    own floor, the distance between the oracle's float32 run of the memory-saving
    backward pass and its float64 stored-activation run (and as close to the
    float32 run).  That distance is what the
    0/1 ReLU decisions leave: a pre-activation summed in float32 differs from
    the float64 one by ~1e-6 of its scale, so a few of the ~5e6 decisions of
    the larger body differ whatever the kernel, each an O(1) change of its
    gradient element (~1e-3 relative for a batch of two).  With bf16 operands
    every rounding step amplifies such differences and two oracle runs are
    already several per cent apart over a chain of seven blocks; there the 2e-2
    bar is held component by component (the subsampling blocks above and the
    stacks in test_gpu_parity.py, each fed the oracle's inputs)."""
    cfg = dict(S.BODIES[name], n=n, conv=conv)
    cfg["depths"] = tuple(1 for _ in cfg["depths"])
    print(f"body {name} n={n} depths={cfg['depths']} conv={conv}", flush=True)
    x, stages, downs, dy = S.draw_body(90, **cfg)
    tol = dict(TOL[conv])
    with oracle.conv_operands(conv):
        tops_ref, kept = oracle.body_fwd(x, stages, downs, keep=True)
        dx_ref, sg_ref, dg_ref = oracle.body_bwd_stored(kept, stages, downs, dy)
    del kept
    out = run_body(cfg, x, stages, downs, dy)
    fwd, rec, dx, g = body_errors(oracle, out, tops_ref, dx_ref, sg_ref, dg_ref, x)
    worst = max(g, key=g.get)
    print("  rel. errors: tops %.2e  x_rec %.2e  dx %.2e  worst parameter gradient %s %.2e" % (fwd, rec, dx, worst, g[worst]), flush=True)
    if conv == "bf16":
        floors, vs32, f_fwd = body_floors(oracle, out, x, stages, downs, dy, tops_ref, dx_ref, sg_ref, dg_ref)
    else:   # fp32 operands: the same construction with exact operands (a few ReLU decisions differ between float32 and float64)
        with oracle.conv_operands("exact"):
            f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
            st32 = [S.cast_params(st, np.float32) for st in stages]
            dn32 = [cast_down(P, np.float32) for P in downs]
            t32 = oracle.body_fwd(f32(x), st32, dn32, np.float32(1e-5))
            dx32, sg32, dg32, _ = oracle.body_reverse(t32, st32, dn32, f32(dy), np.float32(1e-5))
        o32 = dict(tops=t32, x_rec=x, dx=dx32, stage_grads=sg32, down_grads=dg32)
        f_fwd, _, f_dx, f_g = body_errors(oracle, o32, tops_ref, dx_ref, sg_ref, dg_ref, x)
        _, _, v_dx, v_g = body_errors(oracle, out, t32, dx32, sg32, dg32, x)
        floors, vs32 = dict(f_g, dx=f_dx), dict(v_g, dx=v_dx)
        print("  floor (oracle float32 vs float64): tops %.2e, dx %.2e, worst gradient %.2e" % (f_fwd, f_dx, max(f_g.values())), flush=True)
    assert fwd < max(tol["fwd"], 1.5 * f_fwd)
    assert rec < max(TOL[conv]["fwd"], 1.5 * f_fwd)
    used = check_with_floors(dict(g, dx=dx), floors, vs32, tol["grad"], pooled=conv == "f32")
    record(f"body_real_shapes/{name}_n{n}/{conv}", conv=conv, y=fwd, x_rec=rec, dx=dx, worst_param=g[worst], worst_param_name=worst,
           bar=tol["grad"], dx_floor=floors.get("dx"), worst_param_floor=floors.get(worst), dx_vs_f32_oracle=vs32.get("dx"),
           worst_fraction_of_allowance=used)


@pytest.mark.parametrize("name", ["c3_body", "c5_body"])
def test_body_full_size_properties(oracle, torch_cuda, name):
    """Full batch and depths, as the benchmark launches them; properties that
    hold at any size: (i) the backward pass returns the body's input in
    tops[0] (Section 3.2: every stage is reconstructed from its top) -- with
    bf16 operands the reconstruction error grows by a factor of a few per
    block (each rounding step amplifies a difference d to about sqrt(d * 2^-8)),
    to a few per cent over the nine blocks of a stage, which is what the
    single-stage drift reports show as well; (ii) two runs agree bit for bit."""
    cfg = dict(S.BODIES[name])
    x, stages, downs, dy = S.draw_body(91, **cfg)
    outs = [run_body(cfg, x, stages, downs, dy) for _ in range(2)]
    a, b = outs
    rec = oracle.rel_l2(a["x_rec"], x)
    print(f"{name}: reconstruction of the body input after {sum(cfg['depths'])} blocks: rel. error %.2e" % rec, flush=True)
    assert rec < 0.1
    assert np.isfinite(a["dx"]).all()
    assert np.array_equal(a["dx"], b["dx"]) and np.array_equal(a["x_rec"], b["x_rec"])
    for s in range(len(cfg["channels"])):
        assert np.array_equal(a["tops"][s], b["tops"][s])
    act = a["runner"].activation_bytes()
    print(f"{name}: activation bytes alive between forward and backward: {act}", flush=True)


def test_down_block_with_gapped_planes(oracle, torch_cuda):
    """Channel and image strides are free (sc >= h*w): every tensor of the call
    is a view with a gap after each plane, fp32 and bf16."""
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import upload_down, zeros_like_down, download_down, _dev
    kind, n, c_in, c_out, h, w = "bottleneck", 3, 24, 40, 12, 8
    rng = np.random.default_rng(78)
    x = rng.standard_normal((n, c_in, h, w))
    P = S.draw_down(rng, kind, c_in, c_out, "random")
    dy = rng.standard_normal((n, c_out, h // 2, w // 2))

    def gapped(shape, src=None):
        nn, cc, hh, ww = shape
        buf = torch.full((nn, cc, hh + 3, ww), float("nan"), dtype=torch.float32, device="cuda:0")
        view = buf[:, :, :hh, :]
        if src is not None:
            view.copy_(_dev(src, "cuda:0"))
        return buf, view

    for conv in ("f32", "bf16"):
        with oracle.conv_operands(conv):
            y_ref, stored = oracle.down_fwd(x, P)
            dx_ref, g_ref = oracle.down_bwd(stored, P, dy)
        desc = rv.DownDesc(kind, c_in, c_out, 0, 1e-5, conv)
        ws = torch.empty(max(rv.revnet_down_workspace_bytes(desc, n, h, w)), dtype=torch.uint8, device="cuda:0")
        dp = upload_down(P)
        dg = zeros_like_down(dp)
        (_, X), (_, DY) = gapped(x.shape, x), gapped(dy.shape, dy)
        (ybuf, Y), (dxbuf, DX) = gapped(dy.shape), gapped(x.shape)
        rv.revnet_down_fwd(desc, X, dp, Y, ws)
        rv.revnet_down_bwd(desc, X, DY, dp, DX, dg, 0, ws)
        torch.cuda.synchronize()
        assert torch.isnan(ybuf[:, :, h // 2:, :]).all() and torch.isnan(dxbuf[:, :, h:, :]).all(), "wrote into the gaps"
        tol = TOL[conv]
        assert oracle.rel_l2(Y.cpu().numpy(), y_ref) < tol["fwd"]
        assert oracle.rel_l2(DX.cpu().numpy(), dx_ref) < tol["grad"]
        assert max(down_errors(oracle, download_down(dg), g_ref).values()) < tol["grad"]
