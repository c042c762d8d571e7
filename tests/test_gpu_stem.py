"""GPU parity of the stem (image convolution, 3x3 stride-2 max-pooling) against
the CPU oracle: outputs 1e-5, filter derivative 1e-4 (fp32 throughout)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def run_stem(c_in, c_out, ks, stride, pool, img, w, dy, accumulate_twice=False):
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import _dev
    n, _, h, wd = img.shape
    desc = rv.rvn_stem_desc(c_in, c_out, ks, stride, 1 if pool else 0)
    ho, wo = (h - 1) // stride + 1, (wd - 1) // stride + 1
    I, W = _dev(img, "cuda:0"), _dev(w, "cuda:0")
    conv_out = torch.empty((n, c_out, ho, wo), dtype=torch.float32, device="cuda:0") if pool else None
    yshape = (n, c_out, (ho - 1) // 2 + 1, (wo - 1) // 2 + 1) if pool else (n, c_out, ho, wo)
    Y = torch.empty(yshape, dtype=torch.float32, device="cuda:0")
    rv.revnet_stem_fwd(desc, I, W, conv_out, Y)
    ws = torch.empty(max(rv.revnet_stem_workspace_bytes(desc, n, h, wd), 256), dtype=torch.uint8, device="cuda:0")
    DW = torch.zeros_like(W)
    DY = _dev(dy(yshape), "cuda:0")
    rv.revnet_stem_bwd(desc, I, conv_out, DY, DW, 0, ws)
    if accumulate_twice:
        rv.revnet_stem_bwd(desc, I, conv_out, DY, DW, 1, ws)
    torch.cuda.synchronize()
    assert torch.equal(I.cpu(), torch.as_tensor(img.astype(np.float32)))
    return Y.cpu().numpy().astype(np.float64), DW.cpu().numpy().astype(np.float64), DY.cpu().numpy().astype(np.float64)


STEM_CASES = [
    # c_in, c_out, ks, stride, pool, n, h, w
    (3, 32, 3, 1, False, 8, 32, 32),     # the 32x32 network's stem
    (3, 64, 7, 2, True, 2, 224, 224),    # large-image stem: 7x7 stride 2, then pooling to 56x56 (fewer channels: oracle time)
    (3, 256, 7, 2, True, 1, 64, 48),     # its real channel count on a smaller image
    (3, 20, 7, 2, True, 3, 37, 29),      # ragged: odd sizes, channel count not a multiple of the per-thread groups
    (4, 9, 5, 1, True, 2, 11, 6),
    (1, 5, 1, 2, False, 2, 7, 9),           # 1x1: the direct kernels
    (2, 70, 5, 2, True, 2, 21, 19),         # two channel groups, the second ragged
    (16, 48, 3, 2, False, 2, 12, 20),       # many input channels: 144 taps, three tap tiles per wavefront
    (3, 8, 3, 1, False, 48, 40, 100),       # filter gradient: several bands per workgroup, the last run shorter
    (3, 8, 7, 1, False, 1, 6, 1500),        # too wide for the matrix-core kernels' LDS band: the direct kernels
]


@pytest.mark.parametrize("c_in,c_out,ks,stride,pool,n,h,w", STEM_CASES)
def test_stem_matches_oracle(oracle, torch_cuda, c_in, c_out, ks, stride, pool, n, h, w):
    print(f"stem {c_in}->{c_out} {ks}x{ks} s{stride} pool={pool} n={n} {h}x{w}", flush=True)
    rng = np.random.default_rng(71)
    img = rng.standard_normal((n, c_in, h, w)).astype(np.float32).astype(np.float64)
    wt = (rng.standard_normal((c_out, c_in, ks, ks)) * np.sqrt(2.0 / (c_in * ks * ks))).astype(np.float32).astype(np.float64)
    y, dw, dy = run_stem(c_in, c_out, ks, stride, pool, img, wt, lambda shape: rng.standard_normal(shape))
    S_ = dict(w=wt, stride=stride, pool=pool)
    y_ref, stored = oracle.stem_fwd(img, S_)
    dw_ref = oracle.stem_bwd(stored, S_, dy)
    e_y, e_dw = oracle.rel_l2(y, y_ref), oracle.rel_l2(dw, dw_ref)
    print("  rel. errors: y %.2e  dw %.2e" % (e_y, e_dw), flush=True)
    assert y.shape == y_ref.shape
    assert e_y < 1e-5 and e_dw < 1e-4


def test_stem_full_size_one_image_against_oracle(oracle, torch_cuda):
    """The large-image stem at the size and launch shapes the benchmark times (32 images of 3x224x224,
    256 channels): the outputs of three images against the oracle run on those images alone, and the
    filter derivative with an upstream derivative that is zero outside those images (the derivative is
    a sum over images, so it then equals the oracle's on them alone)."""
    print("stem 3->256 7x7 s2 pool n=32 224x224, images 0, 13, 31 checked", flush=True)
    rng = np.random.default_rng(72)
    n, picks = 32, [0, 13, 31]
    img = rng.standard_normal((n, 3, 224, 224)).astype(np.float32).astype(np.float64)
    wt = (rng.standard_normal((256, 3, 7, 7)) * np.sqrt(2.0 / 147)).astype(np.float32).astype(np.float64)

    def dy(shape):
        d = np.zeros(shape)
        d[picks] = rng.standard_normal((len(picks),) + tuple(shape[1:]))
        return d

    y, dw, dy_used = run_stem(3, 256, 7, 2, True, img, wt, dy)
    S_ = dict(w=wt, stride=2, pool=True)
    y_ref, stored = oracle.stem_fwd(img[picks], S_)
    dw_ref = oracle.stem_bwd(stored, S_, dy_used[picks])
    e_y, e_dw = oracle.rel_l2(y[picks], y_ref), oracle.rel_l2(dw, dw_ref)
    print("  rel. errors: y %.2e  dw %.2e" % (e_y, e_dw), flush=True)
    assert e_y < 1e-5 and e_dw < 1e-4
    assert np.isfinite(y).all()


def test_stem_pooling_tie_rule_and_accumulate(oracle, torch_cuda):
    """Integer-valued images and filters make exact ties in the pooling windows
    (and exact arithmetic on both sides): the derivative must go to the same
    element as in the oracle, the first maximum in row-major order.  A second
    backward call with accumulate set doubles the filter derivative."""
    rng = np.random.default_rng(72)
    img = rng.integers(-1, 2, size=(2, 3, 12, 10)).astype(np.float64)
    wt = rng.integers(-1, 2, size=(6, 3, 3, 3)).astype(np.float64)
    y, dw, dy = run_stem(3, 6, 3, 1, True, img, wt, lambda shape: rng.integers(-3, 4, size=shape).astype(np.float64),
                         accumulate_twice=True)
    S_ = dict(w=wt, stride=1, pool=True)
    y_ref, stored = oracle.stem_fwd(img, S_)
    h = oracle.conv_fwd(img, wt, 1)
    ties = sum(int((h[:, :, max(2 * p - 1, 0):2 * p + 2, max(2 * q - 1, 0):2 * q + 2] == y_ref[:, :, p:p + 1, q:q + 1]).sum(axis=(2, 3)).max() > 1)
               for p in range(y_ref.shape[2]) for q in range(y_ref.shape[3]))
    assert ties > 0, "the case is meant to contain tied windows"
    assert np.array_equal(y, y_ref)
    assert np.array_equal(dw, 2.0 * oracle.stem_bwd(stored, S_, dy))


@pytest.mark.parametrize("name,n", [("c3_net", 4), ("c5_net", 1)])
def test_whole_network_matches_oracle_fp32(oracle, torch_cuda, name, n):
    """Stem, stages and subsampling blocks end to end at the real channel counts
    and image sizes, one reversible block per stage, fp32 operands, small
    batch: last stage's top and every parameter derivative (stem filter
    included) against ordinary stored-activation backprop in float64.  The bar
    allows for the few 0/1 ReLU decisions that fp32 sums take differently (see
    test_body_real_shapes_reduced_batch): a tensor above 1e-4 must be within
    1.5x the largest float32-to-float64 oracle distance of the case."""
    import torch
    import synth_inputs as S
    from paper_1707_04585_amd.torch_harness import NetRunner, download_grads, download_down, _dev
    from test_gpu_body import body_errors, cast_down
    net = dict(S.NETS[name])
    depths = tuple(1 for _ in S.BODIES[net["body"]]["depths"])
    cfg, img, stem, stages, downs, dy = S.draw_net(95, n=n, depths=depths, conv="f32", **net)
    img = img.astype(np.float32).astype(np.float64)

    def oracle_run(dt):
        c = lambda a: np.ascontiguousarray(a, dtype=dt)
        st = [S.cast_params(s_, dt) for s_ in stages]
        dn = [cast_down(P, dt) for P in downs]
        sm = dict(stem, w=c(stem["w"]))
        x0, kept_stem = oracle.stem_fwd(c(img), sm)
        tops, kept = oracle.body_fwd(x0, st, dn, dt(1e-5), keep=True)
        dx0, sg, dg = oracle.body_bwd_stored(kept, st, dn, c(dy), dt(1e-5))
        return x0, tops, dx0, sg, dg, oracle.stem_bwd(kept_stem, sm, dx0)

    x0, tops_ref, dx_ref, sg_ref, dg_ref, dws_ref = oracle_run(np.float64)
    _, t32, dx32, sg32, dg32, dws32 = oracle_run(np.float32)
    o32 = dict(tops=t32, x_rec=x0, dx=dx32, stage_grads=sg32, down_grads=dg32)
    f_fwd, _, f_dx, f_g = body_errors(oracle, o32, tops_ref, dx_ref, sg_ref, dg_ref, x0)
    floors = dict(f_g, dx=f_dx, stem_w=oracle.rel_l2(dws32, dws_ref))
    print(f"{name}: largest floor (oracle float32 vs float64) {max(floors.values()):.2e}", flush=True)

    r = NetRunner(cfg, stem)
    r.set_params(stages, downs)
    r.forward(_dev(img, "cuda:0"))
    torch.cuda.synchronize()
    tops = [t.cpu().numpy().astype(np.float64) for t in r.body.tops]
    r.body.dtops[-1].copy_(_dev(dy, "cuda:0"))
    r.backward()
    torch.cuda.synchronize()
    out = dict(tops=tops, x_rec=r.body.tops[0].cpu().numpy().astype(np.float64),
               dx=r.body.dtops[0].cpu().numpy().astype(np.float64),
               stage_grads=[download_grads(g) for g in r.body.stage_grads],
               down_grads=[download_down(g) for g in r.body.down_grads])
    fwd, rec, dx, g = body_errors(oracle, out, tops_ref, dx_ref, sg_ref, dg_ref, x0)
    e_stem = oracle.rel_l2(r.stem_dw.cpu().numpy(), dws_ref)
    worst = max(g, key=g.get)
    print("  rel. errors: tops %.2e  stem output reconstructed %.2e  dx %.2e  stem filter gradient %.2e  worst other %s %.2e" %
          (fwd, rec, dx, e_stem, worst, g[worst]), flush=True)
    assert fwd < max(1e-5, 1.5 * f_fwd) and rec < 1e-5
    _, _, v_dx, v_g = body_errors(oracle, out, t32, dx32, sg32, dg32, x0)
    from parity_checks import check_with_floors, record
    vs32 = dict(v_g, dx=v_dx, stem_w=oracle.rel_l2(r.stem_dw.cpu().numpy(), dws32))
    used = check_with_floors(dict(g, dx=dx, stem_w=e_stem), floors, vs32, 1e-4, pooled=True)
    record(f"whole_network/{name}_n{n}/f32", conv="f32", y=fwd, x_rec=rec, dx=dx, worst_param=g[worst], worst_param_name=worst,
           bar=1e-4, dx_floor=f_dx, worst_param_floor=floors[worst], dx_vs_f32_oracle=v_dx, stem_w=e_stem,
           worst_fraction_of_allowance=used)


def test_stem_with_gapped_planes(oracle, torch_cuda):
    """All tensors of the stem calls as views with a gap after each plane."""
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import _dev
    rng = np.random.default_rng(73)
    n, h, w, c_out = 2, 18, 14, 12
    img = rng.standard_normal((n, 3, h, w))
    wt = rng.standard_normal((c_out, 3, 7, 7)) * 0.1
    S_ = dict(w=wt, stride=2, pool=True)
    y_ref, stored = oracle.stem_fwd(img, S_)
    dy = rng.standard_normal(y_ref.shape)
    dw_ref = oracle.stem_bwd(stored, S_, dy)

    def gapped(shape, src=None):
        nn, cc, hh, ww = shape
        buf = torch.full((nn, cc, hh + 2, ww), float("nan"), dtype=torch.float32, device="cuda:0")
        view = buf[:, :, :hh, :]
        if src is not None:
            view.copy_(_dev(src, "cuda:0"))
        return buf, view

    desc = rv.rvn_stem_desc(3, c_out, 7, 2, 1)
    (_, I), (_, DY) = gapped(img.shape, img), gapped(dy.shape, dy)
    (cbuf, CO), (ybuf, Y) = gapped((n, c_out, 9, 7)), gapped(dy.shape)
    W, DW = _dev(wt, "cuda:0"), torch.zeros((c_out, 3, 7, 7), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(rv.revnet_stem_workspace_bytes(desc, n, h, w), dtype=torch.uint8, device="cuda:0")
    rv.revnet_stem_fwd(desc, I, W, CO, Y)
    rv.revnet_stem_bwd(desc, I, CO, DY, DW, 0, ws)
    torch.cuda.synchronize()
    assert torch.isnan(cbuf[:, :, 9:, :]).all() and torch.isnan(ybuf[:, :, dy.shape[2]:, :]).all(), "wrote into the gaps"
    assert oracle.rel_l2(Y.cpu().numpy(), y_ref) < 1e-5
    assert oracle.rel_l2(DW.cpu().numpy(), dw_ref) < 1e-4
