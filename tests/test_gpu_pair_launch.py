"""The backward pass puts the data gradient and the filter gradient of a layer
into one launch.  The two kernel bodies are those of the separate launches, so
every output must be the same bits with the launches shared or (environment
variable RVN_SEPARATE_LAUNCHES=1) separate; the shared form must really be in
use (fewer launches, a `conv_dgrad_wgrad` family in the profile).

Shapes: one per pairing the library has -- bottleneck layers (1x1 and 3x3) with
rows of whole 4-pixel groups (28x28), without (14x14), with planes that are not
a multiple of 4 pixels (7x7); basic blocks whose 16-channel filter gradient
runs on the fp32 instruction; the fp32 pairing; a subsampling block."""
import os

import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu

CASES = [
    ("bneck 28x28", dict(kind="bottleneck", n=4, c=128, h=28, w=28, depth=2, width=32, conv="bf16", affine="random")),
    ("bneck 14x14", dict(kind="bottleneck", n=6, c=256, h=14, w=14, depth=1, width=64, conv="bf16", affine="random")),
    ("bneck 7x7", dict(kind="bottleneck", n=8, c=512, h=7, w=7, depth=1, width=128, conv="bf16", affine="random")),
    ("basic 16 channels", dict(kind="basic", n=8, c=32, h=32, w=32, depth=2, width=None, conv="bf16", affine="random")),
    ("basic 56 channels", dict(kind="basic", n=16, c=112, h=8, w=8, depth=1, width=None, conv="bf16", affine="random")),
    ("basic fp32", dict(kind="basic", n=8, c=32, h=32, w=32, depth=1, width=None, conv="f32", affine="random")),
]


def run_backward(cfg, x, params, dy):
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import StackRunner, download_grads
    r = StackRunner(**cfg)
    r.set_params(params)
    X, DY = r.new_pair(x), r.new_pair(dy)
    r.forward(X, X)
    rv.revnet_profile_begin()
    r.backward(X, DY, X, DY)
    torch.cuda.synchronize()
    stats = rv.revnet_profile_end()
    return r.to_host(X[0]), r.to_host(DY[0]), download_grads(r.grads), stats


def same_bits(a, b):
    return np.array_equal(np.asarray(a).view(np.uint32), np.asarray(b).view(np.uint32))


@pytest.fixture
def separate_launches():
    def switch(on):
        if on:
            os.environ["RVN_SEPARATE_LAUNCHES"] = "1"
        else:
            os.environ.pop("RVN_SEPARATE_LAUNCHES", None)
    yield switch
    os.environ.pop("RVN_SEPARATE_LAUNCHES", None)


@pytest.mark.parametrize("label,cfg", CASES, ids=[c[0] for c in CASES])
def test_shared_launch_gives_the_bits_of_separate_launches(label, cfg, separate_launches):
    x, params, dy = S.draw_stack(S.BASE_SEED + 4242, **cfg)
    separate_launches(False)
    x_a, dx_a, g_a, st_a = run_backward(cfg, x, params, dy)
    separate_launches(True)
    x_b, dx_b, g_b, st_b = run_backward(cfg, x, params, dy)
    separate_launches(False)
    layers = 2 * cfg["depth"] * (3 if cfg["kind"] == "bottleneck" else 2)
    n_a, n_b = (sum(s["launches"] for s in st.values()) for st in (st_a, st_b))
    print(label, "launches shared", n_a, "separate", n_b, flush=True)
    assert st_a.get("conv_dgrad_wgrad", {}).get("launches") == layers, st_a.keys()
    assert "conv_dgrad_wgrad" not in st_b and st_b["conv_dgrad"]["launches"] == layers
    assert n_b == n_a + layers
    assert same_bits(x_a, x_b) and same_bits(dx_a, dx_b)
    for ba, bb in zip(g_a, g_b):
        for fn in ("F", "G"):
            for la, lb in zip(ba[fn], bb[fn]):
                for key in ("w", "gamma", "beta"):
                    assert same_bits(la[key], lb[key]), (label, fn, key)


def test_subsampling_block_shared_launch(separate_launches):
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import upload_down, zeros_like_down, _dev
    rng = np.random.default_rng(S.BASE_SEED + 4243)
    n, ci, co, h = 4, 64, 128, 28
    x = rng.standard_normal((n, ci, h, h)).astype(np.float32)
    dy = rng.standard_normal((n, co, h // 2, h // 2)).astype(np.float32)
    P = S.draw_down(rng, "bottleneck", ci, co, "random")
    desc = rv.DownDesc("bottleneck", ci, co, 0, 1e-5, "bf16")
    fb, bb = rv.revnet_down_workspace_bytes(desc, n, h, h)
    out = []
    for sep in (False, True):
        separate_launches(sep)
        ws = torch.empty(max(fb, bb), dtype=torch.uint8, device="cuda:0")
        dp = upload_down(P)
        dg = zeros_like_down(dp)
        X, DY = _dev(x, "cuda:0"), _dev(dy, "cuda:0")
        DX = torch.empty_like(X)
        rv.revnet_profile_begin()
        rv.revnet_down_bwd(desc, X, DY, dp, DX, dg, 0, ws)
        torch.cuda.synchronize()
        st = rv.revnet_profile_end()
        flat = [DX.cpu().numpy()]

        def walk(t):
            if hasattr(t, "cpu"):
                flat.append(t.cpu().numpy())
            elif isinstance(t, dict):
                for k in sorted(t):
                    walk(t[k])
            elif isinstance(t, (list, tuple)):
                for v in t:
                    walk(v)
        walk(dg)
        out.append((flat, st))
    separate_launches(False)
    (fa, sa), (fb_, sb) = out
    assert sa.get("conv_dgrad_wgrad", {}).get("launches") == 4 and "conv_dgrad_wgrad" not in sb
    assert len(fa) == len(fb_) and len(fa) > 4
    for a, b in zip(fa, fb_):
        assert same_bits(a, b)
