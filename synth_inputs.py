"""Seeded synthetic inputs for the reversible-block tests and benchmark.

This module holds no arithmetic of the method: it only draws random tensors of
the shapes the workloads need.  Both the CPU oracle's tests and the GPU path's
tests are fed from here so that they see identical inputs.

The paper trains on CIFAR-10/100 (32x32 images, batch 100) and ImageNet
(224x224 crops, 32-64 images per GPU); neither is needed to time or check the
block arithmetic, so i.i.d. normal tensors of the same shapes stand in.

Draw order for a stack (fixed, so a seed names one input set):
  x  [N, C, H, W]  ~ N(0,1)          (x1 = channels [0,C/2), x2 = [C/2,C))
  for each block, F then G, for each layer:
      w     [K, Cin, k, k] ~ N(0, 2/(Cin*k*k))     (He-normal, fan-in)
      gamma [Cin]  = 1            or ~ U(0.5, 1.5)  (affine="random")
      beta  [Cin]  = 0            or ~ N(0, 0.1^2)
  dy [N, C, H, W]  ~ N(0,1)
All values are float64; callers cast to the precision they test.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 170704585

# Residual-function shapes: list of (c_in, c_out, k) per layer.


def func_layers(kind: str, c_half: int, width: int | None = None):
    if kind == "basic":
        return [(c_half, c_half, 3), (c_half, c_half, 3)]
    if kind == "bottleneck":
        assert width is not None
        return [(c_half, width, 1), (width, width, 3), (width, c_half, 1)]
    raise ValueError(kind)


# The reversible stacks of the five workloads (stack-level shapes only).
STACKS = {
    # name: kind, N, C, H, W, depth, width, conv dtype, affine
    "c1_block":   dict(kind="basic", n=4, c=16, h=8, w=8, depth=1, width=None, conv="f32", affine="unit"),
    "c2_stack9":  dict(kind="basic", n=128, c=32, h=32, w=32, depth=9, width=None, conv="f32", affine="random"),
    "c3_stage1":  dict(kind="basic", n=128, c=32, h=32, w=32, depth=9, width=None, conv="bf16", affine="random"),
    "c3_stage2":  dict(kind="basic", n=128, c=64, h=16, w=16, depth=9, width=None, conv="bf16", affine="random"),
    "c3_stage3":  dict(kind="basic", n=128, c=112, h=8, w=8, depth=9, width=None, conv="bf16", affine="random"),
    "c4_bneck12": dict(kind="bottleneck", n=64, c=256, h=56, w=56, depth=12, width=64, conv="bf16", affine="random"),
    "c5_stage1":  dict(kind="bottleneck", n=32, c=256, h=56, w=56, depth=3, width=64, conv="bf16", affine="random"),
    "c5_stage2":  dict(kind="bottleneck", n=32, c=512, h=28, w=28, depth=4, width=128, conv="bf16", affine="random"),
    "c5_stage3":  dict(kind="bottleneck", n=32, c=1024, h=14, w=14, depth=6, width=256, conv="bf16", affine="random"),
    "c5_stage4":  dict(kind="bottleneck", n=32, c=2048, h=7, w=7, depth=3, width=512, conv="bf16", affine="random"),
    # Not one of the paper's workloads: one block whose 3x3 layer (512 -> 512 channels at 28x28) is wide enough
    # to be bound by the matrix unit rather than by HBM, for the utilisation figures of the kernel profiles.
    "wide_bneck1": dict(kind="bottleneck", n=32, c=2048, h=28, w=28, depth=1, width=512, conv="bf16", affine="random"),
}


def draw_func(rng, kind, c_half, width, affine):
    layers = []
    for (cin, cout, k) in func_layers(kind, c_half, width):
        w = rng.standard_normal((cout, cin, k, k)) * np.sqrt(2.0 / (cin * k * k))
        if affine == "unit":
            gamma = np.ones(cin)
            beta = np.zeros(cin)
        else:
            gamma = rng.uniform(0.5, 1.5, cin)
            beta = rng.standard_normal(cin) * 0.1
        layers.append(dict(w=w, gamma=gamma, beta=beta))
    return layers


def draw_stack(seed, kind, n, c, h, w, depth, width=None, affine="random", **_unused):
    """Return (x, params, dy): x, dy float64 [N,C,H,W]; params[d] = dict(F=, G=)."""
    assert c % 2 == 0
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, c, h, w))
    params = []
    for _ in range(depth):
        F = draw_func(rng, kind, c // 2, width, affine)
        G = draw_func(rng, kind, c // 2, width, affine)
        params.append(dict(F=F, G=G))
    dy = rng.standard_normal((n, c, h, w))
    return x, params, dy


def down_layers(kind: str, c_in: int, c_out: int):
    """Layers (c_in, c_out, k, stride) of the residual branch of a subsampling
    block; the bottleneck's inner width is c_out / 4."""
    if kind == "basic":
        return [(c_in, c_out, 3, 2), (c_out, c_out, 3, 1)]
    if kind == "bottleneck":
        w = c_out // 4
        return [(c_in, w, 1, 1), (w, w, 3, 2), (w, c_out, 1, 1)]
    raise ValueError(kind)


def draw_down(rng, kind, c_in, c_out, affine):
    layers = []
    for (ci, co, k, s) in down_layers(kind, c_in, c_out):
        w = rng.standard_normal((co, ci, k, k)) * np.sqrt(2.0 / (ci * k * k))
        if affine == "unit":
            gamma, beta = np.ones(ci), np.zeros(ci)
        else:
            gamma, beta = rng.uniform(0.5, 1.5, ci), rng.standard_normal(ci) * 0.1
        layers.append(dict(w=w, gamma=gamma, beta=beta, stride=s))
    ws = rng.standard_normal((c_out, c_in, 1, 1)) * np.sqrt(2.0 / c_in)
    return dict(R=layers, S=dict(w=ws))


# Multi-stage bodies: reversible stages joined by subsampling blocks.  The body
# starts at the stem's output (the stem and pooling layers are not part of it).
BODIES = {
    # name: kind, N, H, W of the first stage, per-stage channels C / depth / bottleneck width, conv dtype
    "c3_body": dict(kind="basic", n=128, h=32, w=32, channels=(32, 64, 112), depths=(9, 9, 9), widths=(None, None, None), conv="bf16"),
    "c5_body": dict(kind="bottleneck", n=32, h=56, w=56, channels=(256, 512, 1024, 2048), depths=(3, 4, 6, 3), widths=(64, 128, 256, 512), conv="bf16"),
}


def draw_body(seed, kind, n, h, w, channels, depths, widths, affine="random", **_unused):
    """Return (x, stages, downs, dy): x [N, channels[0], H, W]; stages[s] = list of
    block parameters; downs[s] joins stage s and s+1; dy has the shape of the
    last stage's output.  Draw order: x, then per stage its blocks followed by
    the subsampling block above it, then dy."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, channels[0], h, w))
    stages, downs = [], []
    for s, (c, depth, width) in enumerate(zip(channels, depths, widths)):
        blocks = []
        for _ in range(depth):
            F = draw_func(rng, kind, c // 2, width, affine)
            G = draw_func(rng, kind, c // 2, width, affine)
            blocks.append(dict(F=F, G=G))
        stages.append(blocks)
        if s + 1 < len(channels):
            downs.append(draw_down(rng, kind, c, channels[s + 1], affine))
    last = len(channels) - 1
    dy = rng.standard_normal((n, channels[last], h >> last, w >> last))
    return x, stages, downs, dy


# Whole networks up to the last stage's top: stem (image convolution, optional 3x3 stride-2 max-pooling)
# followed by a body.  The image is N x 3 x H x W; the stem's output is the body's input.
NETS = {
    # name: body, image size, stem kernel / stride / pooling
    "c3_net": dict(body="c3_body", img_h=32, img_w=32, stem_ks=3, stem_stride=1, stem_pool=False),
    "c5_net": dict(body="c5_body", img_h=224, img_w=224, stem_ks=7, stem_stride=2, stem_pool=True),
}


def draw_net(seed, body, img_h, img_w, stem_ks, stem_stride, stem_pool, n=None, **body_override):
    """Return (img, stem, x_shape, stages, downs, dy): img [N, 3, H, W] ~ N(0,1); stem = dict(w=He-normal
    [C0, 3, k, k], stride=, pool=); the body's parameters and dy as draw_body draws them (its own x is not used)."""
    cfg = dict(BODIES[body])
    cfg.update(body_override)
    if n is not None:
        cfg["n"] = n
    rng = np.random.default_rng(seed)
    img = rng.standard_normal((cfg["n"], 3, img_h, img_w))
    c0 = cfg["channels"][0]
    w = rng.standard_normal((c0, 3, stem_ks, stem_ks)) * np.sqrt(2.0 / (3 * stem_ks * stem_ks))
    ho, wo = (img_h - 1) // stem_stride + 1, (img_w - 1) // stem_stride + 1
    if stem_pool:
        ho, wo = (ho - 1) // 2 + 1, (wo - 1) // 2 + 1
    assert (ho, wo) == (cfg["h"], cfg["w"]), "the stem's output must have the body's input size"
    _, stages, downs, dy = draw_body(seed + 1, **cfg)
    return cfg, img, dict(w=w, stride=stem_stride, pool=stem_pool), stages, downs, dy


def draw_named(name, seed_offset=0, **override):
    cfg = dict(STACKS[name])
    cfg.update(override)
    seed = BASE_SEED + list(STACKS).index(name) + 1000 * seed_offset
    x, params, dy = draw_stack(seed, **cfg)
    return cfg, x, params, dy


def cast_params(params, dtype):
    return [
        {fn: [{k: np.ascontiguousarray(v, dtype=dtype) for k, v in L.items()} for L in P[fn]]
         for fn in ("F", "G")}
        for P in params
    ]
