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
