"""Kernels pick a faster addressing / loading path when every plane of their
tensors is 16-byte aligned (and small enough for 32-bit offsets); tensors that
start one float off an aligned address take the general path of every kernel
(scalar loads, per-element bounds, unaligned 16-byte accesses).  The two paths
sum in different orders (four-wide against scalar partial sums in the BN
reductions), so they agree to rounding, not bit for bit: forward values and
reconstruction are held to each other at the parity bars, gradients at those
bars for the typical image, with the few ReLU decisions that rounding can flip
bounded in number and size."""
import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu

CASES = [
    ("basic fp32 16 channels", dict(kind="basic", n=8, c=32, h=32, w=32, depth=2, width=None, conv="f32", affine="random")),
    ("basic fp32 ragged channels", dict(kind="basic", n=4, c=24, h=16, w=16, depth=1, width=None, conv="f32", affine="random")),
    ("bottleneck fp32", dict(kind="bottleneck", n=4, c=64, h=16, w=16, depth=1, width=16, conv="f32", affine="random")),
    ("bottleneck bf16", dict(kind="bottleneck", n=4, c=128, h=28, w=28, depth=1, width=32, conv="bf16", affine="random")),
    ("basic bf16", dict(kind="basic", n=8, c=64, h=16, w=16, depth=1, width=None, conv="bf16", affine="random")),
]


def run(cfg, x, params, dy, shift):
    """Forward and reconstructing backward with every stream tensor `shift` floats past a 256-byte aligned address."""
    import torch
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import StackRunner, download_grads
    r = StackRunner(**cfg)
    r.set_params(params)
    n, c, h, w = cfg["n"], cfg["c"], cfg["h"], cfg["w"]
    ch = c // 2

    def tensor(src):
        flat = torch.empty(n * c * h * w + 64, dtype=torch.float32, device=r.device)
        t = flat[shift:shift + n * c * h * w].view(n, c, h, w)
        t.copy_(torch.as_tensor(np.ascontiguousarray(src, dtype=np.float32)).to(r.device))
        assert t.data_ptr() % 16 == (4 * shift) % 16
        return t

    X, DY = tensor(x), tensor(dy)
    halves = lambda t: (t[:, :ch], t[:, ch:])
    (x1, x2), (d1, d2) = halves(X), halves(DY)
    rv.revnet_stack_fwd(r.desc, cfg["depth"], x1, x2, r.params, x1, x2, r.ws)
    torch.cuda.synchronize()
    y = X.cpu().numpy().copy()
    rv.revnet_stack_bwd(r.desc, cfg["depth"], x1, x2, d1, d2, r.params, x1, x2, d1, d2, r.grads, 0, r.ws)
    torch.cuda.synchronize()
    return y, X.cpu().numpy(), DY.cpu().numpy(), download_grads(r.grads)


def rel(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


@pytest.mark.parametrize("label,cfg", CASES, ids=[c[0] for c in CASES])
def test_aligned_and_unaligned_tensors_agree(label, cfg):
    x, params, dy = S.draw_stack(S.BASE_SEED + 5151, **cfg)
    y_a, x_a, dx_a, g_a = run(cfg, x, params, dy, shift=0)
    y_b, x_b, dx_b, g_b = run(cfg, x, params, dy, shift=1)
    fwd, grad = (1e-5, 1e-4) if cfg["conv"] == "f32" else (1e-2, 2e-2)
    errs = dict(y=rel(y_a, y_b), x_rec=rel(x_a, x_b), dx=rel(dx_a, dx_b))
    worst = 0.0
    for ba, bb in zip(g_a, g_b):
        for fn in ("F", "G"):
            for la, lb in zip(ba[fn], bb[fn]):
                for key in ("w", "gamma", "beta"):
                    worst = max(worst, rel(la[key], lb[key]))
    print(label, {k: "%.1e" % v for k, v in errs.items()}, "worst parameter gradient %.1e" % worst, flush=True)
    assert errs["y"] < fwd and errs["x_rec"] < fwd
    # Gradients pass through ReLU derivatives: a pre-activation within rounding of zero can be taken the other
    # way by the other summation order, an O(1) change of single elements (and of the per-channel sums they
    # enter).  So: the typical image must meet the bar, such elements must be rare, nothing may be far off.
    a, b = dx_a.astype(np.float64), dx_b.astype(np.float64)
    per_image = np.sqrt(((a - b) ** 2).sum(axis=(1, 2, 3)) / np.maximum((b ** 2).sum(axis=(1, 2, 3)), 1e-30))
    rms = np.sqrt((b ** 2).mean())
    outliers = float((np.abs(a - b) > 0.25 * rms).mean())
    print("   dx: median image %.1e  worst image %.1e  elements off by more than rms/4: %.1e" %
          (np.median(per_image), per_image.max(), outliers), flush=True)
    assert np.median(per_image) < grad and outliers < 1e-4
    assert errs["dx"] < 50 * grad and worst < 50 * grad
