"""A toy training loop through the GPU path (analogue of the paper's check of
numerical error during training, Section 5.1 "Impact of numerical error" and
its figure of gradient angles): a small reversible stack is fitted to a fixed
random target with SGD + momentum 0.9, every gradient coming from the
reconstructing backward pass on the GPU.  At several points of the run the
gradient is compared with the oracle's stored-activation gradient (float64) at
the same parameters, and the loss curve with the one the oracle produces when
it trains the same stack itself in float64.  Synthetic data; the optimiser is
host arithmetic on the downloaded gradients."""
import copy

import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu

CFG = dict(kind="basic", n=16, c=16, h=8, w=8, depth=6, width=None, conv="f32", affine="random")
STEPS, LR, MOMENTUM = 30, 0.1, 0.9
CHECK_AT = (0, 10, 20, 29)


def sgd_step(params, grads, velocity):
    for B, G, V in zip(params, grads, velocity):
        for fn in ("F", "G"):
            for L, g, v in zip(B[fn], G[fn], V[fn]):
                for k in ("w", "gamma", "beta"):
                    v[k] = MOMENTUM * v[k] + np.asarray(g[k], dtype=np.float64)
                    L[k] = L[k] - LR * v[k]


def zeros_like(params):
    return [{fn: [{k: np.zeros_like(v) for k, v in L.items()} for L in B[fn]] for fn in ("F", "G")} for B in params]


def as_f32_values(params):
    """The parameters the GPU sees: float32 values, held in float64."""
    return [{fn: [{k: v.astype(np.float32).astype(np.float64) for k, v in L.items()} for L in B[fn]]
             for fn in ("F", "G")} for B in params]


def oracle_loss_and_grads(oracle, x, target, params):
    c = x.shape[1] // 2
    y1, y2, _, stored = oracle.stack_fwd(x[:, :c].copy(), x[:, c:].copy(), params, keep=True)
    y = np.concatenate([y1, y2], 1)
    d = (y - target) / y.size
    _, _, grads = oracle.stack_bwd_stored(stored, params, d[:, :c].copy(), d[:, c:].copy())
    return 0.5 * np.sum((y - target) ** 2) / y.size, grads


def test_toy_training_loop_gradient_angle_and_loss_curve(oracle):
    import torch
    from paper_1707_04585_amd.torch_harness import StackRunner, download_grads
    assert torch.cuda.is_available(), "this test needs the GPU"
    x, params0, _ = S.draw_stack(4242, **CFG)
    x = x.astype(np.float32).astype(np.float64)
    target = np.random.default_rng(4243).standard_normal(x.shape).astype(np.float32).astype(np.float64)

    # the oracle trains the stack itself, float64 throughout
    P, V, ref_losses = copy.deepcopy(params0), zeros_like(params0), []
    for _ in range(STEPS):
        loss, grads = oracle_loss_and_grads(oracle, x, target, P)
        ref_losses.append(loss)
        sgd_step(P, grads, V)

    # the same loop with the GPU's forward and reconstructing backward pass; a second runner keeps the
    # residual stream in fixed point (exact reconstruction) for comparison
    r = StackRunner(**CFG)
    # (24 fraction bits: codes of 6e-8, the spacing of fp32 near 1; the stream stays far inside +-128.
    # With 16 bits the 1.5e-5 steps move a handful of the run's 4e5 ReLU decisions per pass, each an O(1)
    # change of its gradient element, and the angle jumps to 0.1-0.3 degrees at the steps where that happens.)
    r_fixed = StackRunner(frac_bits=24, **CFG)
    P, V, losses, angles, angles_fixed = copy.deepcopy(params0), zeros_like(params0), [], {}, {}
    for step in range(STEPS):
        r.set_params(P)
        X = r.new_pair(x)
        r.forward(X, X)
        torch.cuda.synchronize()
        y = r.to_host(X[0])
        losses.append(0.5 * np.sum((y - target) ** 2) / y.size)
        d = (y - target) / y.size
        DY = r.new_pair(d)
        r.backward(X, DY, X, DY)
        torch.cuda.synchronize()
        grads = download_grads(r.grads)
        if step in CHECK_AT:
            _, g_ref = oracle_loss_and_grads(oracle, x, target, as_f32_values(P))
            flat_ref = oracle.flatten_grads(g_ref)
            angles[step] = oracle.angle_deg(oracle.flatten_grads(grads), flat_ref)
            assert oracle.rel_l2(oracle.flatten_grads(grads), flat_ref) < 1e-4
            r_fixed.set_params(P)
            XF = r_fixed.new_stream_pair(x)
            r_fixed.forward(XF, XF)
            DF = r_fixed.new_pair(d)
            r_fixed.backward(XF, DF, XF, DF)
            torch.cuda.synchronize()
            angles_fixed[step] = oracle.angle_deg(oracle.flatten_grads(download_grads(r_fixed.grads)), flat_ref)
        sgd_step(P, grads, V)

    print("loss, every third step: GPU    " + " ".join("%.4f" % l for l in losses[::3]), flush=True)
    print("                        oracle " + " ".join("%.4f" % l for l in ref_losses[::3]), flush=True)
    print("gradient angle to the stored-activation gradient (degrees): " +
          ", ".join("step %d: %.1e (fixed-point stream %.1e)" % (s, angles[s], angles_fixed[s]) for s in CHECK_AT),
          flush=True)
    assert losses[-1] < 0.4 * losses[0], "the loop does not train"
    assert max(angles.values()) < 1e-2 and max(angles_fixed.values()) < 1e-1
    worst = max(abs(a - b) / b for a, b in zip(losses, ref_losses))
    print("largest relative distance between the two loss curves: %.1e" % worst, flush=True)
    assert worst < 1e-3
