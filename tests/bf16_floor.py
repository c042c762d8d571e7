"""How far a correct float32 evaluation can be from the float64 reference when
convolution operands are rounded to bf16: the oracle's Algorithm 1 (Section
3.2) run in float32 against the oracle's stored-activation backprop in
float64, both with bf16 operands.  Rounding to bf16 turns summation-order
differences of 1e-7 into differences of a whole bf16 step for a fraction of the
values, some ReLU decisions then differ, and the reversible backward pass
recomputes the functions at reconstructed inputs that carry such differences
(Section 3.2, "Numerical error").  Uses the oracle only."""
import numpy as np

import synth_inputs as S


def oracle_float32(oracle, cfg, x, params, dy, y=None):
    """The oracle's reversible backward pass in float32 with bf16 operands:
    dict(y, dx, grads).  It starts from `y` if given (as float32), else from
    the float32 forward pass of x."""
    c = x.shape[1] // 2
    sp32 = lambda t: (np.ascontiguousarray(t[:, :c], dtype=np.float32), np.ascontiguousarray(t[:, c:], dtype=np.float32))
    p32 = S.cast_params(params, np.float32)
    eps = np.float32(cfg.get("eps", 1e-5))
    with oracle.conv_operands("bf16"):
        y1, y2 = sp32(y) if y is not None else oracle.stack_fwd(*sp32(x), p32, eps=eps)
        _, (dx1, dx2), grads, _ = oracle.stack_reverse(y1, y2, *sp32(dy), p32, eps=eps)
    return dict(y=np.concatenate([y1, y2], 1), dx=np.concatenate([dx1, dx2], 1), grads=grads)


def bf16_grad_floor(oracle, cfg, x, params, dy, ref, want32=False, y=None):
    r32 = oracle_float32(oracle, cfg, x, params, dy, y=y)
    floor = oracle.rel_l2(r32["dx"], ref["dx"])
    return (floor, r32) if want32 else floor
