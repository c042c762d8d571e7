"""How far two correct summation orders can be apart when convolution operands
are rounded to bf16: the oracle in float32 against the oracle in float64, both
with bf16 operands.  Uses the oracle only."""
import numpy as np

import synth_inputs as S


def bf16_grad_floor(oracle, cfg, x, params, dy, ref):
    c = x.shape[1] // 2
    sp32 = lambda t: (np.ascontiguousarray(t[:, :c], dtype=np.float32), np.ascontiguousarray(t[:, c:], dtype=np.float32))
    p32 = S.cast_params(params, np.float32)
    with oracle.conv_operands("bf16"):
        y1, y2, _, stored = oracle.stack_fwd(*sp32(x), p32, eps=np.float32(cfg.get("eps", 1e-5)), keep=True)
        dx1, dx2, _ = oracle.stack_bwd_stored(stored, p32, *sp32(dy), eps=np.float32(cfg.get("eps", 1e-5)))
    return oracle.rel_l2(np.concatenate([dx1, dx2], 1), ref["dx"])
