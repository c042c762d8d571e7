"""CPU oracle for the reversible-residual-network hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product (the HIP library and its
Python binding) may import or call this module; only ``tests/``, the smoke
check and the benchmark's ``cpu_baseline`` leg do.  It shares no code with the
GPU path.

What it computes, and where the paper defines it:

* ``func_fwd``      -- a residual function built from the units of Section 2.2
                       (``a(x) = ReLU(BN(x))``, ``c_k(x) = Conv_kxk(a(x))``,
                       ``Basic = c3(c3(x))``, ``Bottleneck = c1(c3(c1(x)))``),
                       storing every intermediate.
* ``func_bwd``      -- ordinary backprop through it (Section 2.1, the backprop
                       rule), from the stored intermediates.
* ``block_fwd``     -- the reversible block, Section 3.1:
                       ``y1 = x1 + F(x2)``, ``y2 = x2 + G(y1)``.
* ``block_inverse`` -- its inverse, Section 3.1:
                       ``x2 = y2 - G(y1)``, ``x1 = y1 - F(x2)``.
* ``block_bwd_stored`` / ``stack_bwd_stored`` -- the gradient *definition*:
                       forward pass that keeps all activations, then the
                       backprop rule node by node.  This is what the method
                       must reproduce (Section 3.2: the algorithm combines the
                       reconstruction formulas with the backprop rule, so in
                       exact arithmetic its result is the ordinary gradient).
* ``block_reverse`` / ``stack_reverse`` -- Algorithm 1 (Section 3.2) as its data
                       flow (undo G and backprop it, then F), from ``(y, ybar)``
                       only; used to pin
                       Algorithm 1 == stored backprop and to report
                       reconstruction drift versus depth (Section 3.2
                       "Numerical error", Section 5.2 "Impact of numerical
                       error").

* ``fixed_encode`` / ``stack_fwd_fixed`` / ``stack_reverse_fixed`` -- the
                       variant of Section 3.2 "Numerical error": the x's and
                       y's in fixed point, F and G in floating point, so that
                       the reconstruction is exact.
* ``down_fwd`` / ``down_bwd`` -- the non-reversible subsampling block between
                       two stages (Section 3.1: a reversible block has stride
                       1, so the network also needs ordinary layers whose
                       inputs are stored; Section 3.2 end).  The paper does not
                       give its form; the reading taken here is stated at the
                       functions.
* ``stem_fwd`` / ``stem_bwd`` -- the network's first, non-reversible layers
                       (a convolution of the image, optionally followed by
                       3x3 stride-2 max-pooling), whose inputs are stored.
* ``body_fwd`` / ``body_bwd_stored`` / ``body_reverse`` -- stages of reversible
                       blocks joined by such blocks: ordinary backprop with
                       everything stored, and the memory-saving way (Algorithm
                       1 inside the stages, stored inputs at the subsampling
                       blocks only).

The layer operations (direct-loop convolution and its two adjoints, two-pass
batch norm and its unfused chain-rule backward) are plain C in
``layer_ops_impl.h``; the precision is that of the arrays passed in
(float64 for reference values, float32 to mimic the paper's setting).

Readings of points the paper leaves open:
BN uses batch statistics with the biased variance and ``eps`` added inside the
square root; ReLU'(0) = 0; every unit, including the first of F and G, is
BN -> ReLU -> conv; convolutions are zero padded by (k-1)/2 with no bias.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle_layer_ops.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C layer operations with gcc (host only)."""
    src = os.path.join(_HERE, "layer_ops.c")
    hdr = os.path.join(_HERE, "layer_ops_impl.h")
    stale = (not os.path.exists(_LIB_PATH)
             or os.path.getmtime(_LIB_PATH) < max(os.path.getmtime(src), os.path.getmtime(hdr)))
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", src,
                               "-o", _LIB_PATH, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB_PATH)
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


def _sfx(dtype) -> str:
    if dtype == np.float64:
        return "_f64"
    if dtype == np.float32:
        return "_f32"
    raise TypeError(f"oracle works in float64 or float32, got {dtype}")


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _real(dtype, v):
    return ctypes.c_double(v) if dtype == np.float64 else ctypes.c_float(v)


# ---------------------------------------------------------------------------
# layer operations (thin ctypes wrappers over the C definitions)
# ---------------------------------------------------------------------------

# Number of calls of each convolution routine since the last reset; lets a test
# check the paper's operation count (Section 3.2 "Computational overhead").
CONV_CALLS = {"fwd": 0, "dgrad": 0, "wgrad": 0}


def reset_conv_calls():
    for k in CONV_CALLS:
        CONV_CALLS[k] = 0


# Precision of the convolution OPERANDS.  The paper works in float32
# throughout (Section 3.2 "Numerical error"); the GPU library can also feed its
# matrix units bf16 operands with fp32 sums.  Rounding an operand moves some
# pre-activations across zero, and the ReLU derivative is a 0/1 decision, so a
# comparison with such a path is only meaningful if the oracle takes those
# decisions from equally rounded convolutions.  With "bf16" every convolution
# routine rounds both of its inputs to bfloat16 (nearest, ties to even) and
# otherwise computes as before, in the arrays' precision.
_OPERANDS = "exact"


class conv_operands:
    """Context manager: ``with conv_operands("bf16"): ...``"""

    def __init__(self, mode):
        assert mode in ("exact", "f32", "bf16")
        self.mode = "exact" if mode == "f32" else mode

    def __enter__(self):
        global _OPERANDS
        self.prev, _OPERANDS = _OPERANDS, self.mode

    def __exit__(self, *exc):
        global _OPERANDS
        _OPERANDS = self.prev


def bf16_round(a):
    """Round to the nearest bfloat16 (8 significant bits), ties to even, and
    return in the input's dtype.  Finite inputs only."""
    a = np.asarray(a)
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(a.dtype)


def _operand(a):
    return bf16_round(a) if _OPERANDS == "bf16" else a


def conv_fwd(a, w, stride=1):
    dt = a.dtype
    a, w = _c(_operand(a), dt), _c(_operand(w), dt)
    n, c, h, wd = a.shape
    k, c2, ks, ks2 = w.shape
    assert c2 == c and ks == ks2
    pad = (ks - 1) // 2
    ho = (h + 2 * pad - ks) // stride + 1
    wo = (wd + 2 * pad - ks) // stride + 1
    out = np.empty((n, k, ho, wo), dtype=dt)
    CONV_CALLS["fwd"] += 1
    getattr(_load(), "orc_conv_fwd" + _sfx(dt))(_p(a), _p(w), _p(out), n, c, k, h, wd, ks, stride)
    return out


def conv_dgrad(dout, w, in_hw, stride=1):
    dt = dout.dtype
    dout, w = _c(_operand(dout), dt), _c(_operand(w), dt)
    n, k = dout.shape[:2]
    k2, c, ks, _ = w.shape
    assert k2 == k
    h, wd = in_hw
    da = np.empty((n, c, h, wd), dtype=dt)
    CONV_CALLS["dgrad"] += 1
    getattr(_load(), "orc_conv_dgrad" + _sfx(dt))(_p(dout), _p(w), _p(da), n, c, k, h, wd, ks, stride)
    return da


def conv_wgrad(a, dout, ks, stride=1):
    dt = a.dtype
    a, dout = _c(_operand(a), dt), _c(_operand(dout), dt)
    n, c, h, wd = a.shape
    k = dout.shape[1]
    dw = np.empty((k, c, ks, ks), dtype=dt)
    CONV_CALLS["wgrad"] += 1
    getattr(_load(), "orc_conv_wgrad" + _sfx(dt))(_p(a), _p(dout), _p(dw), n, c, k, h, wd, ks, stride)
    return dw


def bn_relu_fwd(x, gamma, beta, eps):
    """a(x) = ReLU(BN(x)); returns a and everything stored backprop needs."""
    dt = x.dtype
    x, gamma, beta = _c(x, dt), _c(gamma, dt), _c(beta, dt)
    n, c, h, w = x.shape
    mean = np.empty(c, dt)
    var = np.empty(c, dt)
    xhat = np.empty_like(x)
    u = np.empty_like(x)
    a = np.empty_like(x)
    getattr(_load(), "orc_bn_relu_fwd" + _sfx(dt))(
        _p(x), _p(gamma), _p(beta), _real(dt, eps), _p(mean), _p(var), _p(xhat), _p(u), _p(a),
        n, c, h, w)
    return a, dict(x=x, mean=mean, var=var, xhat=xhat, u=u, a=a)


def bn_relu_bwd(da, st, gamma, eps):
    dt = da.dtype
    da, gamma = _c(da, dt), _c(gamma, dt)
    n, c, h, w = da.shape
    dx = np.empty_like(da)
    dgamma = np.empty(c, dt)
    dbeta = np.empty(c, dt)
    getattr(_load(), "orc_bn_relu_bwd" + _sfx(dt))(
        _p(da), _p(st["x"]), _p(gamma), _real(dt, eps), _p(st["mean"]), _p(st["var"]),
        _p(st["xhat"]), _p(st["u"]), _p(dx), _p(dgamma), _p(dbeta), n, c, h, w)
    return dx, dgamma, dbeta


# ---------------------------------------------------------------------------
# residual functions F, G (Section 2.2).  `layers` is a list of dicts with
# keys w [K,C,k,k], gamma [C], beta [C]; Basic has two 3x3 layers, Bottleneck
# 1x1 / 3x3 / 1x1.  Optional key "stride" (default 1) exists only for the
# non-reversible subsampling layers.
# ---------------------------------------------------------------------------

def func_fwd(x, layers, eps=1e-5):
    """Apply c_k units in sequence; return output and per-layer stored state."""
    stored = []
    h = x
    for L in layers:
        a, st = bn_relu_fwd(h, L["gamma"], L["beta"], eps)
        st["in_hw"] = h.shape[2:]
        h = conv_fwd(a, L["w"], L.get("stride", 1))
        stored.append(st)
    return h, stored


def func_bwd(stored, layers, dout, eps=1e-5):
    """Ordinary backprop through a residual function from stored activations.

    Returns (dx, grads) with grads[l] = dict(w=, gamma=, beta=)."""
    grads = [None] * len(layers)
    d = dout
    for l in range(len(layers) - 1, -1, -1):
        L, st = layers[l], stored[l]
        ks = L["w"].shape[2]
        s = L.get("stride", 1)
        dw = conv_wgrad(st["a"], d, ks, s)
        da = conv_dgrad(d, L["w"], st["in_hw"], s)
        d, dg, db = bn_relu_bwd(da, st, L["gamma"], eps)
        grads[l] = dict(w=dw, gamma=dg, beta=db)
    return d, grads


# ---------------------------------------------------------------------------
# reversible block (Section 3.1) and stored-activation backprop (Section 2.1)
# ---------------------------------------------------------------------------

def block_fwd(x1, x2, P, eps=1e-5):
    """y1 = x1 + F(x2); y2 = x2 + G(y1).  P = dict(F=layers, G=layers)."""
    f, st_f = func_fwd(x2, P["F"], eps)
    y1 = x1 + f
    g, st_g = func_fwd(y1, P["G"], eps)
    y2 = x2 + g
    return y1, y2, dict(F=st_f, G=st_g)


def block_inverse(y1, y2, P, eps=1e-5):
    """x2 = y2 - G(y1); x1 = y1 - F(x2)."""
    g, _ = func_fwd(y1, P["G"], eps)
    x2 = y2 - g
    f, _ = func_fwd(x2, P["F"], eps)
    x1 = y1 - f
    return x1, x2


def block_bwd_stored(stored, P, dy1, dy2, eps=1e-5):
    """Backprop rule on the forward graph z1 = x1 + F(x2), y2 = x2 + G(z1),
    y1 = z1, with every activation taken from the stored forward pass.

    z1 has two children (y1 and, through G, y2); x2 has two (y2 directly and,
    through F, z1); x1 has one (z1)."""
    g_in, grads_g = func_bwd(stored["G"], P["G"], dy2, eps)
    dz1 = dy1 + g_in
    f_in, grads_f = func_bwd(stored["F"], P["F"], dz1, eps)
    dx2 = dy2 + f_in
    dx1 = dz1
    return dx1, dx2, dict(F=grads_f, G=grads_g)


def _undo_and_backprop(layers, at, minuend, upstream, eps):
    """One half of the reversible backward pass: evaluate a residual function
    once at `at`, undo its addition (`minuend` - value) and push `upstream`
    back through the activations of that same evaluation (Section 5.1: reusing
    them is what gives the 4N cost of Section 3.2)."""
    value, st = func_fwd(at, layers, eps)
    vjp, grads = func_bwd(st, layers, upstream, eps)
    return minuend - value, vjp, grads


def block_reverse(y1, y2, dy1, dy2, P, eps=1e-5):
    """Algorithm 1 (Section 3.2): from (y, ybar) alone return the inputs,
    their total derivatives and the parameter derivatives.

    Data flow: G is evaluated at y1, which both recovers x2 and carries ybar2
    back to y1's node; F is then evaluated at the recovered x2, which recovers
    x1 and carries the total derivative of y1's node back to x2.  x1 feeds only
    that node, so it inherits its derivative; x2 also feeds y2 directly."""
    x2, into_y1, grads_g = _undo_and_backprop(P["G"], y1, y2, dy2, eps)
    d_node1 = dy1 + into_y1
    x1, into_x2, grads_f = _undo_and_backprop(P["F"], x2, y1, d_node1, eps)
    return (x1, x2), (d_node1, dy2 + into_x2), dict(F=grads_f, G=grads_g)


# ---------------------------------------------------------------------------
# stacks of reversible blocks (Section 3.2, "applying Algorithm 1 repeatedly")
# ---------------------------------------------------------------------------

def stack_fwd(x1, x2, params, eps=1e-5, keep=False):
    """Apply blocks params[0..D-1] in order.  With keep=True also return the
    list of every block's input pair and stored state (the memory-hungry
    ordinary way)."""
    inputs, stored = [], []
    for P in params:
        if keep:
            inputs.append((x1, x2))
        x1, x2, st = block_fwd(x1, x2, P, eps)
        if keep:
            stored.append(st)
    if keep:
        return x1, x2, inputs, stored
    return x1, x2


def stack_bwd_stored(stored, params, dy1, dy2, eps=1e-5):
    """Ordinary backprop through the stack from stored activations."""
    grads = [None] * len(params)
    for k in range(len(params) - 1, -1, -1):
        dy1, dy2, grads[k] = block_bwd_stored(stored[k], params[k], dy1, dy2, eps)
    return dy1, dy2, grads


def stack_reverse(y1, y2, dy1, dy2, params, eps=1e-5):
    """Backprop through the stack given only the top activations and their
    derivatives.  Also returns the reconstructed input pair of every block
    (index k = input of block k) for the drift-versus-depth report."""
    grads = [None] * len(params)
    recon = [None] * len(params)
    for k in range(len(params) - 1, -1, -1):
        (y1, y2), (dy1, dy2), grads[k] = block_reverse(y1, y2, dy1, dy2, params[k], eps)
        recon[k] = (y1, y2)
    return (y1, y2), (dy1, dy2), grads, recon


# ---------------------------------------------------------------------------
# fixed-point residual stream (Section 3.2, "Numerical error": fixed-point
# arithmetic on the x's and y's, ordinary floating point for F and G, gives
# exact reconstruction).  A stream value is an integer code q (int64 here)
# standing for q * 2^-frac_bits; `dtype` is the floating-point type F and G
# are computed in.  The paper does not say how a function value enters the
# stream; the reading here is rounding to the nearest code (ties to even).
# ---------------------------------------------------------------------------

def fixed_encode(x, frac_bits):
    return np.rint(np.asarray(x, dtype=np.float64) * 2.0 ** frac_bits).astype(np.int64)


def fixed_decode(q, frac_bits, dtype=np.float64):
    return q.astype(dtype) * dtype(2.0 ** -frac_bits)


def _to_codes(f, frac_bits):
    return np.rint(f * f.dtype.type(2.0 ** frac_bits)).astype(np.int64)


def block_fwd_fixed(q1, q2, P, frac_bits, eps=1e-5, dtype=np.float64):
    """y1 = x1 + F(x2), y2 = x2 + G(y1) with integer sums; returns the codes
    and the stored state of both functions."""
    f, st_f = func_fwd(fixed_decode(q2, frac_bits, dtype), P["F"], eps)
    y1 = q1 + _to_codes(f, frac_bits)
    g, st_g = func_fwd(fixed_decode(y1, frac_bits, dtype), P["G"], eps)
    y2 = q2 + _to_codes(g, frac_bits)
    return y1, y2, dict(F=st_f, G=st_g)


def block_reverse_fixed(y1, y2, dy1, dy2, P, frac_bits, eps=1e-5, dtype=np.float64):
    """block_reverse with the stream in fixed point: the functions read decoded
    values and the two additions are undone as integer differences."""
    def half(layers, at_codes, minuend_codes, upstream):
        value, st = func_fwd(fixed_decode(at_codes, frac_bits, dtype), layers, eps)
        vjp, grads = func_bwd(st, layers, upstream, eps)
        return minuend_codes - _to_codes(value, frac_bits), vjp, grads

    x2, into_y1, grads_g = half(P["G"], y1, y2, dy2)
    d_node1 = dy1 + into_y1
    x1, into_x2, grads_f = half(P["F"], x2, y1, d_node1)
    return (x1, x2), (d_node1, dy2 + into_x2), dict(F=grads_f, G=grads_g)


def stack_fwd_fixed(q1, q2, params, frac_bits, eps=1e-5, dtype=np.float64, keep=False):
    stored = []
    for P in params:
        q1, q2, st = block_fwd_fixed(q1, q2, P, frac_bits, eps, dtype)
        if keep:
            stored.append(st)
    return (q1, q2, stored) if keep else (q1, q2)


def stack_reverse_fixed(y1, y2, dy1, dy2, params, frac_bits, eps=1e-5, dtype=np.float64):
    grads = [None] * len(params)
    for k in range(len(params) - 1, -1, -1):
        (y1, y2), (dy1, dy2), grads[k] = block_reverse_fixed(y1, y2, dy1, dy2, params[k], frac_bits, eps, dtype)
    return (y1, y2), (dy1, dy2), grads


# ---------------------------------------------------------------------------
# non-reversible subsampling block and multi-stage body (Section 3.1: "the
# network must also contain non-reversible layers such as subsampling layers";
# Section 3.2: their inputs are stored explicitly).
#
# Reading (the paper leaves the form open): an ordinary pre-activation residual
# block on the concatenated tensor [N, C_in, H, W] -> [N, C_out, H/2, W/2],
#     a0 = ReLU(BN_0(x));  y = Conv_1x1,stride2(a0; Ws) + R(x),
# where R is the Basic / Bottleneck function of Section 2.2 with stride 2 on
# its (first) 3x3 convolution and C_out outputs; the projection shortcut reads
# the same pre-activation a0 as R's first convolution.  P = dict(R=layers with
# a "stride" key, S=dict(w=[C_out, C_in, 1, 1])).
# ---------------------------------------------------------------------------

def down_fwd(x, P, eps=1e-5):
    """Returns y and the stored state of every layer of R."""
    R = P["R"]
    stored = []
    h = x
    short = None
    for l, L in enumerate(R):
        a, st = bn_relu_fwd(h, L["gamma"], L["beta"], eps)
        st["in_hw"] = h.shape[2:]
        if l == 0:
            short = conv_fwd(a, P["S"]["w"], 2)
        h = conv_fwd(a, L["w"], L.get("stride", 1))
        stored.append(st)
    return short + h, stored


def down_bwd(stored, P, dy, eps=1e-5):
    """Ordinary backprop through the subsampling block from stored activations.
    Returns (dx, dict(R=[per-layer grads], S=dict(w=)))."""
    R = P["R"]
    grads = [None] * len(R)
    d = dy
    for l in range(len(R) - 1, -1, -1):
        L, st = R[l], stored[l]
        ks = L["w"].shape[2]
        s = L.get("stride", 1)
        dw = conv_wgrad(st["a"], d, ks, s)
        da = conv_dgrad(d, L["w"], st["in_hw"], s)
        if l == 0:  # a0 has a second child: the shortcut convolution
            dws = conv_wgrad(st["a"], dy, 1, 2)
            da = da + conv_dgrad(dy, P["S"]["w"], st["in_hw"], 2)
        d, dg, db = bn_relu_bwd(da, st, L["gamma"], eps)
        grads[l] = dict(w=dw, gamma=dg, beta=db)
    return d, dict(R=grads, S=dict(w=dws))


# ---------------------------------------------------------------------------
# stem: the first layers of the network, ahead of the reversible stages
# (Section 3.2: non-reversible layers, inputs stored).  Reading (the paper only
# cites the residual-network design it follows): a plain convolution of the
# image, k x k with stride s and padding (k-1)/2, no bias, optionally followed
# by max-pooling over 3x3 windows with stride 2 and padding 1 (positions
# outside the image never win).  S = dict(w=[C0, C_img, k, k], stride=s,
# pool=bool).  Where several elements of a window share the maximum, the first
# in row-major order takes the whole derivative.
# ---------------------------------------------------------------------------

def maxpool3s2_fwd(x):
    """Returns (y, arg): arg[n,c,p,q] = flat index (i*W + j) of the winning input element."""
    n, c, h, w = x.shape
    ho, wo = (h + 2 - 3) // 2 + 1, (w + 2 - 3) // 2 + 1
    y = np.full((n, c, ho, wo), -np.inf, dtype=x.dtype)
    arg = np.zeros((n, c, ho, wo), dtype=np.int64)
    for r in range(3):
        for s in range(3):
            for p in range(ho):
                i = 2 * p + r - 1
                if i < 0 or i >= h:
                    continue
                for q in range(wo):
                    j = 2 * q + s - 1
                    if j < 0 or j >= w:
                        continue
                    v = x[:, :, i, j]
                    better = v > y[:, :, p, q]          # strict: the first maximum in row-major order stays
                    y[:, :, p, q] = np.where(better, v, y[:, :, p, q])
                    arg[:, :, p, q] = np.where(better, i * w + j, arg[:, :, p, q])
    return y, arg


def maxpool3s2_bwd(dy, arg, in_hw):
    n, c, ho, wo = dy.shape
    h, w = in_hw
    dx = np.zeros((n, c, h * w), dtype=dy.dtype)
    flat_dy, flat_arg = dy.reshape(n, c, -1), arg.reshape(n, c, -1)
    for k in range(ho * wo):   # windows overlap: accumulate one window position at a time
        np.add.at(dx, (np.arange(n)[:, None], np.arange(c)[None, :], flat_arg[:, :, k]), flat_dy[:, :, k])
    return dx.reshape(n, c, h, w)


def stem_fwd(img, S):
    """Returns the body's input and what backprop needs (the stored inputs of both layers)."""
    h = conv_fwd(img, S["w"], S.get("stride", 1))
    if S.get("pool", False):
        y, arg = maxpool3s2_fwd(h)
        return y, dict(img=img, h_hw=h.shape[2:], arg=arg)
    return h, dict(img=img, h_hw=h.shape[2:], arg=None)


def stem_bwd(stored, S, dy):
    """Derivative with respect to the stem's filter (the image needs none)."""
    dh = maxpool3s2_bwd(dy, stored["arg"], stored["h_hw"]) if stored["arg"] is not None else dy
    return conv_wgrad(stored["img"], dh, S["w"].shape[2], S.get("stride", 1))


def _halves(t):
    c = t.shape[1] // 2
    return np.ascontiguousarray(t[:, :c]), np.ascontiguousarray(t[:, c:])


def body_fwd(x, stages, downs, eps=1e-5, keep=False):
    """stages[s] = list of block parameters; downs[s] joins stage s and s+1.
    Channels [0, C/2) of a stage's tensor are x1, the rest x2 (Section 3.1).
    Returns the top activation of every stage (the last is the output); with
    keep=True also everything ordinary backprop needs."""
    tops, kept = [], []
    for s, params in enumerate(stages):
        x1, x2 = _halves(x)
        if keep:
            y1, y2, _, st = stack_fwd(x1, x2, params, eps, keep=True)
        else:
            y1, y2 = stack_fwd(x1, x2, params, eps)
            st = None
        y = np.concatenate([y1, y2], axis=1)
        tops.append(y)
        st_down = None
        if s + 1 < len(stages):
            x, st_down = down_fwd(y, downs[s], eps)
        kept.append((st, st_down))
    return (tops, kept) if keep else tops


def body_bwd_stored(kept, stages, downs, dy, eps=1e-5):
    """Ordinary backprop with every activation stored.  Returns (dx,
    stage_grads[s][block], down_grads[s])."""
    sg, dg = [None] * len(stages), [None] * (len(stages) - 1)
    d = dy
    for s in range(len(stages) - 1, -1, -1):
        st, st_down = kept[s]
        if st_down is not None:
            d, dg[s] = down_bwd(st_down, downs[s], d, eps)
        d1, d2 = _halves(d)
        d1, d2, sg[s] = stack_bwd_stored(st, stages[s], d1, d2, eps)
        d = np.concatenate([d1, d2], axis=1)
    return d, sg, dg


def body_reverse(tops, stages, downs, dy, eps=1e-5):
    """The memory-saving backward pass: from the stored top activation of every
    stage only.  A subsampling block recomputes its internals from its stored
    input; a stage runs Algorithm 1.  Also returns each stage's reconstructed
    input."""
    sg, dg = [None] * len(stages), [None] * (len(stages) - 1)
    recon = [None] * len(stages)
    d = dy
    for s in range(len(stages) - 1, -1, -1):
        if s + 1 < len(stages):
            _, st_down = down_fwd(tops[s], downs[s], eps)
            d, dg[s] = down_bwd(st_down, downs[s], d, eps)
        y1, y2 = _halves(tops[s])
        d1, d2 = _halves(d)
        (x1, x2), (d1, d2), sg[s], _ = stack_reverse(y1, y2, d1, d2, stages[s], eps)
        recon[s] = np.concatenate([x1, x2], axis=1)
        d = np.concatenate([d1, d2], axis=1)
    return d, sg, dg, recon


def body_fwd_fixed(x, stages, downs, frac_bits, eps=1e-5, dtype=np.float64):
    """body_fwd with the stage tensors in fixed point: x is encoded, every stage
    runs on codes, a subsampling block reads the decoded top and its output is
    encoded for the next stage.  Returns the tops (codes) and what stored
    backprop needs."""
    tops, kept = [], []
    q = fixed_encode(x, frac_bits)
    for s, params in enumerate(stages):
        c = q.shape[1] // 2
        y1, y2, st = stack_fwd_fixed(q[:, :c], q[:, c:], params, frac_bits, eps, dtype, keep=True)
        top = np.concatenate([y1, y2], axis=1)
        tops.append(top)
        st_down = None
        if s + 1 < len(stages):
            y, st_down = down_fwd(fixed_decode(top, frac_bits, dtype), downs[s], eps)
            q = fixed_encode(y, frac_bits)
        kept.append((st, st_down))
    return tops, kept


def body_reverse_fixed(tops, stages, downs, dy, frac_bits, eps=1e-5, dtype=np.float64):
    """The memory-saving backward pass of the fixed-point body; also returns each
    stage's reconstructed input codes."""
    sg, dg = [None] * len(stages), [None] * (len(stages) - 1)
    recon = [None] * len(stages)
    d = dy
    for s in range(len(stages) - 1, -1, -1):
        if s + 1 < len(stages):
            _, st_down = down_fwd(fixed_decode(tops[s], frac_bits, dtype), downs[s], eps)
            d, dg[s] = down_bwd(st_down, downs[s], d, eps)
        c = tops[s].shape[1] // 2
        d1, d2 = _halves(d)
        (x1, x2), (d1, d2), sg[s] = stack_reverse_fixed(tops[s][:, :c], tops[s][:, c:], d1, d2, stages[s], frac_bits, eps, dtype)
        recon[s] = np.concatenate([x1, x2], axis=1)
        d = np.concatenate([d1, d2], axis=1)
    return d, sg, dg, recon


# ---------------------------------------------------------------------------
# error measures used by tests and reports
# ---------------------------------------------------------------------------

def rel_l2(got, ref) -> float:
    """Per-tensor relative error ||got - ref||_2 / max(||ref||_2, 1e-30), in float64."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm((got - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-30))


def angle_deg(g, h) -> float:
    """Angle in degrees between two gradients (the quantity of the paper's
    figure on stored versus reconstructed activations, Section 5.2)."""
    g = np.asarray(g, dtype=np.float64).ravel()
    h = np.asarray(h, dtype=np.float64).ravel()
    c = float(np.dot(g, h) / max(np.linalg.norm(g) * np.linalg.norm(h), 1e-300))
    return float(np.degrees(np.arccos(min(1.0, max(-1.0, c)))))


def flatten_grads(grads_per_block):
    """Concatenate all parameter gradients of a stack into one vector."""
    parts = []
    for gb in grads_per_block:
        for fn in ("F", "G"):
            for gl in gb[fn]:
                parts += [np.ravel(gl["w"]), np.ravel(gl["gamma"]), np.ravel(gl["beta"])]
    return np.concatenate(parts)
