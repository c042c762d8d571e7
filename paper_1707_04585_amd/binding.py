"""ctypes binding of ``include/revnet.h``: argument marshalling only.

Tensors may be any object with ``data_ptr()``, ``shape`` and ``stride()``
(torch CUDA tensors in practice: PyTorch is used for device memory and streams,
nothing else).  Parameter and gradient sets are passed as
``{"F": [layer, ...], "G": [layer, ...]}`` with ``layer = {"w": t, "gamma": t,
"beta": t}``.  Every function has the name and argument order of the C entry
point it calls and raises ``RevnetError`` on a negative status.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

F32, BF16 = 0, 1
BASIC, BOTTLENECK = 0, 1

EXPORTS = [
    "revnet_workspace_bytes", "revnet_block_fwd", "revnet_block_bwd_reconstruct", "revnet_stack_fwd",
    "revnet_stack_bwd", "revnet_stack_cost", "revnet_last_error", "revnet_version",
    "revnet_profile_begin", "revnet_profile_end",
    "revnet_down_workspace_bytes", "revnet_down_fwd", "revnet_down_bwd",
    "revnet_body_workspace_bytes", "revnet_body_fwd", "revnet_body_bwd",
    "revnet_fixed_workspace_bytes", "revnet_fixed_from_float", "revnet_fixed_to_float",
    "revnet_stack_fwd_fixed", "revnet_stack_bwd_fixed",
    "revnet_stem_workspace_bytes", "revnet_stem_fwd", "revnet_stem_bwd",
    "revnet_body_fixed_workspace_bytes", "revnet_body_fwd_fixed", "revnet_body_bwd_fixed",
    "revnet_stack_fwd_static",
]
STATIC_WS_BYTES = 32 << 20   # RVN_STATIC_WS_BYTES

MAX_STAGES = 8


class RevnetError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"revnet status {status}: {message}")
        self.status = status


class rvn_tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p)] + [(k, C.c_int64) for k in ("n", "c", "h", "w", "sn", "sc", "sh", "sw")]


class rvn_block_desc(C.Structure):
    _fields_ = [("kind", C.c_int), ("c_half", C.c_int32), ("width", C.c_int32), ("bn_eps", C.c_float),
                ("conv_dtype", C.c_int)]


class rvn_func_ptrs(C.Structure):  # layout shared by rvn_func_params and rvn_func_grads
    _fields_ = [("conv_w", C.c_void_p * 3), ("bn_gamma", C.c_void_p * 3), ("bn_beta", C.c_void_p * 3)]


class rvn_block_ptrs(C.Structure):  # rvn_block_params / rvn_block_grads
    _fields_ = [("F", rvn_func_ptrs), ("G", rvn_func_ptrs)]


class rvn_down_desc(C.Structure):
    _fields_ = [("kind", C.c_int), ("c_in", C.c_int32), ("c_out", C.c_int32), ("width", C.c_int32),
                ("bn_eps", C.c_float), ("conv_dtype", C.c_int)]


class rvn_down_ptrs(C.Structure):  # rvn_down_params / rvn_down_grads
    _fields_ = [("R", rvn_func_ptrs), ("shortcut_w", C.c_void_p)]


class rvn_body_desc(C.Structure):
    _fields_ = [("stages", C.c_int32), ("stage", rvn_block_desc * MAX_STAGES), ("depth", C.c_int32 * MAX_STAGES),
                ("down", rvn_down_desc * MAX_STAGES)]


class rvn_stem_desc(C.Structure):
    _fields_ = [("c_in", C.c_int32), ("c_out", C.c_int32), ("ks", C.c_int32), ("stride", C.c_int32), ("pool", C.c_int32)]


class rvn_cost(C.Structure):
    _fields_ = [("kernel_launches", C.c_int64), ("conv_fwd_calls", C.c_int64), ("conv_dgrad_calls", C.c_int64),
                ("conv_wgrad_calls", C.c_int64), ("conv_flops", C.c_double), ("algorithmic_bytes", C.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class rvn_kernel_stat(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("algorithmic_bytes", C.c_double), ("flops", C.c_double)]


def lib_path() -> str:
    return os.path.join(_HERE, "librevnet_hip.so")


def load_library():
    """Load the HIP library; there is no fallback if it has not been built."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_1707_04585_amd.build` "
                               "(there is no CPU or PyTorch fallback)")
        lib = C.CDLL(path)
        lib.revnet_last_error.restype = C.c_char_p
        for name in EXPORTS:
            getattr(lib, name)  # fail early if an entry point is missing
        _LIB = lib
    return _LIB


class BlockDesc:
    def __init__(self, kind, c_half, width=0, bn_eps=1e-5, conv_dtype=F32):
        self.kind = {"basic": BASIC, "bottleneck": BOTTLENECK}.get(kind, kind)
        self.conv_dtype = {"f32": F32, "bf16": BF16}.get(conv_dtype, conv_dtype)
        self.c_half, self.width, self.bn_eps = int(c_half), int(width or 0), float(bn_eps)

    def c(self):
        return rvn_block_desc(self.kind, self.c_half, self.width, self.bn_eps, self.conv_dtype)

    def num_layers(self):
        return 2 if self.kind == BASIC else 3


class DownDesc:
    """Subsampling block c_in -> c_out channels; the bottleneck's inner width defaults to c_out / 4."""

    def __init__(self, kind, c_in, c_out, width=0, bn_eps=1e-5, conv_dtype=F32):
        self.kind = {"basic": BASIC, "bottleneck": BOTTLENECK}.get(kind, kind)
        self.conv_dtype = {"f32": F32, "bf16": BF16}.get(conv_dtype, conv_dtype)
        self.c_in, self.c_out, self.bn_eps = int(c_in), int(c_out), float(bn_eps)
        self.width = int(width or (c_out // 4 if self.kind == BOTTLENECK else 0))

    def c(self):
        return rvn_down_desc(self.kind, self.c_in, self.c_out, self.width, self.bn_eps, self.conv_dtype)


class BodyDesc:
    """Reversible stages (BlockDesc, depth) joined by subsampling blocks."""

    def __init__(self, stages, depths, downs):
        assert len(stages) == len(depths) == len(downs) + 1 <= MAX_STAGES
        self.stages, self.depths, self.downs = list(stages), [int(d) for d in depths], list(downs)

    def c(self):
        out = rvn_body_desc()
        out.stages = len(self.stages)
        for s, st in enumerate(self.stages):
            out.stage[s] = st.c()
            out.depth[s] = self.depths[s]
        for s, dn in enumerate(self.downs):
            out.down[s] = dn.c()
        return out


def _desc(d):
    return d.c() if isinstance(d, (BlockDesc, DownDesc, BodyDesc)) else d


def _tensor(t):
    if isinstance(t, rvn_tensor):
        return t
    n, c, h, w = (int(v) for v in t.shape)
    sn, sc, sh, sw = (int(v) for v in t.stride())
    return rvn_tensor(t.data_ptr(), n, c, h, w, sn, sc, sh, sw)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "is_contiguous") and not t.is_contiguous():
        raise ValueError("parameter tensors must be contiguous")
    return t.data_ptr()


def _pack(block) -> rvn_block_ptrs:
    out = rvn_block_ptrs()
    for name in ("F", "G"):
        f = getattr(out, name)
        for l, layer in enumerate(block[name]):
            f.conv_w[l] = _ptr(layer["w"])
            f.bn_gamma[l] = _ptr(layer["gamma"])
            f.bn_beta[l] = _ptr(layer["beta"])
    return out


def pack_params(blocks):
    """[{F: [...], G: [...]}, ...] -> C array of rvn_block_params (host memory)."""
    if isinstance(blocks, C.Array):
        return blocks
    arr = (rvn_block_ptrs * len(blocks))()
    for k, b in enumerate(blocks):
        arr[k] = _pack(b)
    return arr


pack_grads = pack_params


def _pack_down(P) -> rvn_down_ptrs:
    out = rvn_down_ptrs()
    for l, layer in enumerate(P["R"]):
        out.R.conv_w[l] = _ptr(layer["w"])
        out.R.bn_gamma[l] = _ptr(layer["gamma"])
        out.R.bn_beta[l] = _ptr(layer["beta"])
    out.shortcut_w = _ptr(P["S"]["w"])
    return out


def pack_down(downs):
    """[{R: [layer, ...], S: {w: t}}, ...] -> C array of rvn_down_params / rvn_down_grads."""
    if isinstance(downs, C.Array):
        return downs
    arr = (rvn_down_ptrs * max(len(downs), 1))()
    for k, P in enumerate(downs):
        arr[k] = _pack_down(P)
    return arr


def pack_stages(stages):
    """[[block, ...], ...] -> (C array of pointers to per-stage arrays, the arrays kept alive).
    A value this function returned earlier is passed through, so that a caller
    can pack once and call many times."""
    if isinstance(stages, tuple):
        return stages
    arrays = [pack_params(st) for st in stages]
    ptrs = (C.c_void_p * len(arrays))(*[C.cast(a, C.c_void_p).value for a in arrays])
    return ptrs, arrays


def _tensor_array(ts):
    arr = (rvn_tensor * len(ts))()
    for i, t in enumerate(ts):
        arr[i] = _tensor(t)
    return arr


def _stream(stream):
    if stream is None:
        return None
    return getattr(stream, "cuda_stream", stream)


def _ws(ws):
    if ws is None:
        return None, 0
    if isinstance(ws, tuple):
        return ws
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _check(rc):
    if rc != 0:
        raise RevnetError(rc, revnet_last_error())


def revnet_last_error() -> str:
    return load_library().revnet_last_error().decode()


def revnet_version() -> int:
    return int(load_library().revnet_version())


def revnet_workspace_bytes(desc, n, h, w):
    fwd, bwd = C.c_size_t(0), C.c_size_t(0)
    d = _desc(desc)
    _check(load_library().revnet_workspace_bytes(C.byref(d), C.c_int64(n), C.c_int64(h), C.c_int64(w),
                                                 C.byref(fwd), C.byref(bwd)))
    return int(fwd.value), int(bwd.value)


def revnet_block_fwd(desc, x1, x2, params, y1, y2, ws, stream=None):
    d = _desc(desc)
    p = pack_params([params] if isinstance(params, dict) else params)
    wp, wb = _ws(ws)
    t = [_tensor(v) for v in (x1, x2, y1, y2)]
    _check(load_library().revnet_block_fwd(C.byref(d), C.byref(t[0]), C.byref(t[1]), p, C.byref(t[2]),
                                           C.byref(t[3]), C.c_void_p(wp), C.c_size_t(wb),
                                           C.c_void_p(_stream(stream))))


def revnet_block_bwd_reconstruct(desc, y1, y2, dy1, dy2, params, x1, x2, dx1, dx2, grads,
                                 accumulate_wgrads, ws, stream=None):
    d = _desc(desc)
    p = pack_params([params] if isinstance(params, dict) else params)
    g = pack_grads([grads] if isinstance(grads, dict) else grads)
    wp, wb = _ws(ws)
    t = [_tensor(v) for v in (y1, y2, dy1, dy2, x1, x2, dx1, dx2)]
    _check(load_library().revnet_block_bwd_reconstruct(
        C.byref(d), C.byref(t[0]), C.byref(t[1]), C.byref(t[2]), C.byref(t[3]), p, C.byref(t[4]),
        C.byref(t[5]), C.byref(t[6]), C.byref(t[7]), g, C.c_int(int(accumulate_wgrads)), C.c_void_p(wp),
        C.c_size_t(wb), C.c_void_p(_stream(stream))))


def revnet_stack_fwd(desc, depth, x1, x2, params, y1, y2, ws, stream=None):
    d = _desc(desc)
    p = pack_params(params)
    wp, wb = _ws(ws)
    t = [_tensor(v) for v in (x1, x2, y1, y2)]
    _check(load_library().revnet_stack_fwd(C.byref(d), C.c_int32(depth), C.byref(t[0]), C.byref(t[1]), p,
                                           C.byref(t[2]), C.byref(t[3]), C.c_void_p(wp), C.c_size_t(wb),
                                           C.c_void_p(_stream(stream))))


def revnet_stack_fwd_static(desc, depth, x1, x2, params, y1, y2, stream=None):
    d = _desc(desc)
    p = pack_params(params)
    t = [_tensor(v) for v in (x1, x2, y1, y2)]
    _check(load_library().revnet_stack_fwd_static(C.byref(d), C.c_int32(depth), C.byref(t[0]), C.byref(t[1]), p,
                                                  C.byref(t[2]), C.byref(t[3]), C.c_void_p(_stream(stream))))


def revnet_stack_bwd(desc, depth, y1, y2, dy1, dy2, params, x1, x2, dx1, dx2, grads, accumulate_wgrads,
                     ws, stream=None):
    d = _desc(desc)
    p = pack_params(params)
    g = pack_grads(grads)
    wp, wb = _ws(ws)
    t = [_tensor(v) for v in (y1, y2, dy1, dy2, x1, x2, dx1, dx2)]
    _check(load_library().revnet_stack_bwd(
        C.byref(d), C.c_int32(depth), C.byref(t[0]), C.byref(t[1]), C.byref(t[2]), C.byref(t[3]), p,
        C.byref(t[4]), C.byref(t[5]), C.byref(t[6]), C.byref(t[7]), g, C.c_int(int(accumulate_wgrads)),
        C.c_void_p(wp), C.c_size_t(wb), C.c_void_p(_stream(stream))))


def revnet_stack_cost(desc, depth, n, h, w):
    d = _desc(desc)
    fwd, bwd = rvn_cost(), rvn_cost()
    _check(load_library().revnet_stack_cost(C.byref(d), C.c_int32(depth), C.c_int64(n), C.c_int64(h),
                                            C.c_int64(w), C.byref(fwd), C.byref(bwd)))
    return fwd.as_dict(), bwd.as_dict()


def revnet_down_workspace_bytes(desc, n, h, w):
    fwd, bwd = C.c_size_t(0), C.c_size_t(0)
    d = _desc(desc)
    _check(load_library().revnet_down_workspace_bytes(C.byref(d), C.c_int64(n), C.c_int64(h), C.c_int64(w),
                                                      C.byref(fwd), C.byref(bwd)))
    return int(fwd.value), int(bwd.value)


def revnet_down_fwd(desc, x, params, y, ws, stream=None):
    d = _desc(desc)
    p = pack_down([params])
    wp, wb = _ws(ws)
    tx, ty = _tensor(x), _tensor(y)
    _check(load_library().revnet_down_fwd(C.byref(d), C.byref(tx), p, C.byref(ty), C.c_void_p(wp), C.c_size_t(wb),
                                          C.c_void_p(_stream(stream))))


def revnet_down_bwd(desc, x, dy, params, dx, grads, accumulate_wgrads, ws, stream=None):
    d = _desc(desc)
    p, g = pack_down([params]), pack_down([grads])
    wp, wb = _ws(ws)
    tx, tdy, tdx = _tensor(x), _tensor(dy), _tensor(dx)
    _check(load_library().revnet_down_bwd(C.byref(d), C.byref(tx), C.byref(tdy), p, C.byref(tdx), g,
                                          C.c_int(int(accumulate_wgrads)), C.c_void_p(wp), C.c_size_t(wb),
                                          C.c_void_p(_stream(stream))))


def revnet_body_workspace_bytes(desc, n, h, w):
    fwd, bwd = C.c_size_t(0), C.c_size_t(0)
    d = _desc(desc)
    _check(load_library().revnet_body_workspace_bytes(C.byref(d), C.c_int64(n), C.c_int64(h), C.c_int64(w),
                                                      C.byref(fwd), C.byref(bwd)))
    return int(fwd.value), int(bwd.value)


def revnet_body_fwd(desc, x, stage_params, down_params, tops, ws, stream=None):
    d = _desc(desc)
    sp, keep = pack_stages(stage_params)
    dp = pack_down(down_params)
    wp, wb = _ws(ws)
    tx, tt = _tensor(x), _tensor_array(tops)
    _check(load_library().revnet_body_fwd(C.byref(d), C.byref(tx), sp, dp, tt, C.c_void_p(wp), C.c_size_t(wb),
                                          C.c_void_p(_stream(stream))))
    del keep


def revnet_body_bwd(desc, tops, dtops, stage_params, down_params, stage_grads, down_grads, accumulate_wgrads, ws,
                    stream=None):
    d = _desc(desc)
    sp, keep_p = pack_stages(stage_params)
    sg, keep_g = pack_stages(stage_grads)
    dp, dg = pack_down(down_params), pack_down(down_grads)
    wp, wb = _ws(ws)
    tt, td = _tensor_array(tops), _tensor_array(dtops)
    _check(load_library().revnet_body_bwd(C.byref(d), tt, td, sp, dp, sg, dg, C.c_int(int(accumulate_wgrads)),
                                          C.c_void_p(wp), C.c_size_t(wb), C.c_void_p(_stream(stream))))
    del keep_p, keep_g


def revnet_fixed_workspace_bytes(desc, n, h, w):
    fwd, bwd = C.c_size_t(0), C.c_size_t(0)
    d = _desc(desc)
    _check(load_library().revnet_fixed_workspace_bytes(C.byref(d), C.c_int64(n), C.c_int64(h), C.c_int64(w),
                                                       C.byref(fwd), C.byref(bwd)))
    return int(fwd.value), int(bwd.value)


def revnet_fixed_from_float(src, frac_bits, dst, stream=None):
    ts, td = _tensor(src), _tensor(dst)
    _check(load_library().revnet_fixed_from_float(C.byref(ts), C.c_int32(frac_bits), C.byref(td),
                                                  C.c_void_p(_stream(stream))))


def revnet_fixed_to_float(src, frac_bits, dst, stream=None):
    ts, td = _tensor(src), _tensor(dst)
    _check(load_library().revnet_fixed_to_float(C.byref(ts), C.c_int32(frac_bits), C.byref(td),
                                                C.c_void_p(_stream(stream))))


def revnet_stack_fwd_fixed(desc, depth, frac_bits, x1, x2, params, y1, y2, ws, stream=None):
    d = _desc(desc)
    p = pack_params(params)
    wp, wb = _ws(ws)
    t = [_tensor(v) for v in (x1, x2, y1, y2)]
    _check(load_library().revnet_stack_fwd_fixed(C.byref(d), C.c_int32(depth), C.c_int32(frac_bits), C.byref(t[0]),
                                                 C.byref(t[1]), p, C.byref(t[2]), C.byref(t[3]), C.c_void_p(wp),
                                                 C.c_size_t(wb), C.c_void_p(_stream(stream))))


def revnet_stack_bwd_fixed(desc, depth, frac_bits, y1, y2, dy1, dy2, params, x1, x2, dx1, dx2, grads,
                           accumulate_wgrads, ws, stream=None):
    d = _desc(desc)
    p = pack_params(params)
    g = pack_grads(grads)
    wp, wb = _ws(ws)
    t = [_tensor(v) for v in (y1, y2, dy1, dy2, x1, x2, dx1, dx2)]
    _check(load_library().revnet_stack_bwd_fixed(
        C.byref(d), C.c_int32(depth), C.c_int32(frac_bits), C.byref(t[0]), C.byref(t[1]), C.byref(t[2]),
        C.byref(t[3]), p, C.byref(t[4]), C.byref(t[5]), C.byref(t[6]), C.byref(t[7]), g,
        C.c_int(int(accumulate_wgrads)), C.c_void_p(wp), C.c_size_t(wb), C.c_void_p(_stream(stream))))


def revnet_body_fixed_workspace_bytes(desc, n, h, w):
    fwd, bwd = C.c_size_t(0), C.c_size_t(0)
    d = _desc(desc)
    _check(load_library().revnet_body_fixed_workspace_bytes(C.byref(d), C.c_int64(n), C.c_int64(h), C.c_int64(w),
                                                            C.byref(fwd), C.byref(bwd)))
    return int(fwd.value), int(bwd.value)


def revnet_body_fwd_fixed(desc, frac_bits, x, stage_params, down_params, tops, ws, stream=None):
    d = _desc(desc)
    sp, keep = pack_stages(stage_params)
    dp = pack_down(down_params)
    wp, wb = _ws(ws)
    tx, tt = _tensor(x), _tensor_array(tops)
    _check(load_library().revnet_body_fwd_fixed(C.byref(d), C.c_int32(frac_bits), C.byref(tx), sp, dp, tt, C.c_void_p(wp),
                                                C.c_size_t(wb), C.c_void_p(_stream(stream))))
    del keep


def revnet_body_bwd_fixed(desc, frac_bits, tops, dtops, stage_params, down_params, stage_grads, down_grads,
                          accumulate_wgrads, ws, stream=None):
    d = _desc(desc)
    sp, keep_p = pack_stages(stage_params)
    sg, keep_g = pack_stages(stage_grads)
    dp, dg = pack_down(down_params), pack_down(down_grads)
    wp, wb = _ws(ws)
    tt, td = _tensor_array(tops), _tensor_array(dtops)
    _check(load_library().revnet_body_bwd_fixed(C.byref(d), C.c_int32(frac_bits), tt, td, sp, dp, sg, dg,
                                                C.c_int(int(accumulate_wgrads)), C.c_void_p(wp), C.c_size_t(wb),
                                                C.c_void_p(_stream(stream))))
    del keep_p, keep_g


def _opt_tensor(t):
    return None if t is None else C.byref(_tensor(t))


def revnet_stem_workspace_bytes(desc, n, h, w):
    bwd = C.c_size_t(0)
    _check(load_library().revnet_stem_workspace_bytes(C.byref(desc), C.c_int64(n), C.c_int64(h), C.c_int64(w), C.byref(bwd)))
    return int(bwd.value)


def revnet_stem_fwd(desc, img, w, conv_out, y, stream=None):
    ti, ty = _tensor(img), _tensor(y)
    _check(load_library().revnet_stem_fwd(C.byref(desc), C.byref(ti), C.c_void_p(_ptr(w)), _opt_tensor(conv_out),
                                          C.byref(ty), C.c_void_p(_stream(stream))))


def revnet_stem_bwd(desc, img, conv_out, dy, d_w, accumulate_wgrads, ws, stream=None):
    ti, td = _tensor(img), _tensor(dy)
    wp, wb = _ws(ws)
    _check(load_library().revnet_stem_bwd(C.byref(desc), C.byref(ti), _opt_tensor(conv_out), C.byref(td),
                                          C.c_void_p(_ptr(d_w)), C.c_int(int(accumulate_wgrads)), C.c_void_p(wp),
                                          C.c_size_t(wb), C.c_void_p(_stream(stream))))


def revnet_profile_begin():
    _check(load_library().revnet_profile_begin())


def revnet_profile_end():
    """-> {kernel family: dict(launches, total_ms, algorithmic_bytes, flops)}"""
    stats = (rvn_kernel_stat * 32)()
    n = C.c_int32(0)
    rc = load_library().revnet_profile_end(stats, C.c_int32(32), C.byref(n))
    if rc != 0:
        raise RevnetError(rc, "event timing failed")
    return {stats[i].name.decode(): dict(launches=stats[i].launches, total_ms=stats[i].total_ms,
                                         algorithmic_bytes=stats[i].algorithmic_bytes, flops=stats[i].flops)
            for i in range(min(n.value, 32))}
