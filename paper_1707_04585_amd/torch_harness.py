"""Device-memory plumbing for tests, the smoke check and the benchmark.

PyTorch is used here only to allocate device buffers, copy host arrays in and
out, and provide a stream; every arithmetic step runs in the HIP library.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _dev(a, device):
    return torch.as_tensor(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def upload_params(params, device="cuda:0"):
    """[{F: [{w,gamma,beta}], G: [...]}] of host arrays -> same structure of device tensors."""
    return [{fn: [{k: _dev(L[k], device) for k in ("w", "gamma", "beta")} for L in P[fn]]
             for fn in ("F", "G")} for P in params]


def zeros_like_params(dparams):
    return [{fn: [{k: torch.zeros_like(v) for k, v in L.items()} for L in P[fn]] for fn in ("F", "G")}
            for P in dparams]


def download_grads(dgrads):
    return [{fn: [{k: v.detach().cpu().numpy().astype(np.float64) for k, v in L.items()} for L in P[fn]]
             for fn in ("F", "G")} for P in dgrads]


class StackRunner:
    """Owns the device buffers of one reversible stack and calls the C ABI.

    x1/x2 (and every other pair) are the two channel halves of one
    [N, C, H, W] buffer, i.e. strided views, unless split_buffers=True."""

    def __init__(self, kind, n, c, h, w, depth, width=None, conv="f32", eps=1e-5, device="cuda:0",
                 split_buffers=False, frac_bits=0, **_unused):
        self.desc = B.BlockDesc(kind, c // 2, width or 0, eps, conv)
        self.n, self.c, self.h, self.w, self.depth = n, c, h, w, depth
        self.device = torch.device(device)
        self.split_buffers = split_buffers
        # frac_bits > 0: the residual stream is kept in fixed point (int32 codes of 2^-frac_bits)
        self.frac_bits = int(frac_bits)
        query = B.revnet_fixed_workspace_bytes if self.frac_bits else B.revnet_workspace_bytes
        self.fwd_bytes, self.bwd_bytes = query(self.desc, n, h, w)
        self.ws = torch.empty(max(self.fwd_bytes, self.bwd_bytes), dtype=torch.uint8, device=self.device)
        self.params = self.grads = self._pp = self._pg = None

    # -- buffers ------------------------------------------------------------
    def new_pair(self, src=None):
        """Return (full, half1, half2)."""
        ch = self.c // 2
        if self.split_buffers:
            a = torch.empty((self.n, ch, self.h, self.w), dtype=torch.float32, device=self.device)
            b = torch.empty_like(a)
            if src is not None:
                a.copy_(_dev(src[:, :ch], self.device))
                b.copy_(_dev(src[:, ch:], self.device))
            return (a, b), a, b
        full = torch.empty((self.n, self.c, self.h, self.w), dtype=torch.float32, device=self.device)
        if src is not None:
            full.copy_(_dev(src, self.device))
        return full, full[:, :ch], full[:, ch:]

    def new_stream_pair(self, src=None):
        """A pair of the residual stream's type: int32 codes when frac_bits > 0
        (src, real values, is converted by the library), else as new_pair."""
        if not self.frac_bits:
            return self.new_pair(src)
        assert not self.split_buffers
        pair = self.new_pair(src)
        full = pair[0]
        if src is not None:
            B.revnet_fixed_from_float(full, self.frac_bits, full)   # in place: same bytes, now int32 codes
        q = full.view(torch.int32)
        ch = self.c // 2
        return q, q[:, :ch], q[:, ch:]

    def stream_to_host(self, full):
        """Real values of a stream tensor as float64."""
        if not self.frac_bits:
            return self.to_host(full)
        out = torch.empty(full.shape, dtype=torch.float32, device=self.device)
        B.revnet_fixed_to_float(full, self.frac_bits, out)
        return out.cpu().numpy().astype(np.float64)

    def to_host(self, full):
        if self.split_buffers:
            return np.concatenate([full[0].cpu().numpy(), full[1].cpu().numpy()], axis=1).astype(np.float64)
        return full.cpu().numpy().astype(np.float64)

    def set_params(self, params):
        self.params = upload_params(params, self.device)
        self.grads = zeros_like_params(self.params)
        self._pp = B.pack_params(self.params)
        self._pg = B.pack_grads(self.grads)

    # -- calls ----------------------------------------------------------------
    def forward(self, xpair, ypair, stream=None):
        if self.frac_bits:
            B.revnet_stack_fwd_fixed(self.desc, self.depth, self.frac_bits, xpair[1], xpair[2], self._pp, ypair[1],
                                     ypair[2], self.ws, stream)
        else:
            B.revnet_stack_fwd(self.desc, self.depth, xpair[1], xpair[2], self._pp, ypair[1], ypair[2],
                               self.ws, stream)

    def backward(self, ypair, dypair, xpair, dxpair, accumulate=False, stream=None):
        if self.frac_bits:
            B.revnet_stack_bwd_fixed(self.desc, self.depth, self.frac_bits, ypair[1], ypair[2], dypair[1], dypair[2],
                                     self._pp, xpair[1], xpair[2], dxpair[1], dxpair[2], self._pg, int(accumulate),
                                     self.ws, stream)
        else:
            B.revnet_stack_bwd(self.desc, self.depth, ypair[1], ypair[2], dypair[1], dypair[2], self._pp,
                               xpair[1], xpair[2], dxpair[1], dxpair[2], self._pg, int(accumulate), self.ws,
                               stream)

    def activation_bytes(self):
        """Bytes alive between the end of forward and the end of backward:
        top-of-stack activations, their gradients, and the backward workspace."""
        s = self.n * self.c * self.h * self.w * 4
        return dict(stream=s, grads=s, workspace=self.bwd_bytes, total=2 * s + self.bwd_bytes)


def upload_down(P, device="cuda:0"):
    """{R: [{w,gamma,beta,stride}], S: {w}} of host arrays -> device tensors (the stride is part of the descriptor)."""
    return dict(R=[{k: _dev(L[k], device) for k in ("w", "gamma", "beta")} for L in P["R"]],
                S=dict(w=_dev(P["S"]["w"], device)))


def zeros_like_down(D):
    return dict(R=[{k: torch.zeros_like(v) for k, v in L.items()} for L in D["R"]], S=dict(w=torch.zeros_like(D["S"]["w"])))


def download_down(D):
    f = lambda v: v.detach().cpu().numpy().astype(np.float64)
    return dict(R=[{k: f(v) for k, v in L.items()} for L in D["R"]], S=dict(w=f(D["S"]["w"])))


class BodyRunner:
    """Device buffers of a multi-stage body (reversible stages joined by
    subsampling blocks) and the calls into the C ABI.  Keeps one activation
    and one gradient tensor per stage, whatever the stages' depths."""

    def __init__(self, kind, n, h, w, channels, depths, widths, conv="f32", eps=1e-5, device="cuda:0", frac_bits=0,
                 **_unused):
        self.n, self.h, self.w, self.channels, self.depths = n, h, w, tuple(channels), tuple(depths)
        self.frac_bits = int(frac_bits)   # > 0: the stage tops hold fixed-point codes (int32 bit patterns in the fp32 tensors)
        self.device = torch.device(device)
        stages = [B.BlockDesc(kind, c // 2, wd or 0, eps, conv) for c, wd in zip(channels, widths)]
        downs = [B.DownDesc(kind, channels[s], channels[s + 1], 0, eps, conv) for s in range(len(channels) - 1)]
        self.down_descs = downs
        self.desc = B.BodyDesc(stages, depths, downs)
        query = B.revnet_body_fixed_workspace_bytes if self.frac_bits else B.revnet_body_workspace_bytes
        self.fwd_bytes, self.bwd_bytes = query(self.desc, n, h, w)
        self.ws = torch.empty(max(self.fwd_bytes, self.bwd_bytes), dtype=torch.uint8, device=self.device)
        shape = lambda s: (n, channels[s], h >> s, w >> s)
        self.tops = [torch.empty(shape(s), dtype=torch.float32, device=self.device) for s in range(len(channels))]
        self.dtops = [torch.empty_like(t) for t in self.tops]

    def set_params(self, stages, downs):
        self.stage_params = [upload_params(st, self.device) for st in stages]
        self.down_params = [upload_down(P, self.device) for P in downs]
        self.stage_grads = [zeros_like_params(st) for st in self.stage_params]
        self.down_grads = [zeros_like_down(D) for D in self.down_params]
        # marshalled once: the per-call work is then independent of the depths
        self._sp, self._sg = B.pack_stages(self.stage_params), B.pack_stages(self.stage_grads)
        self._dp, self._dg = B.pack_down(self.down_params), B.pack_down(self.down_grads)

    def forward(self, x, stream=None):
        """x: device tensor [n, channels[0], h, w]; it may be self.tops[0]."""
        if self.frac_bits:
            B.revnet_body_fwd_fixed(self.desc, self.frac_bits, x, self._sp, self._dp, self.tops, self.ws, stream)
        else:
            B.revnet_body_fwd(self.desc, x, self._sp, self._dp, self.tops, self.ws, stream)

    def backward(self, accumulate=False, stream=None):
        """self.dtops[-1] holds the upstream derivative; see revnet_body_bwd for what is left where."""
        if self.frac_bits:
            B.revnet_body_bwd_fixed(self.desc, self.frac_bits, self.tops, self.dtops, self._sp, self._dp, self._sg,
                                    self._dg, int(accumulate), self.ws, stream)
        else:
            B.revnet_body_bwd(self.desc, self.tops, self.dtops, self._sp, self._dp, self._sg, self._dg, int(accumulate),
                              self.ws, stream)

    def top_to_host(self, s):
        """Real values of stage s's top as float64."""
        if not self.frac_bits:
            return self.tops[s].cpu().numpy().astype(np.float64)
        out = torch.empty_like(self.tops[s])
        B.revnet_fixed_to_float(self.tops[s], self.frac_bits, out)
        return out.cpu().numpy().astype(np.float64)

    def activation_bytes(self):
        """Bytes alive between the end of forward and the end of backward."""
        acts = sum(t.numel() * 4 for t in self.tops)
        return dict(stream=acts, grads=acts, workspace=self.bwd_bytes, total=2 * acts + self.bwd_bytes)


class NetRunner:
    """Stem (image convolution, optional pooling) followed by a body: the whole
    network up to the last stage's top.  Stored between forward and backward:
    the image, the convolution's output when it is pooled, and one activation
    per stage."""

    def __init__(self, cfg, stem, device="cuda:0"):
        self.body = BodyRunner(device=device, **cfg)
        self.device = self.body.device
        c0 = cfg["channels"][0]
        ks = int(stem["w"].shape[2])
        self.stem_desc = B.rvn_stem_desc(3, c0, ks, int(stem["stride"]), 1 if stem["pool"] else 0)
        self.stem_w = _dev(stem["w"], self.device)
        self.stem_dw = torch.zeros_like(self.stem_w)
        self.pool = bool(stem["pool"])
        self.stride = int(stem["stride"])
        self.conv_out = None
        self.ws = None

    def set_params(self, stages, downs):
        self.body.set_params(stages, downs)

    def forward(self, img, stream=None):
        n, _, h, w = img.shape
        if self.pool and self.conv_out is None:
            ho, wo = (h - 1) // self.stride + 1, (w - 1) // self.stride + 1
            self.conv_out = torch.empty((n, self.stem_w.shape[0], ho, wo), dtype=torch.float32, device=self.device)
        if self.ws is None:
            self.ws = torch.empty(max(B.revnet_stem_workspace_bytes(self.stem_desc, n, h, w), 256), dtype=torch.uint8,
                                  device=self.device)
        self.img = img
        # the stem writes the body's input into tops[0]; stage 0 then runs in place
        B.revnet_stem_fwd(self.stem_desc, img, self.stem_w, self.conv_out, self.body.tops[0], stream)
        self.body.forward(self.body.tops[0], stream)

    def backward(self, stream=None):
        """body.dtops[-1] holds the upstream derivative."""
        self.body.backward(stream=stream)
        B.revnet_stem_bwd(self.stem_desc, self.img, self.conv_out, self.body.dtops[0], self.stem_dw, 0, self.ws, stream)

    def activation_bytes(self):
        act = self.body.activation_bytes()
        stem = self.img.numel() * 4 + (self.conv_out.numel() * 4 if self.conv_out is not None else 0)
        act["stem_stored"] = stem
        act["stem_workspace"] = self.ws.numel()
        act["total"] += stem + self.ws.numel()
        return act
