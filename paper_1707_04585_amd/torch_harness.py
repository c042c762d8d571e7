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
                 split_buffers=False, **_unused):
        self.desc = B.BlockDesc(kind, c // 2, width or 0, eps, conv)
        self.n, self.c, self.h, self.w, self.depth = n, c, h, w, depth
        self.device = torch.device(device)
        self.split_buffers = split_buffers
        self.fwd_bytes, self.bwd_bytes = B.revnet_workspace_bytes(self.desc, n, h, w)
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
        B.revnet_stack_fwd(self.desc, self.depth, xpair[1], xpair[2], self._pp, ypair[1], ypair[2],
                           self.ws, stream)

    def backward(self, ypair, dypair, xpair, dxpair, accumulate=False, stream=None):
        B.revnet_stack_bwd(self.desc, self.depth, ypair[1], ypair[2], dypair[1], dypair[2], self._pp,
                           xpair[1], xpair[2], dxpair[1], dxpair[2], self._pg, int(accumulate), self.ws,
                           stream)

    def activation_bytes(self):
        """Bytes alive between the end of forward and the end of backward:
        top-of-stack activations, their gradients, and the backward workspace."""
        s = self.n * self.c * self.h * self.w * 4
        return dict(stream=s, grads=s, workspace=self.bwd_bytes, total=2 * s + self.bwd_bytes)
