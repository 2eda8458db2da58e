"""torch.autograd front end of the quantisation layer W -> r_tau(W, C*(W)) (Alg. 2, per-layer steps).

Argument marshalling only: the forward is one idkm_forward call, the backward one idkm_backward call on the same
context; every step runs in the library's kernels.  One context per layer (the library keeps C*, n*, F* and a borrowed
pointer to W between the two calls).
"""
from __future__ import annotations

import torch

from . import binding


class _Quantize(torch.autograd.Function):
    @staticmethod
    def forward(fn, W, C0, layer):
        out = layer.ctx.forward(W.detach(), C0, layer.tau, layer.tol, layer.max_iter, layer.dist, want_Wq=True)
        layer.last_forward = out["info"]
        layer.C = out["C"]
        fn.layer = layer
        fn.mark_non_differentiable(out["C"])
        return out["Wq"], out["C"]

    @staticmethod
    def backward(fn, dWq, _dC):
        layer = fn.layer
        res = layer.ctx.backward(dWq.contiguous(), layer.bwd_mode, tol=layer.bwd_tol, max_iter=layer.bwd_max_iter,
                                 alpha=layer.alpha)
        layer.last_backward = res["info"]
        return res["dW"], None, None


class SoftKMeansQuantize:
    """One layer's quantiser.  `layer(W, C0)` returns (Wq, C*) with Wq differentiable with respect to W by implicit
    differentiation of the soft k-means fixed point (bwd_mode: binding.BWD_IMPLICIT, BWD_JFB, BWD_DENSE, BWD_GMRES).
    C* is returned detached, to warm-start the next step's C0."""

    def __init__(self, tau, dist, tol=1e-6, max_iter=200, bwd_mode=binding.BWD_IMPLICIT, bwd_tol=1e-6,
                 bwd_max_iter=1000, alpha=1.0, device=0):
        self.ctx = binding.Context(device)
        self.tau, self.dist, self.tol, self.max_iter = float(tau), int(dist), float(tol), int(max_iter)
        self.bwd_mode, self.bwd_tol, self.bwd_max_iter, self.alpha = int(bwd_mode), float(bwd_tol), int(bwd_max_iter), float(alpha)
        self.last_forward = self.last_backward = self.C = None

    def __call__(self, W, C0):
        if W.dim() != 2 or C0.dim() != 2 or W.shape[1] != C0.shape[1]:
            raise ValueError("W must be [m, d] and C0 [k, d]")
        return _Quantize.apply(W.contiguous(), C0.contiguous(), self)

    def close(self):
        self.ctx.close()
