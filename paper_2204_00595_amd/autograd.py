"""torch.autograd glue for the library: no arithmetic here, only which C-ABI call runs when.

``monarch_linear(x, R, L, bias)`` is differentiable: its forward is ``monarch_fwd_bias`` (or, without a
bias and with ``save_intermediate=True``, ``monarch_fwd_save``), its backward ``monarch_bwd_bias`` /
``monarch_bwd_saved``.  ``MonarchLinear`` holds the two factors (and the bias) as parameters.  Leading
dimensions of ``x`` are flattened into the batch.  Everything runs in the HIP kernels; there is no
fallback for CPU tensors.
"""
from __future__ import annotations

import math

import torch

from . import binding


class _MonarchLinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, R, L, bias, save_intermediate):
        k, q, p = R.shape
        x2 = x.reshape(-1, k * p)
        if not x2.is_contiguous():
            x2 = x2.contiguous()
        saved = None
        if bias is None and save_intermediate:
            y, saved = binding.monarch_fwd_save(x2, R, L)
        elif bias is None:
            y = binding.monarch_fwd(x2, R, L)
        else:
            y = binding.monarch_fwd_bias(x2, R, L, bias)
        ctx.save_for_backward(x2, R, L, saved if saved is not None else x2.new_empty(0))
        ctx.has_saved = saved is not None
        ctx.has_bias = bias is not None
        ctx.x_shape = x.shape
        return y.reshape(*x.shape[:-1], y.shape[-1])

    @staticmethod
    def backward(ctx, dy):
        x2, R, L, saved = ctx.saved_tensors
        k, s, q = L.shape
        dy2 = dy.reshape(-1, k * s)
        if not dy2.is_contiguous():
            dy2 = dy2.contiguous()
        dx, dR, dL, dbias = binding.monarch_bwd_saved(dy2, x2, saved if ctx.has_saved else None, R, L,
                                                      want_dbias=ctx.has_bias)
        return dx.reshape(ctx.x_shape), dR, dL, dbias, None


def monarch_linear(x: torch.Tensor, R: torch.Tensor, L: torch.Tensor, bias: torch.Tensor | None = None,
                   save_intermediate: bool = True) -> torch.Tensor:
    """y = x M^T (+ bias) with M = P L P^T R; differentiable in x, R, L and bias."""
    return _MonarchLinearFn.apply(x, R, L, bias, save_intermediate)


class MonarchLinear(torch.nn.Module):
    """A linear layer whose weight is a Monarch matrix with `nblocks` blocks per factor.

    in_features = nblocks * p, out_features = nblocks * s, inner block size q = min(p, s) unless given
    (the shapes of the paper's Transformer layers: 768 -> 3072 is p = q = 192, s = 768 with four blocks).
    """

    def __init__(self, in_features: int, out_features: int, nblocks: int = 4, bias: bool = True, q: int | None = None,
                 device=None, dtype=torch.bfloat16, save_intermediate: bool = True):
        super().__init__()
        if in_features % nblocks or out_features % nblocks:
            raise ValueError("nblocks must divide in_features and out_features")
        p, s = in_features // nblocks, out_features // nblocks
        q = min(p, s) if q is None else q
        self.in_features, self.out_features, self.nblocks = in_features, out_features, nblocks
        self.save_intermediate = save_intermediate
        self.R = torch.nn.Parameter(torch.empty((nblocks, q, p), device=device, dtype=dtype))
        self.L = torch.nn.Parameter(torch.empty((nblocks, s, q), device=device, dtype=dtype))
        self.bias = torch.nn.Parameter(torch.zeros((out_features,), device=device, dtype=dtype)) if bias else None
        with torch.no_grad():
            self.R.normal_(0.0, 1.0 / math.sqrt(p))
            self.L.normal_(0.0, 1.0 / math.sqrt(q))

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        return monarch_linear(x, self.R, self.L, self.bias, self.save_intermediate)

    def to_dense(self) -> torch.Tensor:
        """The (out_features, in_features) matrix this layer applies (the sparse-to-dense switch)."""
        return binding.monarch_to_dense(self.R.detach(), self.L.detach())
