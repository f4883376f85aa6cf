"""torch.autograd wrapper of the Lory layer (Algorithm 1 of the paper and its gradient).

`lory_layer(x, R, Wg, Wu, Wd, T)` is what the paper's listing calls on the
hidden states of a transformer block: route every segment on the previous
segment's mean, merge the experts, apply the merged SwiGLU FFN.  Everything
is computed by the HIP library through `binding`; this module only chains the
entry points and hands torch the gradients (dX, dR, dWg, dWu, dWd).
"""
from __future__ import annotations

import torch

from . import binding as lb


class _LoryLayer(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, R, Wg, Wu, Wd, T, save_merged):
        B, L, d = x.shape
        E, _, d_ff = Wg.shape
        S = B * (L // T)
        x = x.contiguous()
        hbar = torch.empty((S, d), dtype=torch.float32, device=x.device)
        w = lb.lory_route(x, R, T, hbar=hbar, d_ff=d_ff)
        G = torch.empty((B * L, d_ff), dtype=x.dtype, device=x.device)
        U = torch.empty_like(G)
        Wbar = None
        if save_merged:
            Wbar = lb.alloc_merged_save(lb.make_shape(B, L, T, d, d_ff, E, x.dtype), x.device)
        y = lb.lory_merged_ffn_fwd(x, w, Wg, Wu, Wd, T, G_save=G, U_save=U, Wbar_save=Wbar)
        ctx.save_for_backward(x, R, Wg, Wu, Wd, w, hbar, G, U)
        ctx.Wbar = Wbar
        ctx.T = T
        return y

    @staticmethod
    def backward(ctx, dy):
        x, R, Wg, Wu, Wd, w, hbar, G, U = ctx.saved_tensors
        T = ctx.T
        d_ff = Wg.shape[2]
        dX, dWg, dWu, dWd, dw = lb.lory_merged_ffn_bwd(x, w, Wg, Wu, Wd, dy.contiguous(), T, G_save=G, U_save=U,
                                                       grad_dtype=Wg.dtype, Wbar_save=ctx.Wbar)
        dR = lb.lory_route_bwd(R, w, hbar, dw, dX, T, d_ff=d_ff)   # adds the router path into dX
        return dX, dR.to(R.dtype), dWg, dWu, dWd, None, None


def lory_layer(x: torch.Tensor, R: torch.Tensor, Wg: torch.Tensor, Wu: torch.Tensor, Wd: torch.Tensor,
               T: int, save_merged: bool = True) -> torch.Tensor:
    """y [B, L, d] = Lory MoE FFN layer of x [B, L, d]; differentiable in x, R and the expert stacks.

    R [d, E]; Wg, Wu [E, d, d_ff]; Wd [E, d_ff, d]; all of x's dtype (bf16 or fp32), on the GPU.
    save_merged keeps the merged parameters of all segments for the backward (3*S*d*d_ff elements)
    where the shape supports it, instead of re-merging.
    """
    if save_merged and x.dtype != torch.bfloat16:
        save_merged = False
    if save_merged:
        B, L, d = x.shape
        E, _, d_ff = Wg.shape
        if lb.lory_merged_save_bytes(lb.make_shape(B, L, T, d, d_ff, E, x.dtype)) == 0:
            save_merged = False
    return _LoryLayer.apply(x, R, Wg, Wu, Wd, T, save_merged)
