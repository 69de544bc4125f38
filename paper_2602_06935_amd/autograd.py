"""torch.autograd plumbing around the C-ABI binding: forward calls cotten_attn_fwd, backward
calls cotten_attn_bwd (which rebuilds the d x d state from K, V: nothing but the inputs is
saved).  The kernels return d loss / d log(scale) per slice; the one piece of arithmetic done
here, in torch, is its conversion to d loss / d scale (a division by the scale, [B,H] values)."""
from __future__ import annotations

from typing import Optional

import torch

from . import binding


class _CosineAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, mask, scale, eps, slice_scale, layout):
        ctx.save_for_backward(Q, K, V, mask, slice_scale)
        ctx.scale, ctx.eps, ctx.layout = scale, eps, layout
        return binding.cotten_attn_fwd(Q, K, V, mask, scale=scale, eps=eps, slice_scale=slice_scale,
                                       layout=layout)

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, mask, slice_scale = ctx.saved_tensors
        dlog = None
        if slice_scale is not None and ctx.needs_input_grad[6]:
            B, H, _, _ = binding._dims(Q, ctx.layout)
            dlog = torch.empty(B, H, device=Q.device, dtype=torch.float32)
        dQ, dK, dV = binding.cotten_attn_bwd(Q, K, V, mask, dO.contiguous(), scale=ctx.scale,
                                             eps=ctx.eps, slice_scale=slice_scale,
                                             dlog_scale=dlog, layout=ctx.layout)
        # d loss / d scale = (d loss / d log scale) / scale
        dscale = None if dlog is None else dlog / slice_scale
        return dQ, dK, dV, None, None, None, dscale, None


def cosine_attention(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                     mask: Optional[torch.Tensor] = None, *, scale: Optional[float] = None,
                     eps: Optional[float] = None, slice_scale: Optional[torch.Tensor] = None,
                     layout: str = "bhnd") -> torch.Tensor:
    """O = scale * Qhat (Khat^T V) under the key mask, differentiable in Q, K, V and, when
    given, in the per-slice scales `slice_scale` ([B,H] float32)."""
    return _CosineAttention.apply(Q, K, V, mask, scale, eps, slice_scale, layout)
