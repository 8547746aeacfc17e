"""torch.autograd plumbing over the binding: no arithmetic happens here, forward and backward are the library's
nsa_sel_fwd / nsa_sel_bwd (or their gated variants) on the tensors autograd hands over."""
from __future__ import annotations

from typing import Optional

import torch

from .binding import SelAttention


class _SelectedAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, idx, cu, attn: SelAttention, rebuild_index: bool):
        o, lse = attn.forward(q, k, v, idx, cu, rebuild_index=rebuild_index)
        ctx.attn, ctx.cu = attn, cu
        ctx.save_for_backward(q, k, v, o, lse)
        ctx.mark_non_differentiable(lse)
        return o, lse

    @staticmethod
    def backward(ctx, do, _dlse):
        q, k, v, o, lse = ctx.saved_tensors
        dq, dk, dv = ctx.attn.backward(q, k, v, o, lse, do.contiguous(), ctx.cu)
        return dq, dk, dv, None, None, None, None


class _GatedSelectedAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, idx, gate, o_acc, cu, attn: SelAttention, rebuild_index: bool):
        o_out, o, lse = attn.forward_gated(q, k, v, idx, gate, o_acc, cu, rebuild_index=rebuild_index)
        ctx.attn, ctx.cu, ctx.has_acc = attn, cu, o_acc is not None
        ctx.save_for_backward(q, k, v, o, lse, gate)
        return o_out

    @staticmethod
    def backward(ctx, do_out):
        q, k, v, o, lse, gate = ctx.saved_tensors
        do_out = do_out.contiguous()
        dq, dk, dv, dgate = ctx.attn.backward_gated(q, k, v, o, lse, do_out, gate, ctx.cu)
        return dq, dk, dv, None, dgate, (do_out if ctx.has_acc else None), None, None, None


def selected_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, idx: torch.Tensor, attn: SelAttention,
                       cu: Optional[torch.Tensor] = None, *, gate: Optional[torch.Tensor] = None,
                       o_acc: Optional[torch.Tensor] = None, rebuild_index: bool = True):
    """Differentiable selected-block (or, with attn's window, sliding-window) attention on bf16 device tensors.

    Without `gate`: returns (O, LSE).  With `gate` (fp32 [tokens, hq]): returns O_acc + gate * O, differentiable in
    q, k, v, gate and o_acc.  `attn` owns the workspaces; the backward reuses the index the forward built, so one
    `attn` serves one forward/backward pair at a time."""
    if gate is None:
        return _SelectedAttention.apply(q, k, v, idx, cu, attn, rebuild_index)
    return _GatedSelectedAttention.apply(q, k, v, idx, gate, o_acc, cu, attn, rebuild_index)
