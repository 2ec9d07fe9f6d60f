"""torch.autograd glue over the C-ABI library: `tensorized_attention(q, k, v, dims, ...)` is a
differentiable call whose forward and backward are ta_multihop_forward / ta_multihop_backward
(Algorithm 1 of arXiv 2410.20926 and its derivative).  Nothing is computed here: this module
only allocates the output, the workspace that keeps the inter-hop O tensors for the backward,
and the gradient buffers, and hands pointers to the library.  Tensors are dense [B, N, H, D]."""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import tensattn as _ta

_PLANS = {}


def _plan(q: torch.Tensor, k: torch.Tensor, dims, causal, scale, window, valid_len) -> _ta.Plan:
    dtype = {torch.bfloat16: _ta.TA_BF16, torch.float32: _ta.TA_F32}.get(q.dtype)
    if dtype is None:
        raise TypeError(f"tensorized_attention: dtype {q.dtype} is not supported (bfloat16 or float32)")
    B, N, Hq, D = q.shape
    key = (B, Hq, k.shape[2], D, tuple(int(n) for n in dims), dtype, bool(causal), float(scale),
           None if window is None else tuple(int(w) for w in window), int(valid_len))
    plan = _PLANS.get(key)
    if plan is None:
        plan = _ta.ta_plan_create(B, Hq, k.shape[2], D, key[4], dtype, bool(causal), scale=float(scale),
                                  window=key[8], valid_len=int(valid_len))
        _PLANS[key] = plan
    return plan


class _TensorizedAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, dims, causal, scale, window, valid_len):
        for name, t in (("q", q), ("k", k), ("v", v)):
            if not (t.is_cuda and t.is_contiguous() and t.dim() == 4):
                raise ValueError(f"tensorized_attention: {name} must be a contiguous [B, N, H, D] tensor on the GPU")
        if k.shape != v.shape or q.dtype != k.dtype or q.dtype != v.dtype:
            raise ValueError("tensorized_attention: k and v must have the same shape, and q, k, v the same dtype")
        plan = _plan(q, k, dims, causal, scale, window, valid_len)
        save = any(ctx.needs_input_grad[:3])
        o = torch.empty_like(q)
        wsb = plan.workspace_bytes(save)
        ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device=q.device)
        _ta.ta_multihop_forward(plan, q, k, v, o, ws, wsb, save)
        if save:
            ctx.plan, ctx.wsb = plan, wsb
            ctx.save_for_backward(q, k, v, ws)
        return o

    @staticmethod
    def backward(ctx, d_o):
        q, k, v, ws = ctx.saved_tensors
        plan = ctx.plan
        d_o = d_o.contiguous()
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        scb = plan.backward_scratch_bytes()
        sc = torch.empty(max(scb, 256), dtype=torch.uint8, device=q.device)
        _ta.ta_multihop_backward(plan, q, k, v, d_o, ws, ctx.wsb, dq, dk, dv, sc, scb)
        return dq, dk, dv, None, None, None, None, None


def tensorized_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, dims: Sequence[int], causal: bool = True,
                         scale: float = 0.0, window: Optional[Sequence[int]] = None, valid_len: int = 0) -> torch.Tensor:
    """o = Algorithm 1 on the sequence viewed as a tensor of shape `dims` (their product = N).

    q: [B, N, H_q, D]; k, v: [B, N, H_kv, D]; bfloat16 or float32, contiguous, on the GPU.
    `scale` 0 means 1/sqrt(D); `window[i]` > 0 bands axis i; `valid_len` marks trailing padding.
    Differentiable in q, k, v (the backward is the library's, deterministic)."""
    return _TensorizedAttention.apply(q, k, v, tuple(dims), causal, scale, window, valid_len)
