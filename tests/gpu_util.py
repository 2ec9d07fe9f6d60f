"""Helpers for the GPU parity tests: move seeded host inputs to the device, call the
C-ABI through the binding, bring results back as float64."""
import numpy as np
import torch

import paper_2410_20926_amd as ta

TOL = {"f32": 1e-5, "bf16": 2e-2}          # max-abs forward tolerance per dtype (vs the float64 oracle)


def ta_dtype(dtype: str) -> int:
    return ta.TA_F32 if dtype == "f32" else ta.TA_BF16


def torch_dtype(dtype: str):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to("cuda").to(torch_dtype(dtype)).contiguous()


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def alloc_bytes(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def multihop_forward(q, k, v, dims, dtype, causal, save=False, **plan_kw):
    """q,k,v: host float32 arrays [B,N,H,D].  Returns (o as float64 host array, plan, device tensors)."""
    B, N, Hq, D = q.shape
    Hkv = k.shape[2]
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta_dtype(dtype), causal, **plan_kw)
    dq, dk, dv = to_dev(q, dtype), to_dev(k, dtype), to_dev(v, dtype)
    o = torch.full((B, N, Hq, D), float("nan"), dtype=torch_dtype(dtype), device="cuda")
    wsb = plan.workspace_bytes(save)
    ws = alloc_bytes(wsb)
    ta.ta_multihop_forward(plan, dq, dk, dv, o, ws, wsb, save)
    torch.cuda.synchronize()
    return to_host(o), plan, dict(q=dq, k=dk, v=dv, o=o, ws=ws, wsb=wsb)


def multihop_backward(plan, dev, d_o, dtype):
    """After multihop_forward(save=True): returns dq, dk, dv as float64 host arrays."""
    g = to_dev(d_o, dtype)
    dq = torch.full_like(dev["q"], float("nan"))
    dk = torch.full_like(dev["k"], float("nan"))
    dv = torch.full_like(dev["v"], float("nan"))
    scb = plan.backward_scratch_bytes()
    sc = alloc_bytes(scb)
    ta.ta_multihop_backward(plan, dev["q"], dev["k"], dev["v"], g, dev["ws"], dev["wsb"], dq, dk, dv, sc, scb)
    torch.cuda.synchronize()
    return to_host(dq), to_host(dk), to_host(dv)
