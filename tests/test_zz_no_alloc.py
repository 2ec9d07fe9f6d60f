"""The multi-hop forward that allocates nothing (ta_multihop_forward_static), through the C ABI:
its output against ta_multihop_forward's on the same inputs, bit for bit (the same kernels run;
only the home of the inter-hop tensors differs), on two calls in a row, the second with a
smaller input, so that what the first call left in the library's own workspace would show."""
import numpy as np
import pytest
import torch

import paper_2410_20926_amd as ta
from gpu_util import TOL, alloc_bytes, to_dev, to_host
from oracle import tensattn_oracle as orc
from paper_2410_20926_amd.workloads import make_inputs

pytestmark = pytest.mark.gpu


def run_both(dims, B, Hq, Hkv, D, seed, causal=True):
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=seed, dtype="bf16")
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, causal)
    tq, tk, tv = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
    o_ref = torch.full((B, N, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    o_sta = torch.full_like(o_ref, float("nan"))
    wsb = plan.workspace_bytes(False)
    ws = alloc_bytes(wsb)
    ta.ta_multihop_forward(plan, tq, tk, tv, o_ref, ws, wsb, False)
    ta.ta_multihop_forward_static(plan, tq, tk, tv, o_sta)
    torch.cuda.synchronize()
    assert wsb > 0, "the case must use inter-hop tensors"
    return (q, k, v), o_ref, o_sta, plan


def test_static_workspace_forward_matches_the_caller_workspace_forward_twice():
    # first call: three separate hops, two ping-pong tensors of 4 MiB; second call: a smaller problem
    # with fused last hops (one intermediate tensor of 1 MiB) over the workspace the first one used
    for dims, B, Hq, Hkv, D, seed in (((16, 8, 16), 1, 8, 2, 128, 11), ((2, 32, 32), 1, 2, 1, 128, 12)):
        (q, k, v), o_ref, o_sta, plan = run_both(dims, B, Hq, Hkv, D, seed)
        assert torch.equal(o_ref.view(torch.int16), o_sta.view(torch.int16)), f"dims {dims}: outputs differ"
        ref = orc.tensorized_attention_forward(q, k, v, dims, True)
        err = np.abs(to_host(o_sta) - ref).max()
        assert err <= TOL["bf16"], f"dims {dims}: max-abs error {err:.3e} against the oracle"


def test_static_workspace_forward_refuses_what_does_not_fit():
    # two ping-pong tensors of 64 MiB each
    plan = ta.ta_plan_create(1, 32, 8, 128, (16, 32, 16), ta.TA_BF16, True)
    assert plan.workspace_bytes(False) > ta.TA_STATIC_WORKSPACE_BYTES
    t = torch.zeros(1, 8192, 32, 128, dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros(1, 8192, 8, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ta.TaError) as e:
        ta.ta_multihop_forward_static(plan, t, kv, kv, torch.empty_like(t))
    assert e.value.name == "TA_ERR_WORKSPACE" and "64" in e.value.detail or "67108864" in e.value.detail
    # the same tokens with a fused last pair need one tensor of 64 MiB: accepted
    fits = ta.ta_plan_create(1, 32, 8, 128, (8, 32, 32), ta.TA_BF16, True)
    assert fits.workspace_bytes(False) == ta.TA_STATIC_WORKSPACE_BYTES
    o = torch.full_like(t, float("nan"))
    ta.ta_multihop_forward_static(fits, t, kv, kv, o)
    torch.cuda.synchronize()
    assert torch.count_nonzero(o).item() == 0          # V = 0 gives O = 0, and no NaN is left


def test_static_workspace_forward_under_graph_capture():
    """What the entry point is for: the call allocates nothing and takes no workspace, so it can be
    captured into a HIP graph as it stands; every replay, with eager work and synchronisations in
    between, reproduces the eager result.  (The first call on the device, above or here, happens
    outside the capture: it looks up the address of the library's workspace.)"""
    dims, B, Hq, Hkv, D = (4, 32, 32), 1, 8, 2, 128
    N = int(np.prod(dims))
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, True)
    gen = torch.Generator(device="cuda"); gen.manual_seed(21)
    q = torch.randn(B, N, Hq, D, device="cuda", generator=gen).bfloat16()
    k = torch.randn(B, N, Hkv, D, device="cuda", generator=gen).bfloat16()
    v = torch.randn(B, N, Hkv, D, device="cuda", generator=gen).bfloat16()
    o = torch.zeros(B, N, Hq, D, device="cuda", dtype=torch.bfloat16)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ta.ta_multihop_forward_static(plan, q, k, v, o)               # warm-up on the capture stream
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ta.ta_multihop_forward_static(plan, q, k, v, o)
    wsb = plan.workspace_bytes(False)
    for it in range(3):
        q.copy_(torch.randn(B, N, Hq, D, device="cuda", generator=gen).bfloat16())
        v.copy_(torch.randn(B, N, Hkv, D, device="cuda", generator=gen).bfloat16())
        eager = torch.empty_like(o)
        ta.ta_multihop_forward(plan, q, k, v, eager, alloc_bytes(wsb), wsb, False)
        torch.cuda.synchronize()
        o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, eager), f"replay {it} differs from the eager result"
