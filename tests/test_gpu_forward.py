"""GPU parity, forward: the HIP path, called through the C ABI, against the CPU oracle,
element by element on the same seeded inputs.  Tolerances: max-abs 1e-5 (fp32) and
2e-2 (bf16) against the float64 oracle evaluated on the identical (bf16-rounded) inputs."""
import math

import numpy as np
import pytest
import torch

import paper_2410_20926_amd as ta
from gpu_util import TOL, alloc_bytes, multihop_forward, ta_dtype, to_dev, to_host, torch_dtype
from oracle import tensattn_oracle as orc
from paper_2410_20926_amd.workloads import WORKLOADS, make_inputs, make_workload_inputs

pytestmark = pytest.mark.gpu


def check(got, ref, tol, what=""):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref).max()
    assert err <= tol, f"{what}: max-abs error {err:.3e} > {tol:.1e}"
    return err


def test_config1_fp32_16x16():
    """fp32, B=1, H=1, D=64, N=256 as 16x16, non-causal; also the d=1 full-attention case."""
    w = WORKLOADS["c1"]
    q, k, v = make_workload_inputs(w)
    got, plan, _ = multihop_forward(q, k, v, w.dims, "f32", False)
    ref = orc.tensorized_attention_forward(q, k, v, w.dims, False)
    check(got, ref, TOL["f32"], "c1")
    got1, _, _ = multihop_forward(q, k, v, (256,), "f32", False)
    check(got1, orc.tensorized_attention_forward(q, k, v, (256,), False), TOL["f32"], "c1 d=1")
    ref_full = orc.attention(q[0, :, 0], k[0, :, 0], v[0, :, 0], 1.0 / 8.0, False)
    check(got1[0, :, 0], ref_full, TOL["f32"], "c1 d=1 vs Eq. 1")


CASES = [
    # dims, B, Hq, Hkv, D, causal, dtype, qk_scale
    ((5, 3, 7), 2, 4, 2, 40, True, "f32", 1.0),
    ((5, 3, 7), 1, 2, 2, 64, False, "f32", 1.0),
    ((70,), 1, 2, 1, 64, True, "f32", 1.0),            # streams over three key tiles, ragged tail
    ((3, 45), 1, 1, 1, 128, False, "f32", 1.0),
    ((2, 33, 2), 1, 2, 2, 256, True, "f32", 1.0),      # widest head, 16-row key tiles
    ((1,), 2, 2, 1, 8, True, "f32", 1.0),              # N = 1
    ((1, 6, 1), 1, 1, 1, 16, True, "f32", 1.0),        # unit axes are no-op hops
    ((16, 16), 1, 4, 4, 128, True, "bf16", 1.0),
    ((32, 16, 16), 1, 2, 2, 128, True, "bf16", 1.0 / math.sqrt(128)),
    ((32, 32, 32), 1, 4, 1, 128, True, "bf16", 1.0 / math.sqrt(128)),
    ((32, 32), 2, 8, 2, 128, False, "bf16", 1.0),
    ((64, 32), 1, 4, 1, 128, True, "bf16", 1.0),
    ((16, 64), 1, 2, 2, 64, True, "bf16", 1.0),
    ((7, 48, 5), 1, 2, 1, 64, True, "bf16", 1.0),      # ragged tiles: 4 fibres of 7, one padded 48-row fibre, 6 fibres of 5
    ((130,), 1, 2, 2, 128, False, "bf16", 1.0),        # streaming kernel, ragged last key tile
    ((130,), 1, 2, 1, 128, True, "bf16", 1.0),
    ((128, 4, 2), 1, 4, 1, 128, True, "bf16", 1.0),    # extrapolated first axis (Sec. 4.3), strided
    ((3, 97), 2, 2, 2, 64, True, "bf16", 1.0),
    ((257,), 1, 1, 1, 64, False, "bf16", 1.0),
    ((97, 3), 2, 8, 2, 64, True, "bf16", 1.0),         # group-shared streaming, all query tiles in one workgroup, D = 64, ragged
    ((2, 128), 1, 4, 1, 64, False, "bf16", 1.0),       # the same, non-causal, value input per head on the second hop
    ((300, 2), 1, 8, 2, 64, True, "bf16", 1.0),        # group-shared streaming, one workgroup per query tile, D = 64
    ((2, 161), 1, 4, 1, 128, False, "bf16", 1.0),
    ((6, 9, 4), 1, 4, 4, 100, True, "bf16", 1.0),      # head width 100 (OpenLLaMA-3B's): 8-byte-granular rows in 128-wide tiles
    ((32, 32), 2, 8, 2, 100, True, "bf16", 1.0),       # the same with grouped-query heads (group-shared kernel)
    ((48, 5), 1, 4, 1, 96, False, "bf16", 1.0),        # two-tile kernels, width 96
    ((7, 64), 1, 3, 3, 40, True, "bf16", 1.0),         # width 40 in 64-wide tiles
    ((10, 6), 1, 2, 2, 90, True, "bf16", 1.0),         # even but not a multiple of 4: generic kernels
    ((130, 2), 1, 3, 3, 100, True, "bf16", 1.0),       # width 100 on the streaming kernels: per head,
    ((100, 4), 2, 8, 2, 96, True, "bf16", 1.0),        # group-shared with all query tiles in one workgroup,
    ((2, 300), 1, 4, 1, 40, False, "bf16", 1.0),       # and group-shared with one workgroup per query tile
    ((5, 12), 2, 2, 1, 36, False, "f32", 1.0),
]


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype,qs", CASES)
def test_multihop_forward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype, qs):
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=1000 + N + D, dtype=dtype, qk_scale=qs)
    got, plan, _ = multihop_forward(q, k, v, dims, dtype, causal)
    ref = orc.tensorized_attention_forward(q, k, v, dims, causal)
    check(got, ref, TOL[dtype], f"{dims} {dtype}")


@pytest.mark.parametrize("dtype,dims,D", [("f32", (4, 6, 5), 64), ("bf16", (32, 16), 128)])
def test_axis_forward_each_axis_and_both_value_inputs(dtype, dims, D):
    """ta_axis_attn_forward alone, for every axis, with V (H_kv heads) and with an O
    (H_q heads) as the value input, against Eq. 4 in the oracle."""
    B, Hq, Hkv = 2, 4, 2
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=77, dtype=dtype)
    x = make_inputs(B, N, Hq, Hq, D, seed=78, dtype=dtype)[2]          # stands for a previous O
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta_dtype(dtype), True)
    dq, dk, dv, dx = (to_dev(a, dtype) for a in (q, k, v, x))
    for axis in range(len(dims)):
        for vin, src, srch in ((ta.TA_VIN_KV, dv, v), (ta.TA_VIN_O, dx, x)):
            o = torch.full((B, N, Hq, D), float("nan"), dtype=torch_dtype(dtype), device="cuda")
            ta.ta_axis_attn_forward(plan, axis, dq, dk, src, vin, o)
            torch.cuda.synchronize()
            got = to_host(o)
            for b in range(B):
                for h in range(Hq):
                    hv = h // 2 if vin == ta.TA_VIN_KV else h
                    ref = orc.axis_attention(q[b, :, h], k[b, :, h // 2], srch[b, :, hv], dims, axis,
                                             1.0 / math.sqrt(D), True)
                    check(got[b, :, h], ref, TOL[dtype], f"axis {axis} vin {vin}")


def test_hop_order_and_scale_are_honoured():
    dims, D = (6, 5), 64
    q, k, v = make_inputs(1, 30, 2, 1, D, seed=5, dtype="f32")
    got, _, _ = multihop_forward(q, k, v, dims, "f32", True, hop_order=(1, 0), scale=0.2)
    ref = orc.tensorized_attention_forward(q, k, v, dims, True, scale=0.2, hop_order=(1, 0))
    check(got, ref, TOL["f32"], "reversed hop order")
    other = orc.tensorized_attention_forward(q, k, v, dims, True, scale=0.2)
    assert np.abs(other - ref).max() > 1e-3


@pytest.mark.parametrize("dtype,dims", [("f32", (32, 6)), ("bf16", (32, 6)), ("bf16", (3, 32, 32))])   # the last: fused pair
def test_strided_head_major_layout(dtype, dims):
    """Every tensor stored [B, H, N, D]; results must equal the dense call's."""
    B, Hq, Hkv, D = 2, 4, 2, 128
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=9, dtype=dtype)
    ref = orc.tensorized_attention_forward(q, k, v, dims, True)
    sq = (Hq * N * D, D, N * D)
    skv = (Hkv * N * D, D, N * D)
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta_dtype(dtype), True, q_strides=sq, kv_strides=skv, o_strides=sq)
    dq, dk, dv = (to_dev(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), dtype) for a in (q, k, v))
    o = torch.full((B, Hq, N, D), float("nan"), dtype=torch_dtype(dtype), device="cuda")
    wsb = plan.workspace_bytes(False)
    ws = alloc_bytes(wsb)
    ta.ta_multihop_forward(plan, dq, dk, dv, o, ws, wsb, False)
    torch.cuda.synchronize()
    check(to_host(o).transpose(0, 2, 1, 3), ref, TOL[dtype], "head-major")


def test_inputs_are_not_modified_and_output_is_deterministic():
    w = WORKLOADS["c2"]
    q, k, v = make_inputs(1, w.seq_len, 2, 2, 128, seed=3, dtype="bf16", qk_scale=w.qk_prescale)
    got1, plan, dev = multihop_forward(q, k, v, w.dims, "bf16", True)
    assert np.array_equal(to_host(dev["q"]), q) and np.array_equal(to_host(dev["k"]), k)
    assert np.array_equal(to_host(dev["v"]), v)
    got2, _, _ = multihop_forward(q, k, v, w.dims, "bf16", True)
    assert np.array_equal(got1, got2)


def zero_query_reference(v, dims, G, causal):
    """Q = 0: every attention row is uniform over its allowed keys, so the output is a
    mean of V (non-causal) or a running mean along every axis (causal)."""
    B, N, Hkv, D = v.shape
    x = v.astype(np.float64).reshape((B,) + tuple(dims) + (Hkv, D))
    if not causal:
        ref = np.broadcast_to(x.reshape(B, N, Hkv, D).mean(1, keepdims=True), (B, N, Hkv, D))
    else:
        for ax, n in enumerate(dims):
            x = np.cumsum(x, axis=ax + 1)
            shape = [1] * x.ndim
            shape[ax + 1] = n
            x = x / np.arange(1, n + 1).reshape(shape)
        ref = x.reshape(B, N, Hkv, D)
    return np.repeat(ref, G, axis=2)


# ---- full-size configurations, in the launch configuration the benchmark times ----------

def full_size_case(name, sample_heads):
    w = WORKLOADS[name]
    q, k, v = make_workload_inputs(w, with_grad=False)
    got, plan, _ = multihop_forward(q, k, v, w.dims, w.dtype, w.causal)
    G = w.n_q_heads // w.n_kv_heads
    worst = 0.0
    for h in sample_heads:
        g = h // G
        ref = orc.tensorized_attention_forward(q[:, :, h:h + 1], k[:, :, g:g + 1], v[:, :, g:g + 1],
                                               w.dims, w.causal)
        worst = max(worst, check(got[:, :, h:h + 1], ref, TOL[w.dtype], f"{name} head {h}"))
    assert np.isfinite(got).all()
    return plan, worst


def test_config2_full_size_all_heads():
    plan, worst = full_size_case("c2", range(32))
    assert plan.hop_kernel(0, 0) != "generic"
    print(f"config 2, all heads: max-abs error {worst:.3e}")


def test_config3_full_size_all_heads():
    plan, worst = full_size_case("c3", range(32))
    assert plan.hop_kernel(0, 0) != "generic"
    print(f"config 3, all heads: max-abs error {worst:.3e}")


def test_config4_full_size_all_heads():
    """131,072 tokens as 64 x 64 x 32, every head."""
    plan, worst = full_size_case("c4", range(32))
    assert plan.hop_kernel(0, 0) != "generic"
    print(f"config 4, all heads: max-abs error {worst:.3e}")


def test_extrapolated_128k_shape_full_size_all_heads():
    """128 x 32 x 32: a streamed first hop, then the fused pair; every head."""
    plan, worst = full_size_case("c6", range(32))
    assert plan.hop_kernel(0, 0) == "mfma_bf16_stream_shared_kv" and plan.fused_position() == 1
    print(f"128 x 32 x 32, all heads: max-abs error {worst:.3e}")


@pytest.mark.parametrize("name,causal", [("c3", True), ("c3", False), ("c4", True), ("c6", True)])
def test_zero_queries_closed_form_at_full_size(name, causal):
    """Property that holds at any size and touches every fibre of every head."""
    w = WORKLOADS[name]
    rng = np.random.default_rng(w.seed)
    from paper_2410_20926_amd.workloads import draw
    k = draw((w.batch, w.seq_len, w.n_kv_heads, w.head_dim), rng, w.qk_prescale, "bf16")
    v = draw((w.batch, w.seq_len, w.n_kv_heads, w.head_dim), rng, 1.0, "bf16")
    q = np.zeros((w.batch, w.seq_len, w.n_q_heads, w.head_dim), dtype=np.float32)
    got, _, _ = multihop_forward(q, k, v, w.dims, "bf16", causal)
    ref = zero_query_reference(v, w.dims, w.n_q_heads // w.n_kv_heads, causal)
    check(got, ref, TOL["bf16"], f"{name} Q=0 causal={causal}")


def test_offsets_near_the_32_bit_limit():
    """524,288 tokens of 32 heads x 128 bf16 features: the last row of Q starts 4,294,959,104
    bytes into the batch element, just inside the MFMA kernels' 32-bit row offsets.  Checked
    with the Q = 0 closed form (a running mean along every axis), which touches every fibre."""
    dims, Hq, Hkv, D = (128, 64, 64), 32, 8, 128
    N = int(np.prod(dims))
    rng = np.random.default_rng(99)
    from paper_2410_20926_amd.workloads import draw
    v = draw((1, N, Hkv, D), rng, 1.0, "bf16")
    plan = ta.ta_plan_create(1, Hq, Hkv, D, dims, ta.TA_BF16, True)
    assert [plan.hop_kernel(a, 1) for a in range(3)] == ["mfma_bf16_stream_shared", "mfma_bf16_n64_shared", "mfma_bf16_n64_shared"]
    tq = torch.zeros(1, N, Hq, D, dtype=torch.bfloat16, device="cuda")
    tk = torch.zeros(1, N, Hkv, D, dtype=torch.bfloat16, device="cuda")
    tv = to_dev(v, "bf16")
    o = torch.empty_like(tq)
    wsb = plan.workspace_bytes(False)
    ws = alloc_bytes(wsb)
    ta.ta_multihop_forward(plan, tq, tk, tv, o, ws, wsb, False)
    torch.cuda.synchronize()
    del ws, tq, tk
    ref = zero_query_reference(v, dims, 1, True)                     # per key/value head
    for g in (0, 7):                                                  # first and last group: lowest and highest addresses
        for h in (4 * g, 4 * g + 3):
            got = to_host(o[:, :, h])
            check(got, ref[:, :, g], TOL["bf16"], f"head {h}")
    # one token past this size the offsets no longer fit and the plan falls back
    big = ta.ta_plan_create(1, Hq, Hkv, D, (128, 64, 65), ta.TA_BF16, True)
    assert big.hop_kernel(2, 1) == "generic"


@pytest.mark.parametrize("dims", [(16, 32, 8), (2, 32, 32)])      # every hop on its own; last two hops fused
def test_multihop_forward_under_graph_capture(dims):
    """The library only enqueues kernels on the given stream (no allocation, no memset, no
    synchronisation), so a multi-hop forward can be captured into a HIP graph; every replay,
    with eager work and synchronisations in between, must reproduce the eager result."""
    B, Hq, Hkv, D = 1, 8, 2, 128
    N = int(np.prod(dims))
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, True)
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    q = torch.randn(B, N, Hq, D, device="cuda", generator=gen).bfloat16()
    k = torch.randn(B, N, Hkv, D, device="cuda", generator=gen).bfloat16()
    v = torch.randn(B, N, Hkv, D, device="cuda", generator=gen).bfloat16()
    o = torch.zeros(B, N, Hq, D, device="cuda", dtype=torch.bfloat16)
    wsb = plan.workspace_bytes(False)
    ws = alloc_bytes(wsb)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ta.ta_multihop_forward(plan, q, k, v, o, ws, wsb, False)     # warm-up on the capture stream
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        ta.ta_multihop_forward(plan, q, k, v, o, ws, wsb, False)
    for it in range(3):
        q.copy_(torch.randn(B, N, Hq, D, device="cuda", generator=gen).bfloat16())
        v.copy_(torch.randn(B, N, Hkv, D, device="cuda", generator=gen).bfloat16())
        eager = torch.empty_like(o)
        ws2 = alloc_bytes(wsb)
        ta.ta_multihop_forward(plan, q, k, v, eager, ws2, wsb, False)
        torch.cuda.synchronize()
        o.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, eager), f"replay {it} differs from the eager result"
