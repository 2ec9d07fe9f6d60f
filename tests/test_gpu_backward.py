"""GPU parity, backward: dQ, dK, dV from the HIP path against the oracle's analytic
backward (itself pinned by finite differences on the CPU).

Tolerances are per element (tests/grad_bounds.py).  bf16: 2e-2 + 2^-8 * R, R = the sum of
the absolute values of what the path stores in bf16 on the way to that element (the running
dQ / dK sums after each hop and launch, the inter-hop gradients, the result): 2e-2 is the
forward's bound and 2^-8 the half-ulp of a bf16 rounding.  fp32: 1e-5 + 2^-20 * M, M = the sum
of the absolute values of the element's terms.  Every check prints its largest
error / tolerance."""
import math

import numpy as np
import pytest
import torch

import paper_2410_20926_amd as ta
from gpu_util import multihop_backward, multihop_forward, ta_dtype, to_dev, to_host, torch_dtype
from grad_bounds import backward_reference_and_tolerance, check_gradient
from oracle import tensattn_oracle as orc
from paper_2410_20926_amd.workloads import WORKLOADS, make_inputs, make_workload_inputs

pytestmark = pytest.mark.gpu


CASES = [
    ((16, 16), 1, 1, 1, 64, False, "f32"),          # the fp32 configuration's shape
    ((16, 16), 1, 1, 1, 64, True, "f32"),
    ((4, 2, 3), 2, 4, 2, 8, True, "f32"),
    ((5, 37), 1, 4, 1, 40, True, "f32"),            # two key tiles, ragged, 4 heads per group
    ((70,), 1, 2, 2, 128, False, "f32"),
    ((1, 3, 1), 1, 2, 1, 16, True, "f32"),
    ((3, 20), 1, 2, 1, 256, True, "f32"),
    ((32, 16), 1, 4, 1, 128, True, "bf16"),
    ((16, 32, 4), 2, 4, 2, 128, True, "bf16"),
    ((64, 8), 1, 2, 2, 64, False, "bf16"),           # n = 64: the two-tile kernel, one head per group
    ((64, 4), 1, 4, 1, 128, True, "bf16"),           # the same, causal, a group of 4 heads (dK, dV summed over it)
    ((3, 50), 2, 2, 1, 128, True, "bf16"),           # ragged second tile, 2 heads per group
    ((64, 64, 2), 1, 8, 2, 128, True, "bf16"),       # two hops on 64-long axes: as the value-input hop and as a later hop, dQ / dK accumulate
    ((33, 3), 2, 4, 1, 64, False, "bf16"),           # one row in the second tile
    ((2, 64), 1, 4, 4, 128, False, "bf16"),          # full second tile, non-causal: all four blocks
    ((48, 2), 1, 16, 2, 128, True, "bf16"),          # 8 heads per group on a two-tile axis: the two-tile kernel, two launches of 4 heads
    ((40, 3), 1, 12, 1, 64, True, "bf16"),           # 12 heads per group, width 64: three launches, the later ones add to dK and dV
    ((100, 2), 1, 8, 1, 128, False, "bf16"),         # four tiles, 8 heads per group
    ((2, 200), 1, 4, 2, 64, True, "bf16"),           # seven tiles
    ((333,), 1, 2, 2, 128, True, "bf16"),            # one long axis: plain causal attention, 11 tiles
    ((1024, 2), 1, 4, 1, 128, True, "bf16"),         # the longest axis the blocked kernel takes (more than 64 KB of LDS)
    ((3, 16, 8), 1, 2, 1, 128, True, "bf16"),        # packed fibres (2 and 4 per tile), 2 heads per group
    ((5, 7, 3), 2, 4, 4, 64, True, "bf16"),          # odd lengths: ragged tiles with padding rows
    ((32, 3), 1, 8, 2, 128, False, "bf16"),
    ((6, 32), 1, 8, 1, 64, True, "bf16"),            # 8 heads per group: workgroups of 8 waves
    ((4, 16), 1, 16, 1, 128, True, "bf16"),          # 16 heads per group: two launches of 8 heads, the second adds to dK, dV
    ((8, 32), 2, 32, 1, 64, True, "bf16"),           # multi-query: 32 heads on one key/value head, four launches
    ((64, 4), 1, 16, 1, 128, False, "bf16"),         # 16 heads per group on a two-tile axis: four launches of 4 heads
    ((66, 2), 1, 16, 1, 128, False, "bf16"),         # the blocked kernel with 16 heads per group
    ((6, 5), 1, 12, 1, 64, True, "bf16"),            # 12 heads per group: a launch of 8 and one of 4
    ((8, 16), 1, 7, 1, 128, True, "bf16"),           # 7 heads per group (28 query / 4 key-value heads is a real geometry)
    ((5, 40), 2, 6, 2, 128, False, "bf16"),          # 3 heads per group, blocked kernel on the second axis
    ((6, 9), 1, 4, 4, 100, True, "bf16"),            # head width 100: 8-byte-granular rows in 128-wide tiles
    ((32, 4, 8), 2, 8, 2, 96, True, "bf16"),         # width 96, groups of 4 heads, three hops (dQ, dK accumulate)
    ((16, 32), 1, 2, 2, 40, False, "bf16"),          # width 40 in 64-wide tiles
    ((40, 3), 1, 2, 2, 100, True, "bf16"),           # width 100 on an axis of two tiles: the blocked kernel
    ((3, 90), 1, 4, 1, 96, False, "bf16"),           # width 96, three tiles, a group of 4 heads
    ((32, 8), 2, 16, 2, 128, False, "bf16"),         # 8 heads per group, full-width heads
]


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype", CASES)
def test_multihop_backward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype):
    N = int(np.prod(dims))
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=2000 + N + D, dtype=dtype, with_grad=True)
    _, plan, dev = multihop_forward(q, k, v, dims, dtype, causal, save=True)
    got = multihop_backward(plan, dev, d_o, dtype)
    ref, tol = backward_reference_and_tolerance(q, k, v, d_o, dims, causal, dtype)
    for g_, r_, t_, name in zip(got, ref, tol, ("dq", "dk", "dv")):
        check_gradient(g_, r_, t_, name)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_axis_backward_single_hop_and_accumulate(dtype):
    """ta_axis_attn_backward alone: one hop with an O-layout value input, overwrite then
    accumulate."""
    dims, B, Hq, Hkv, D = (6, 16), 1, 4, 2, 64
    N = 96
    q, k, v, g = make_inputs(B, N, Hq, Hkv, D, seed=31, dtype=dtype, with_grad=True)
    x = make_inputs(B, N, Hq, Hq, D, seed=32, dtype=dtype)[2]
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta_dtype(dtype), True)
    tq, tk, tx, tg = (to_dev(a, dtype) for a in (q, k, x, g))
    dx = torch.full_like(tx, float("nan"))
    dq = torch.full_like(tq, float("nan"))
    dk = torch.full_like(tk, float("nan"))
    axis = 1
    ta.ta_axis_attn_backward(plan, axis, tq, tk, tx, ta.TA_VIN_O, tg, dx, dq, dk, False)
    torch.cuda.synchronize()
    # oracle for a single hop along the contiguous axis: its fibres are the batch elements of an
    # order-1 problem (plain attention on n rows), one query head at a time with its key/value head
    # and its own value input
    n = dims[axis]
    F = N // n
    rq = np.zeros_like(q, dtype=np.float64); rk = np.zeros_like(k, dtype=np.float64); rx = np.zeros_like(x, dtype=np.float64)
    tq_, tk_, tx_ = np.zeros_like(rq), np.zeros_like(rk), np.zeros_like(rx)
    fib = lambda a: a.reshape(B * F, n, 1, D)
    for h in range(Hq):
        gk = h // 2
        (a, bk, c), (ta_, tb_, tc_) = backward_reference_and_tolerance(fib(q[:, :, h]), fib(k[:, :, gk]), fib(x[:, :, h]), fib(g[:, :, h]),
                                                                       (n,), True, dtype)
        rq[:, :, h] = a.reshape(B, N, D); tq_[:, :, h] = ta_.reshape(B, N, D)
        rx[:, :, h] = c.reshape(B, N, D); tx_[:, :, h] = tc_.reshape(B, N, D)
        rk[:, :, gk] += bk.reshape(B, N, D); tk_[:, :, gk] += tb_.reshape(B, N, D)      # the sum of the bounds bounds the sum
    for got, ref, tol, name in ((dq, rq, tq_, "dq"), (dk, rk, tk_, "dk"), (dx, rx, tx_, "dx")):
        check_gradient(to_host(got), ref, tol, name)
    ta.ta_axis_attn_backward(plan, axis, tq, tk, tx, ta.TA_VIN_O, tg, dx, dq, dk, True)
    torch.cuda.synchronize()
    # accumulated once more: the stored value was rounded, then the doubled value is
    check_gradient(to_host(dq), 2 * rq, 3 * tq_, "dq accumulated")
    check_gradient(to_host(dk), 2 * rk, 3 * tk_, "dk accumulated")


def test_config5_shape_all_groups():
    """B=2, 32/8 heads, D=128, 32x32x32 causal, forward + backward at full size, every key/value
    group (dK, dV sum over a group's 4 query heads), every element."""
    w = WORKLOADS["c5"]
    q, k, v, d_o = make_workload_inputs(w)
    _, plan, dev = multihop_forward(q, k, v, w.dims, w.dtype, w.causal, save=True)
    assert plan.hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_n32"
    assert plan.hop_backward_kernel(2, ta.TA_VIN_O) == "mfma_bf16_bwd_n32"
    dq, dk, dv = multihop_backward(plan, dev, d_o, w.dtype)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    G = w.n_q_heads // w.n_kv_heads
    worst = 0.0
    for g in range(w.n_kv_heads):
        hs = slice(g * G, (g + 1) * G)
        ref, tol = backward_reference_and_tolerance(q[:, :, hs], k[:, :, g:g + 1], v[:, :, g:g + 1], d_o[:, :, hs],
                                                    w.dims, w.causal, w.dtype)
        for got, r_, t_, name in zip((dq[:, :, hs], dk[:, :, g:g + 1], dv[:, :, g:g + 1]), ref, tol, ("dq", "dk", "dv")):
            worst = max(worst, check_gradient(got, r_, t_, f"{name} group {g}"))
    print(f"config 5: largest error / tolerance over all groups {worst:.3f}")


def test_width_100_training_step_full_size():
    """32 ungrouped heads of width 100 (rows of 200 bytes: neither 16-byte aligned nor whole cache lines), 32x32x32 causal,
    forward + backward at full size, in the launch configuration the bench times (workgroups renumbered per XCD, the hops
    on their own): the forward on every head, the gradients on heads 0 and 1 (an aligned and a misaligned row start),
    17 and 31, every element."""
    w = WORKLOADS["c3_w100_train"]
    q, k, v, d_o = make_workload_inputs(w)
    o, plan, dev = multihop_forward(q, k, v, w.dims, w.dtype, w.causal, save=True)
    assert plan.fused_position() == -1 and plan.hop_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_n32"
    assert plan.hop_backward_kernel(1, ta.TA_VIN_O) == "mfma_bf16_bwd_n32"
    ref_o = orc.tensorized_attention_forward(q, k, v, w.dims, w.causal)
    err = float(np.abs(o - ref_o).max())
    assert np.isfinite(o).all() and err <= 2e-2, f"forward: max-abs error {err:.3e}"
    dq, dk, dv = multihop_backward(plan, dev, d_o, w.dtype)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    worst = 0.0
    for h in (0, 1, 17, 31):
        hs = slice(h, h + 1)
        ref, tol = backward_reference_and_tolerance(q[:, :, hs], k[:, :, hs], v[:, :, hs], d_o[:, :, hs], w.dims, w.causal, w.dtype)
        for got, r_, t_, name in zip((dq[:, :, hs], dk[:, :, hs], dv[:, :, hs]), ref, tol, ("dq", "dk", "dv")):
            worst = max(worst, check_gradient(got, r_, t_, f"{name} head {h}"))
    print(f"width 100: forward max-abs error {err:.3e}; largest gradient error / tolerance {worst:.3f}")


def test_training_step_at_131072_tokens_three_groups():
    """32/8 heads, D=128, 64x64x32 causal, forward + backward at full size: the two-tile backward on both 64-long
    axes (once as the hop that emits dV), the one-tile backward on the innermost one; key/value groups 0, 3 and 7,
    every element."""
    w = WORKLOADS["c4_train"]
    q, k, v, d_o = make_workload_inputs(w)
    _, plan, dev = multihop_forward(q, k, v, w.dims, w.dtype, w.causal, save=True)
    assert plan.hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_n64"
    assert plan.hop_backward_kernel(1, ta.TA_VIN_O) == "mfma_bf16_bwd_n64"
    assert plan.hop_backward_kernel(2, ta.TA_VIN_O) == "mfma_bf16_bwd_n32"
    dq, dk, dv = multihop_backward(plan, dev, d_o, w.dtype)
    assert np.isfinite(dq).all() and np.isfinite(dk).all() and np.isfinite(dv).all()
    G = w.n_q_heads // w.n_kv_heads
    worst = 0.0
    for g in (0, 3, 7):
        hs = slice(g * G, (g + 1) * G)
        ref, tol = backward_reference_and_tolerance(q[:, :, hs], k[:, :, g:g + 1], v[:, :, g:g + 1], d_o[:, :, hs],
                                                    w.dims, w.causal, w.dtype)
        for got, r_, t_, name in zip((dq[:, :, hs], dk[:, :, g:g + 1], dv[:, :, g:g + 1]), ref, tol, ("dq", "dk", "dv")):
            worst = max(worst, check_gradient(got, r_, t_, f"{name} group {g}"))
    print(f"64x64x32 training step: largest error / tolerance over three groups {worst:.3f}")


def test_backward_is_deterministic_and_leaves_inputs_alone():
    """No atomics anywhere: two runs give bit-identical gradients; q, k, v, dO are untouched."""
    dims, B, Hq, Hkv, D = (8, 32, 16), 1, 8, 2, 128
    N = int(np.prod(dims))
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=41, dtype="bf16", with_grad=True)
    _, plan, dev = multihop_forward(q, k, v, dims, "bf16", True, save=True)
    a = multihop_backward(plan, dev, d_o, "bf16")
    b = multihop_backward(plan, dev, d_o, "bf16")
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    assert np.array_equal(to_host(dev["q"]), q) and np.array_equal(to_host(dev["k"]), k)
    assert np.array_equal(to_host(dev["v"]), v)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_strided_head_major_layout(dtype):
    """Every tensor stored [B, H, N, D]; gradients must match the oracle as in the dense case."""
    B, Hq, Hkv, D, dims = 2, 4, 2, 64, (6, 32)
    N = 192
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=43, dtype=dtype, with_grad=True)
    (rq, rk, rv), (tq_, tk_, tv_) = backward_reference_and_tolerance(q, k, v, d_o, dims, True, dtype)
    sq = (Hq * N * D, D, N * D)
    skv = (Hkv * N * D, D, N * D)
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta_dtype(dtype), True, q_strides=sq, kv_strides=skv, o_strides=sq)
    hm = lambda a: to_dev(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), dtype)
    tq, tk, tv, tg = hm(q), hm(k), hm(v), hm(d_o)
    o = torch.empty_like(tq)
    wsb = plan.workspace_bytes(True)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    ta.ta_multihop_forward(plan, tq, tk, tv, o, ws, wsb, True)
    dq, dk, dv = torch.full_like(tq, float("nan")), torch.full_like(tk, float("nan")), torch.full_like(tv, float("nan"))
    scb = plan.backward_scratch_bytes()
    sc = torch.empty(max(scb, 256), dtype=torch.uint8, device="cuda")
    ta.ta_multihop_backward(plan, tq, tk, tv, tg, ws, wsb, dq, dk, dv, sc, scb)
    torch.cuda.synchronize()
    for got, ref, tol, name in ((dq, rq, tq_, "dq"), (dk, rk, tk_, "dk"), (dv, rv, tv_, "dv")):
        check_gradient(to_host(got).transpose(0, 2, 1, 3), ref, tol, name)


def test_backward_kernel_choice_for_axes_longer_than_one_tile():
    plan = ta.ta_plan_create(1, 32, 8, 128, (64, 64, 32), ta.TA_BF16, True)
    assert plan.hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_n64"
    assert plan.hop_backward_kernel(1, ta.TA_VIN_O) == "mfma_bf16_bwd_n64"
    assert plan.hop_backward_kernel(2, ta.TA_VIN_O) == "mfma_bf16_bwd_n32"
    assert ta.ta_plan_create(1, 32, 4, 128, (64, 4), ta.TA_BF16, True).hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_n64"       # 8 heads per group: 4 per launch
    assert ta.ta_plan_create(1, 24, 4, 128, (64, 4), ta.TA_BF16, True).hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_blocked"   # 6 heads per group
    assert ta.ta_plan_create(1, 8, 2, 128, (65, 4), ta.TA_BF16, True).hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_blocked"    # three tiles
    long_axis = ta.ta_plan_create(1, 8, 2, 128, (1024, 4), ta.TA_BF16, True)
    assert long_axis.hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_blocked"
    too_long = ta.ta_plan_create(1, 8, 2, 128, (2048, 2), ta.TA_BF16, True)
    assert too_long.hop_backward_kernel(0, ta.TA_VIN_KV) == "unsupported"


def test_backward_reports_unsupported_shapes():
    """An axis whose row statistics do not fit the generic kernel's LDS budget is refused, not mis-computed."""
    plan = ta.ta_plan_create(1, 8, 1, 64, (4096, 2), ta.TA_F32, True)
    assert plan.hop_backward_kernel(0, ta.TA_VIN_KV) == "unsupported"
    assert plan.hop_backward_kernel(1, ta.TA_VIN_O) == "generic"
    t = torch.zeros(1, 8192, 8, 64, device="cuda")
    tk = torch.zeros(1, 8192, 1, 64, device="cuda")
    with pytest.raises(ta.TaError) as ei:
        ta.ta_axis_attn_backward(plan, 0, t, tk, tk, ta.TA_VIN_KV, t.clone(), tk.clone(), t.clone(), tk.clone(), False)
    assert ei.value.name == "TA_ERR_UNSUPPORTED"
