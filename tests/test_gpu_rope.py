"""GPU parity for the tensorized rotary position encoding: ta_rope_apply against the oracle,
both forms (one axis / one feature block per axis), both layouts, fp32 and bf16, in place and
out of place, forward and inverse; and its use for a per-axis-encoded hop."""
import math

import numpy as np
import pytest
import torch

import paper_2410_20926_amd as ta
from gpu_util import TOL, ta_dtype, to_dev, to_host, torch_dtype
from oracle import tensattn_oracle as orc
from paper_2410_20926_amd.workloads import make_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dims,D", [((5, 3, 7), 40), ((32, 16), 128), ((300,), 64)])
def test_rope_matches_oracle(dtype, dims, D):
    B, Hq, Hkv = 2, 4, 2
    N = int(np.prod(dims))
    q, k, _ = make_inputs(B, N, Hq, Hkv, D, seed=71, dtype=dtype)
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta_dtype(dtype), True)
    tol = 1e-5 if dtype == "f32" else TOL["bf16"]
    for which, x in ((0, q), (1, k)):
        tx = to_dev(x, dtype)
        for axis in [-1] + list(range(len(dims))):
            for inverse in (False, True):
                ty = torch.full_like(tx, float("nan"))
                ta.ta_rope_apply(plan, which, axis, tx, ty, base=500.0, inverse=inverse)
                torch.cuda.synchronize()
                ref = orc.tensorized_rope(x, dims, axis, 500.0, inverse)
                err = np.abs(to_host(ty) - ref).max()
                assert err <= tol, f"which {which} axis {axis} inverse {inverse}: {err:.3e}"
        # in place, default base
        ta.ta_rope_apply(plan, which, -1, tx, tx)
        torch.cuda.synchronize()
        assert np.abs(to_host(tx) - orc.tensorized_rope(x, dims, -1)).max() <= tol


def test_hop_with_per_axis_encoding():
    """A hop along axis i on queries and keys encoded with that axis's coordinate: the GPU path
    (encode, then per-axis attention) against the oracle doing the same in float64."""
    dims, B, Hq, Hkv, D = (8, 32), 1, 4, 1, 128
    N = 256
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=72, dtype="bf16")
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, True)
    tq, tk, tv = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
    for axis in (0, 1):
        eq, ek = torch.empty_like(tq), torch.empty_like(tk)
        ta.ta_rope_apply(plan, 0, axis, tq, eq)
        ta.ta_rope_apply(plan, 1, axis, tk, ek)
        o = torch.empty_like(tq)
        ta.ta_axis_attn_forward(plan, axis, eq, ek, tv, ta.TA_VIN_KV, o)
        torch.cuda.synchronize()
        # the oracle consumes the encoded tensors as the device rounded them
        rq, rk = to_host(eq), to_host(ek)
        for h in range(Hq):
            ref = orc.axis_attention(rq[0, :, h], rk[0, :, 0], v[0, :, 0], dims, axis, 1 / math.sqrt(D), True)
            assert np.abs(to_host(o)[0, :, h] - ref).max() <= TOL["bf16"]
        assert np.abs(rq - orc.tensorized_rope(q, dims, axis)).max() <= TOL["bf16"]


# ---- the encoding fused into the hops: plans made with rope_base ------------------------------------------------
# The kernels turn the gathered Q and K rows by their position on the hop's axis between the global load and the
# matrix cores (the backward turns dQ and dK back); the oracle does the same in float64.  Which features take
# which axis is a reading of Sec. 3.2 (the paper gives no formula): parity here is against that reading.

from gpu_util import multihop_backward, multihop_forward
from grad_bounds import check_backward

ROPE_CASES = [
    # dims, B, Hq, Hkv, D, causal, dtype
    ((32, 32), 1, 8, 2, 128, True, "bf16"),          # the two hops fused in one launch (value input V)
    ((3, 32, 32), 2, 4, 1, 128, False, "bf16"),      # a single hop, then the fused pair (value input a previous O)
    ((32, 32), 1, 2, 2, 64, True, "bf16"),           # fused pair at head width 64
    ((2, 32, 32), 1, 4, 4, 100, True, "bf16"),       # fused pair with narrow rows
    ((32, 16), 1, 8, 2, 128, True, "bf16"),          # one tile per fibre, group-shared kernel (K and V shared)
    ((4, 32, 8), 2, 4, 4, 128, True, "bf16"),        # one head per group: the plain one-tile kernel; packed fibres on the last axis
    ((16, 8), 1, 4, 1, 64, False, "bf16"),           # several fibres per tile: positions restart inside a tile
    ((5, 7, 3), 2, 4, 2, 64, True, "bf16"),          # ragged tiles
    ((64, 4), 1, 4, 1, 128, True, "bf16"),           # two key tiles, group-shared
    ((3, 50), 1, 2, 2, 128, False, "bf16"),          # two key tiles, plain, ragged second tile
    ((130, 2), 1, 2, 2, 128, True, "bf16"),          # streaming kernel, one wave per head
    ((128, 4), 1, 4, 1, 128, True, "bf16"),          # streaming, group-shared, a workgroup walks all query tiles
    ((200, 2), 1, 8, 2, 64, False, "bf16"),          # streaming, group-shared, a workgroup per query tile
    ((6, 9), 1, 4, 4, 100, True, "bf16"),            # narrow head width
    ((32, 4, 8), 1, 8, 2, 96, True, "bf16"),
    ((16, 16), 1, 1, 1, 64, False, "f32"),           # generic kernels (double-precision angles)
    ((4, 2, 3), 2, 4, 2, 8, True, "f32"),
    ((5, 37), 1, 4, 1, 40, True, "f32"),
]


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype", ROPE_CASES)
def test_encoded_multihop_forward_and_backward_match_oracle(dims, B, Hq, Hkv, D, causal, dtype):
    N = int(np.prod(dims))
    base = 10000.0 if D >= 64 else 200.0
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=7300 + N + D, dtype=dtype, with_grad=True)
    got, plan, dev = multihop_forward(q, k, v, dims, dtype, causal, save=True, rope_base=base)
    ref = orc.tensorized_attention_forward(q, k, v, dims, causal, rope_base=base)
    plain = orc.tensorized_attention_forward(q, k, v, dims, causal)
    err = np.abs(got - ref).max()
    print(f"encoded forward: max-abs error {err:.3e} (the encoding moves the result by {np.abs(ref - plain).max():.2f})")
    assert np.isfinite(got).all() and err <= TOL[dtype], f"forward: {err:.3e}"
    assert np.abs(ref - plain).max() > 10 * TOL[dtype]   # the case would notice a missing rotation
    grads = multihop_backward(plan, dev, d_o, dtype)
    check_backward(grads, q, k, v, d_o, dims, causal, dtype, rope_base=base)
    if plan.fused_position() >= 0:                       # the inference forward of the same plan does not write the tensor between the fused hops
        inf, _, _ = multihop_forward(q, k, v, dims, dtype, causal, save=False, rope_base=base)
        assert np.array_equal(inf, got)


def test_encoded_hop_equals_standalone_encoding_then_hop():
    """The same hop two ways on the GPU: encoding fused into the hop's gather, and ta_rope_apply followed by
    a plain hop.  Both round the turned rows to bf16 before the matrix cores, so they agree closely."""
    dims, B, Hq, Hkv, D = (8, 32), 1, 4, 1, 128
    N = 256
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=73, dtype="bf16")
    plain = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, True)
    fused = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, True, rope_base=0.0)     # 0 = the default base 10000
    tq, tk, tv = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
    for axis in (0, 1):
        eq, ek = torch.empty_like(tq), torch.empty_like(tk)
        ta.ta_rope_apply(plain, 0, axis, tq, eq)
        ta.ta_rope_apply(plain, 1, axis, tk, ek)
        o1, o2 = torch.empty_like(tq), torch.empty_like(tq)
        ta.ta_axis_attn_forward(plain, axis, eq, ek, tv, ta.TA_VIN_KV, o1)
        ta.ta_axis_attn_forward(fused, axis, tq, tk, tv, ta.TA_VIN_KV, o2)
        torch.cuda.synchronize()
        assert np.abs(to_host(o1) - to_host(o2)).max() <= 1e-2


def test_config3_shape_encoded_full_size_sampled_heads():
    """32 x 32 x 32, 32 / 8 heads, D = 128, causal, with the encoding on: one hop, then the fused pair."""
    from paper_2410_20926_amd.workloads import WORKLOADS, make_workload_inputs
    w = WORKLOADS["c3"]
    q, k, v = make_workload_inputs(w, with_grad=False)
    q, k = q * np.float32(4.0), k * np.float32(4.0)          # exact in bf16; gives the softmax something to do
    got, plan, _ = multihop_forward(q, k, v, w.dims, "bf16", True, rope_base=10000.0)
    assert plan.hop_kernel(0, 0) == "mfma_bf16_n32_shared_kv" and plan.fused_position() == 1
    G = w.n_q_heads // w.n_kv_heads
    for h in (0, 7, 13, 22, 31):
        g = h // G
        ref = orc.tensorized_attention_forward(q[:, :, h:h + 1], k[:, :, g:g + 1], v[:, :, g:g + 1], w.dims, True, rope_base=10000.0)
        err = np.abs(got[:, :, h:h + 1] - ref).max()
        assert err <= TOL["bf16"], f"head {h}: {err:.3e}"


def test_long_encoded_axes_leave_the_matrix_core_kernels():
    assert ta.ta_plan_create(1, 4, 1, 128, (4096, 2), ta.TA_BF16, True, rope_base=1e4).hop_kernel(0, 0) == "mfma_bf16_stream_shared_kv"
    assert ta.ta_plan_create(1, 4, 1, 128, (4097, 2), ta.TA_BF16, True, rope_base=1e4).hop_kernel(0, 0) == "generic"
    assert ta.ta_plan_create(1, 4, 1, 128, (4097, 2), ta.TA_BF16, True).hop_kernel(0, 0) == "mfma_bf16_stream_shared_kv"
