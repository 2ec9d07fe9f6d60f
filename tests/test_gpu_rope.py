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
