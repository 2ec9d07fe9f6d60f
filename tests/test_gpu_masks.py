"""GPU parity for the per-axis band mask (window) and the padding mask (valid_len),
forward and backward, across every kernel variant, against the masked oracle."""
import numpy as np
import pytest

from gpu_util import TOL, multihop_backward, multihop_forward
from oracle import tensattn_oracle as orc
from paper_2410_20926_amd.workloads import make_inputs
from test_gpu_backward import check_grad

pytestmark = pytest.mark.gpu

CASES = [
    # dims, B, Hq, Hkv, D, causal, dtype, window, valid_len
    ((5, 3, 7), 2, 4, 2, 40, True, "f32", (2, 0, 3), None),            # generic kernels
    ((6, 10), 1, 2, 1, 64, False, "f32", (0, 4), 47),
    ((70,), 1, 2, 2, 64, True, "f32", (9,), 50),
    ((32, 16), 1, 2, 2, 128, True, "bf16", (5, 0), None),              # MFMA, plain variant
    ((16, 32), 2, 2, 1, 128, False, "bf16", (0, 7), 300),
    ((8, 32, 4), 1, 4, 1, 128, True, "bf16", (0, 6, 2), 801),          # MFMA, group-shared variant, packed fibres
    ((32, 32), 1, 8, 2, 64, False, "bf16", (3, 0), 700),
    ((64, 8), 1, 4, 1, 128, True, "bf16", (20, 0), 411),               # two key tiles
    ((48, 6), 1, 2, 2, 128, False, "bf16", (40, 2), None),
    ((200, 3), 1, 4, 1, 128, True, "bf16", (70, 0), 500),              # streaming kernel, band skips key tiles
    ((3, 130), 1, 2, 2, 64, False, "bf16", (0, 33), 333),
]


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype,window,valid_len", CASES)
def test_masked_forward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype, window, valid_len):
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=3000 + N + D, dtype=dtype)
    kw = dict(window=window)
    if valid_len is not None:
        kw["valid_len"] = valid_len
    got, plan, _ = multihop_forward(q, k, v, dims, dtype, causal, **kw)
    ref = orc.tensorized_attention_forward(q, k, v, dims, causal, window=window, valid_len=valid_len)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= TOL[dtype], f"max-abs error {err:.3e}"
    if valid_len is not None:
        assert (got[:, valid_len:] == 0).all()


BWD_CASES = [c for c in CASES if max(c[0]) <= 70]       # the generic backward holds row statistics of the whole axis in LDS


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype,window,valid_len", BWD_CASES)
def test_masked_backward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype, window, valid_len):
    N = int(np.prod(dims))
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=4000 + N + D, dtype=dtype, with_grad=True)
    kw = dict(window=window)
    if valid_len is not None:
        kw["valid_len"] = valid_len
    _, plan, dev = multihop_forward(q, k, v, dims, dtype, causal, save=True, **kw)
    dq, dk, dv = multihop_backward(plan, dev, d_o, dtype)
    rq, rk, rv = orc.tensorized_attention_backward(q, k, v, d_o, dims, causal, window=window, valid_len=valid_len)
    check_grad(dq, rq, dtype, "dq")
    check_grad(dk, rk, dtype, "dk")
    check_grad(dv, rv, dtype, "dv")
    if valid_len is not None:
        assert (dq[:, valid_len:] == 0).all() and (dk[:, valid_len:] == 0).all() and (dv[:, valid_len:] == 0).all()
