"""The torch.autograd wrapper: forward and gradients through `tensorized_attention` against the
oracle (it only allocates and passes pointers; the arithmetic is the library's)."""
import numpy as np
import pytest
import torch

from gpu_util import TOL, to_dev, to_host
from oracle import tensattn_oracle as orc
from paper_2410_20926_amd.autograd import tensorized_attention
from paper_2410_20926_amd.workloads import make_inputs
from grad_bounds import check_backward

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype", [
    ((2, 32, 32), 1, 8, 2, 128, True, "bf16"),        # fused last two hops, saving forward
    ((6, 10), 2, 2, 1, 64, False, "f32"),
])
def test_autograd_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype):
    N = int(np.prod(dims))
    # Q, K scaled as in the benchmark workloads
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=9000 + N, dtype=dtype, qk_scale=1.0 / np.sqrt(D), with_grad=True)
    tq, tk, tv = (to_dev(x, dtype).requires_grad_(True) for x in (q, k, v))
    o = tensorized_attention(tq, tk, tv, dims, causal)
    assert np.abs(to_host(o) - orc.tensorized_attention_forward(q, k, v, dims, causal)).max() <= TOL[dtype]
    o.backward(to_dev(d_o, dtype))
    check_backward((to_host(tq.grad), to_host(tk.grad), to_host(tv.grad)), q, k, v, d_o, dims, causal, dtype)


def test_autograd_without_grad_keeps_nothing():
    dims, B, Hq, Hkv, D = (2, 32, 32), 1, 4, 1, 128
    q, k, v = make_inputs(B, 2048, Hq, Hkv, D, seed=9100, dtype="bf16")
    with torch.no_grad():
        o = tensorized_attention(to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16"), dims)
    assert o.grad_fn is None
    assert np.abs(to_host(o) - orc.tensorized_attention_forward(q, k, v, dims, True)).max() <= TOL["bf16"]
