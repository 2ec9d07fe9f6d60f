"""Pins for the CPU oracle's backward (no GPU).  The paper states only that a
backward pass exists (Sec. 3.2), so the oracle's analytic gradient is pinned by
central finite differences of the oracle-independent scalar L = sum(O * dO)
evaluated through the brute-force operator or the forward, by a library autograd
run for d = 1, and by closed forms."""
import math

import numpy as np
import pytest
import torch

import bruteforce as bf
from oracle import tensattn_oracle as orc


def rand_case(seed, B, N, Hq, Hkv, D):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, N, Hq, D)), rng.standard_normal((B, N, Hkv, D)),
            rng.standard_normal((B, N, Hkv, D)), rng.standard_normal((B, N, Hq, D)))


def fd_gradient(f, x, idx_list, eps):
    """Central differences of scalar f at selected flat indices of x."""
    out = []
    flat = x.reshape(-1)
    for i in idx_list:
        old = flat[i]
        flat[i] = old + eps
        fp = f()
        flat[i] = old - eps
        fm = f()
        flat[i] = old
        out.append((fp - fm) / (2 * eps))
    return np.array(out)


@pytest.mark.parametrize("dims,causal,Hq,Hkv,D", [
    ((16, 16), False, 1, 1, 64),          # the fp32 configuration's shape
    ((16, 16), True, 1, 1, 64),
    ((4, 2, 3), True, 2, 2, 8),           # odd order-3 shape
    ((4, 2, 3), False, 4, 2, 8),          # grouped-query heads: dK, dV sum over the group
])
def test_backward_matches_finite_differences(dims, causal, Hq, Hkv, D):
    N = int(np.prod(dims))
    q, k, v, d_o = rand_case(21, 1, N, Hq, Hkv, D)
    dq, dk, dv = orc.tensorized_attention_backward(q, k, v, d_o, dims, causal)

    def loss():
        return float(np.sum(orc.tensorized_attention_forward(q, k, v, dims, causal) * d_o))

    rng = np.random.default_rng(22)
    for x, g in ((q, dq), (k, dk), (v, dv)):
        idx = rng.choice(x.size, size=12, replace=False)
        fd = fd_gradient(loss, x, idx, 1e-5)
        an = g.reshape(-1)[idx]
        denom = np.maximum(np.abs(fd), 1e-3)
        assert np.max(np.abs(fd - an) / denom) < 1e-6, (fd, an)


def test_backward_against_brute_force_operator_loss():
    """Same check with the loss evaluated through the scalar-loop operator W, so the
    differentiated function itself is not the oracle's forward."""
    dims, D = (3, 2, 2), 4
    N = 12
    q, k, v, d_o = rand_case(23, 1, N, 1, 1, D)
    dq, dk, dv = orc.tensorized_attention_backward(q, k, v, d_o, dims, True)

    def loss():
        W = np.array(bf.operator_by_paths(q[0, :, 0].tolist(), k[0, :, 0].tolist(),
                                          list(dims), 0.5, True))
        return float(np.sum((W @ v[0, :, 0]) * d_o[0, :, 0]))

    rng = np.random.default_rng(24)
    for x, g in ((q, dq), (k, dk), (v, dv)):
        idx = rng.choice(x.size, size=8, replace=False)
        fd = fd_gradient(loss, x, idx, 1e-5)
        np.testing.assert_allclose(g.reshape(-1)[idx], fd, rtol=1e-6, atol=1e-8)


@pytest.mark.parametrize("causal", [False, True])
def test_order1_backward_against_library_autograd(causal):
    B, N, H, D = 1, 23, 2, 8
    q, k, v, d_o = rand_case(25, B, N, H, H, D)
    dq, dk, dv = orc.tensorized_attention_backward(q, k, v, d_o, [N], causal)
    tq, tk, tv = (torch.from_numpy(x).permute(0, 2, 1, 3).clone().requires_grad_(True)
                  for x in (q, k, v))
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)
    out.backward(torch.from_numpy(d_o).permute(0, 2, 1, 3))
    for g, t in ((dq, tq), (dk, tk), (dv, tv)):
        np.testing.assert_allclose(g, t.grad.permute(0, 2, 1, 3).numpy(), rtol=0, atol=1e-12)


def test_zero_queries_value_gradient_closed_form():
    """Q = 0, non-causal: O[t] = mean(V) for all t, so dV[u] = mean_t dO[t] for all u,
    and K receives no gradient."""
    dims = (3, 4, 2)
    N = 24
    q, k, v, d_o = rand_case(26, 1, N, 1, 1, 5)
    q[:] = 0.0
    dq, dk, dv = orc.tensorized_attention_backward(q, k, v, d_o, dims, False)
    np.testing.assert_allclose(dv[0, :, 0], np.broadcast_to(d_o[0, :, 0].mean(0), (N, 5)), atol=1e-13)
    np.testing.assert_allclose(dk, 0.0, atol=1e-13)


def test_value_gradient_is_operator_transpose():
    """O is linear in V: dV = W^T dO with the brute-force operator."""
    dims, D = (2, 3, 2), 4
    q, k, v, d_o = rand_case(27, 1, 12, 1, 1, D)
    _, _, dv = orc.tensorized_attention_backward(q, k, v, d_o, dims, True)
    W = np.array(bf.operator_by_products(q[0, :, 0].tolist(), k[0, :, 0].tolist(), list(dims),
                                         1 / math.sqrt(D), True))
    np.testing.assert_allclose(dv[0, :, 0], W.T @ d_o[0, :, 0], rtol=0, atol=1e-12)


def test_shift_invariance_of_keys_gives_zero_sum_query_free_direction():
    """Adding the same vector to every key of a fibre shifts each logit row by a
    constant, which the softmax ignores; hence for d = 1 the gradient w.r.t. K summed
    against q-independent shifts obeys sum_c dS[a, c] = 0, i.e. sum_c dK[c] . w equals
    sum_a (sum_c dS[a,c]) q_a . w * scale = 0 for any w."""
    N, D = 9, 4
    q, k, v, d_o = rand_case(28, 1, N, 1, 1, D)
    q[:] = q[:, :1]                       # identical queries: dK summed over keys vanishes
    _, dk, _ = orc.tensorized_attention_backward(q, k, v, d_o, [N], False)
    np.testing.assert_allclose(dk[0, :, 0].sum(0), 0.0, atol=1e-12)
