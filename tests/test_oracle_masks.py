"""Pins for the oracle's additional per-axis masks (band of width w_i, padding past
valid_len): a library attention routine with an explicit mask at d = 1, the scalar-loop
brute-force operator, closed forms and invariants (no GPU)."""
import math

import numpy as np
import pytest
import torch

import bruteforce as bf
from oracle import tensattn_oracle as orc


def rand_qkv(seed, B, N, Hq, Hkv, D):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, N, Hq, D)), rng.standard_normal((B, N, Hkv, D)),
            rng.standard_normal((B, N, Hkv, D)))


@pytest.mark.parametrize("causal,window", [(False, 3), (True, 4), (True, 1), (False, 50)])
def test_order1_band_mask_against_library(causal, window):
    N, H, D = 29, 2, 8
    q, k, v = rand_qkv(51, 1, N, H, H, D)
    got = orc.tensorized_attention_forward(q, k, v, [N], causal, window=[window])
    a = torch.arange(N)[:, None]
    c = torch.arange(N)[None, :]
    mask = (a - c).abs() < window
    if causal:
        mask &= c <= a
    tq, tk, tv = (torch.from_numpy(x).permute(0, 2, 1, 3) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("dims,causal,window,valid_len", [
    ((2, 3, 4), False, (0, 2, 3), None),
    ((2, 3, 4), True, (2, 0, 2), None),
    ((3, 4), False, None, 7),
    ((3, 4), True, None, 10),
    ((2, 3, 2), False, (0, 2, 0), 9),
])
def test_masked_brute_force_operator(dims, causal, window, valid_len):
    N, D = int(np.prod(dims)), 5
    q, k, v = rand_qkv(52, 1, N, 1, 1, D)
    scale = 1 / math.sqrt(D)
    W = np.array(bf.operator_by_products(q[0, :, 0].tolist(), k[0, :, 0].tolist(), list(dims), scale, causal,
                                         window=window, valid_len=valid_len))
    got = orc.tensorized_attention_forward(q, k, v, dims, causal, window=window, valid_len=valid_len)[0, :, 0]
    np.testing.assert_allclose(got, W @ v[0, :, 0], rtol=0, atol=1e-12)
    L = N if valid_len is None else valid_len
    np.testing.assert_allclose(W[:L].sum(1), 1.0, atol=1e-12)      # real rows stay stochastic
    assert (W[L:] == 0).all() and (W[:, L:] == 0).all()             # padding neither sees nor is seen


def test_window_one_is_identity_and_wide_window_is_no_window():
    dims = (3, 4, 2)
    q, k, v = rand_qkv(53, 1, 24, 2, 1, 6)
    for causal in (False, True):
        ident = orc.tensorized_attention_forward(q, k, v, dims, causal, window=(1, 1, 1))
        np.testing.assert_allclose(ident, np.repeat(v, 2, axis=2), atol=1e-15)
        wide = orc.tensorized_attention_forward(q, k, v, dims, causal, window=(3, 4, 2))
        np.testing.assert_array_equal(wide, orc.tensorized_attention_forward(q, k, v, dims, causal))


def test_causal_padding_changes_nothing_before_valid_len():
    """With the causal mask no token ever looks ahead, so real tokens give the same output
    with or without the padding mask, whatever the padded rows hold; padded rows give zero."""
    dims, L = (3, 4, 2), 17
    q, k, v = rand_qkv(54, 1, 24, 2, 2, 6)
    full = orc.tensorized_attention_forward(q, k, v, dims, True)
    padded = orc.tensorized_attention_forward(q, k, v, dims, True, valid_len=L)
    np.testing.assert_allclose(padded[:, :L], full[:, :L], rtol=0, atol=1e-14)
    assert (padded[:, L:] == 0).all()


def test_noncausal_padding_with_zero_queries_closed_form():
    """Q = 0, whole trailing rows of the tensor padded: every real token ends as the mean of
    the real values."""
    dims, L = (4, 6), 18                     # rows 0..2 of 4 are real
    _, k, v = rand_qkv(55, 1, 24, 1, 1, 3)
    q = np.zeros_like(k)
    got = orc.tensorized_attention_forward(q, k, v, dims, False, valid_len=L)[0, :, 0]
    np.testing.assert_allclose(got[:L], np.broadcast_to(v[0, :L, 0].mean(0), (L, 3)), atol=1e-13)
    assert (got[L:] == 0).all()
    # and the padded values never matter
    v2 = v.copy(); v2[:, L:] = 1e6
    np.testing.assert_array_equal(orc.tensorized_attention_forward(q, k, v2, dims, False, valid_len=L)[0, :L, 0], got[:L])


@pytest.mark.parametrize("causal,window,valid_len", [(True, (2, 3), None), (False, (0, 2), 9), (True, None, 10)])
def test_masked_backward_matches_finite_differences(causal, window, valid_len):
    dims, D = (3, 4), 5
    rng = np.random.default_rng(56)
    q, k, v = rand_qkv(57, 1, 12, 2, 1, D)
    d_o = rng.standard_normal(q.shape)
    dq, dk, dv = orc.tensorized_attention_backward(q, k, v, d_o, dims, causal, window=window, valid_len=valid_len)

    def loss():
        return float(np.sum(orc.tensorized_attention_forward(q, k, v, dims, causal, window=window,
                                                             valid_len=valid_len) * d_o))

    for x, g in ((q, dq), (k, dk), (v, dv)):
        flat = x.reshape(-1)
        for i in rng.choice(x.size, size=10, replace=False):
            old = flat[i]
            flat[i] = old + 1e-5; fp = loss()
            flat[i] = old - 1e-5; fm = loss()
            flat[i] = old
            fd = (fp - fm) / 2e-5
            assert abs(fd - g.reshape(-1)[i]) <= 1e-6 * max(1e-3, abs(fd)) + 1e-9
    if valid_len is not None:
        assert (dq[:, valid_len:] == 0).all() and (dk[:, valid_len:] == 0).all() and (dv[:, valid_len:] == 0).all()
