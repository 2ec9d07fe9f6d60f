"""Pins for the oracle's additional per-axis masks (band of width w_i, padding past
valid_len, explicit boolean tables M_i): a library attention routine with an explicit mask at d = 1, the scalar-loop
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


# ---- explicit per-axis tables M_i -----------------------------------------------------------

def random_mask(rng, n, density=0.6, keep_diagonal=True):
    m = rng.random((n, n)) < density
    if keep_diagonal:
        m |= np.eye(n, dtype=bool)
    return m


@pytest.mark.parametrize("causal", [False, True])
def test_order1_explicit_mask_against_library(causal):
    N, H, D = 23, 2, 8
    rng = np.random.default_rng(58)
    q, k, v = rand_qkv(59, 1, N, H, H, D)
    m = random_mask(rng, N)
    got = orc.tensorized_attention_forward(q, k, v, [N], causal, axis_masks=[m])
    full = torch.from_numpy(m & (np.tril(np.ones((N, N), dtype=bool)) if causal else True))
    tq, tk, tv = (torch.from_numpy(x).permute(0, 2, 1, 3) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=full).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("dims,causal,masked_axes,valid_len", [
    ((2, 3, 4), False, (1, 2), None),
    ((2, 3, 4), True, (0, 2), None),
    ((3, 4), False, (0, 1), 10),
])
def test_explicit_mask_brute_force_operator(dims, causal, masked_axes, valid_len):
    N, D = int(np.prod(dims)), 5
    rng = np.random.default_rng(60)
    q, k, v = rand_qkv(61, 1, N, 1, 1, D)
    masks = [random_mask(rng, n) if i in masked_axes else None for i, n in enumerate(dims)]
    scale = 1 / math.sqrt(D)
    W = np.array(bf.operator_by_products(q[0, :, 0].tolist(), k[0, :, 0].tolist(), list(dims), scale, causal,
                                         valid_len=valid_len,
                                         axis_masks=[None if m is None else m.tolist() for m in masks]))
    got = orc.tensorized_attention_forward(q, k, v, dims, causal, valid_len=valid_len, axis_masks=masks)[0, :, 0]
    np.testing.assert_allclose(got, W @ v[0, :, 0], rtol=0, atol=1e-12)


def test_explicit_masks_that_spell_causal_and_band_give_the_built_in_results():
    dims = (3, 5, 4)
    q, k, v = rand_qkv(62, 1, 60, 2, 1, 6)
    tril = [np.tril(np.ones((n, n), dtype=bool)) for n in dims]
    np.testing.assert_array_equal(orc.tensorized_attention_forward(q, k, v, dims, False, axis_masks=tril),
                                  orc.tensorized_attention_forward(q, k, v, dims, True))
    window = (2, 0, 3)
    band = [None if w == 0 else np.abs(np.subtract.outer(np.arange(n), np.arange(n))) < w for n, w in zip(dims, window)]
    np.testing.assert_array_equal(orc.tensorized_attention_forward(q, k, v, dims, True, axis_masks=band),
                                  orc.tensorized_attention_forward(q, k, v, dims, True, window=window))


def test_block_diagonal_mask_on_one_axis_is_the_hop_over_the_last_of_two_axes():
    """Attention over a single axis of length n1*n2 with the block-diagonal table
    (blocks of n2) is, by Eq. 4, the hop along the last axis of the (n1, n2) tensor."""
    n1, n2, D = 4, 5, 6
    q, k, v = rand_qkv(63, 1, n1 * n2, 1, 1, D)
    block = np.kron(np.eye(n1, dtype=bool), np.ones((n2, n2), dtype=bool))
    scale = 1 / math.sqrt(D)
    for causal in (False, True):
        one_axis = orc.tensorized_attention_forward(q, k, v, [n1 * n2], causal, axis_masks=[block])
        hop = orc.axis_attention(q[0, :, 0], k[0, :, 0], v[0, :, 0], [n1, n2], 1, scale, causal)
        np.testing.assert_allclose(one_axis[0, :, 0], hop, rtol=0, atol=1e-13)


def test_fully_hidden_row_is_zero_and_gets_no_gradient():
    dims, D = (3, 4), 5
    rng = np.random.default_rng(64)
    q, k, v = rand_qkv(65, 1, 12, 1, 1, D)
    m = np.ones((4, 4), dtype=bool); m[2, :] = False                 # row 2 of the last axis sees nothing
    o = orc.tensorized_attention_forward(q, k, v, dims, False, hop_order=(0, 1), axis_masks=[None, m])
    assert (o[0, 2::4] == 0).all() and (o[0, 0::4] != 0).any()
    d_o = rng.standard_normal(q.shape)
    # with a single axis the hidden row's query takes part in nothing, so its gradient is zero
    dq, dk, dv = orc.tensorized_attention_backward(q[:, :4], k[:, :4], v[:, :4], d_o[:, :4], (4,), False, axis_masks=[m])
    assert (dq[0, 2] == 0).all() and (dq[0, 1] != 0).any()


@pytest.mark.parametrize("causal", [False, True])
def test_explicit_mask_backward_matches_finite_differences(causal):
    dims, D = (3, 4), 5
    rng = np.random.default_rng(66)
    q, k, v = rand_qkv(67, 1, 12, 2, 1, D)
    masks = [random_mask(rng, 3), random_mask(rng, 4, 0.5)]
    d_o = rng.standard_normal(q.shape)
    dq, dk, dv = orc.tensorized_attention_backward(q, k, v, d_o, dims, causal, axis_masks=masks)

    def loss():
        return float(np.sum(orc.tensorized_attention_forward(q, k, v, dims, causal, axis_masks=masks) * d_o))

    for x, g in ((q, dq), (k, dk), (v, dv)):
        flat = x.reshape(-1)
        for i in rng.choice(x.size, size=10, replace=False):
            old = flat[i]
            flat[i] = old + 1e-5; fp = loss()
            flat[i] = old - 1e-5; fm = loss()
            flat[i] = old
            fd = (fp - fm) / 2e-5
            assert abs(fd - g.reshape(-1)[i]) <= 1e-6 * max(1e-3, abs(fd)) + 1e-9


def test_valid_len_per_batch_element():
    """One length per batch element (Eq. 3's M_i is a table per fibre; sequences of different lengths in
    a batch are its everyday case): every batch element behaves as if run alone with its own length,
    checked against the scalar-loop operator, forward and (dV = W^T dO) backward; length 0 = all padding."""
    import bruteforce as bf
    dims, D = (3, 2, 2), 4
    N = 12
    rng = np.random.default_rng(91)
    lens = [12, 7, 0, 1]
    B = len(lens)
    q, k, v, d_o = (rng.standard_normal((B, N, 1, D)) for _ in range(4))
    for causal in (False, True):
        got = orc.tensorized_attention_forward(q, k, v, dims, causal, scale=0.7, valid_len=lens)
        dq, dk, dv = orc.tensorized_attention_backward(q, k, v, d_o, dims, causal, scale=0.7, valid_len=lens)
        for b, L in enumerate(lens):
            W = np.array(bf.operator_by_products(q[b, :, 0].tolist(), k[b, :, 0].tolist(), dims, 0.7, causal, valid_len=L))
            np.testing.assert_allclose(got[b, :, 0], W @ v[b, :, 0], rtol=0, atol=1e-12)
            np.testing.assert_allclose(dv[b, :, 0], W.T @ d_o[b, :, 0], rtol=0, atol=1e-12)
            assert (got[b, L:] == 0).all() and (dq[b, L:] == 0).all() and (dk[b, L:] == 0).all() and (dv[b, L:] == 0).all()
            alone = orc.tensorized_attention_forward(q[b:b + 1], k[b:b + 1], v[b:b + 1], dims, causal, scale=0.7, valid_len=L)
            np.testing.assert_array_equal(alone[0], got[b])


# ---- one table per fibre (Eq. 3: M_i has a separate n_i x n_i table for every fibre) -----------------------------

def _random_fibre_masks(rng, F, n, keep_diagonal=True):
    m = rng.random((F, n, n)) < 0.6
    if keep_diagonal:
        m |= np.eye(n, dtype=bool)[None]
    return m


@pytest.mark.parametrize("causal", [False, True])
def test_per_fibre_tables_equal_the_scalar_loop_operator(causal):
    """Every hop takes its own table per fibre; the N x N operator is the product of the per-hop matrices built
    with scalar loops, each fibre looked up by its coordinates on the other axes."""
    import bruteforce as bf
    dims, D = (2, 3, 2), 4
    N = 12
    rng = np.random.default_rng(81)
    q, k, v = rng.standard_normal((N, D)), rng.standard_normal((N, D)), rng.standard_normal((N, 3))
    masks = [_random_fibre_masks(rng, N // n, n, keep_diagonal=(ax != 1)) for ax, n in enumerate(dims)]   # axis 1 may leave rows empty
    W = None
    for axis in range(3):
        P = bf.hop_matrix(q.tolist(), k.tolist(), dims, axis, 0.5, causal, masks_by_fibre=masks[axis].tolist())
        W = P if W is None else bf.matmul(P, W)
    got = orc.tensorized_attention_forward(q[None, :, None], k[None, :, None], v[None, :, None], dims, causal, scale=0.5,
                                           axis_masks=masks)
    np.testing.assert_allclose(got[0, :, 0], np.array(W) @ v, rtol=0, atol=1e-12)
    shared = orc.tensorized_attention_forward(q[None, :, None], k[None, :, None], v[None, :, None], dims, causal, scale=0.5,
                                              axis_masks=[m[0] for m in masks])
    assert np.abs(shared - got).max() > 1e-3                    # the tables do differ between fibres


def test_equal_tables_in_every_fibre_are_the_shared_table():
    rng = np.random.default_rng(82)
    dims, D = (3, 4, 2), 5
    N = 24
    q, k, v = (rng.standard_normal((1, N, 2, D)) for _ in range(3))
    tables = [rng.random((n, n)) < 0.7 for n in dims]
    a = orc.tensorized_attention_forward(q, k, v, dims, True, axis_masks=tables)
    b = orc.tensorized_attention_forward(q, k, v, dims, True, axis_masks=[np.broadcast_to(t, (N // t.shape[0],) + t.shape) for t in tables])
    np.testing.assert_array_equal(a, b)


def test_per_fibre_tables_from_segment_ids_are_attention_within_segments():
    """Documents packed along the innermost axis: the table of a fibre lets a row see the keys of its own segment.
    Every segment of every fibre then is a plain attention problem of its own (library routine)."""
    import torch
    rng = np.random.default_rng(83)
    dims, D = (3, 8), 6
    N = 24
    q, k, v = rng.standard_normal((N, D)), rng.standard_normal((N, D)), rng.standard_normal((N, D))
    seg = np.sort(rng.integers(0, 3, size=(3, 8)), axis=1)      # segment id of every position of every innermost fibre
    masks = seg[:, :, None] == seg[:, None, :]                  # [3 fibres, 8, 8]
    got = orc.axis_attention(q, k, v, dims, 1, D ** -0.5, True, mask=masks)
    for f in range(3):
        for s_id in np.unique(seg[f]):
            rows = f * 8 + np.nonzero(seg[f] == s_id)[0]
            t = lambda a: torch.from_numpy(a[rows])[None]
            ref = torch.nn.functional.scaled_dot_product_attention(t(q), t(k), t(v), is_causal=True)[0].numpy()
            np.testing.assert_allclose(got[rows], ref, rtol=0, atol=1e-12)


def test_per_fibre_tables_fibre_by_fibre_and_batched_forms_agree():
    rng = np.random.default_rng(84)
    dims, D = (3, 4, 5), 4
    N = 60
    q, k, v = rng.standard_normal((N, D)), rng.standard_normal((N, D)), rng.standard_normal((N, 3))
    for axis, n in enumerate(dims):
        m = _random_fibre_masks(rng, N // n, n)
        a = orc.axis_attention(q, k, v, dims, axis, 0.4, True, window=3, valid_len=50, mask=m)
        b = orc.axis_attention_by_fibres(q, k, v, dims, axis, 0.4, True, window=3, valid_len=50, mask=m)
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_per_fibre_tables_backward_matches_finite_differences():
    rng = np.random.default_rng(85)
    dims, D = (3, 2, 4), 4
    N = 24
    q, k, v, d_o = (rng.standard_normal((1, N, 2, D)), rng.standard_normal((1, N, 1, D)),
                    rng.standard_normal((1, N, 1, D)), rng.standard_normal((1, N, 2, D)))
    masks = [_random_fibre_masks(rng, N // n, n) for n in dims]
    dq, dk, dv = orc.tensorized_attention_backward(q, k, v, d_o, dims, True, axis_masks=masks)

    def loss():
        return float(np.sum(orc.tensorized_attention_forward(q, k, v, dims, True, axis_masks=masks) * d_o))

    for x, g in ((q, dq), (k, dk), (v, dv)):
        flat = x.reshape(-1)
        for i in rng.choice(x.size, size=8, replace=False):
            old = flat[i]
            flat[i] = old + 1e-5; fp = loss()
            flat[i] = old - 1e-5; fm = loss()
            flat[i] = old
            fd = (fp - fm) / 2e-5
            assert abs(fd - g.reshape(-1)[i]) <= 1e-6 * max(abs(fd), 1e-3), (fd, g.reshape(-1)[i])
