"""Pins for the oracle's tensorized rotary position encoding (no GPU).  The rotary mechanics
are pinned against a library routine (Hugging Face Llama's apply_rotary_pos_emb, after the
fixed permutation between its half-split feature order and the interleaved pairs used here)
and by the properties every rotary encoding has.  Which features take which axis position
is not stated in the paper: that part is a reading ("parity unpinned")."""
import numpy as np
import pytest
import torch

from oracle import tensattn_oracle as orc


def hf_rope(x, positions, base):
    """x [B, N, H, D] with interleaved pairs -> library rotation -> interleaved pairs."""
    from transformers.models.llama.modeling_llama import apply_rotary_pos_emb
    B, N, H, D = x.shape
    perm = np.concatenate([np.arange(0, D, 2), np.arange(1, D, 2)])         # interleaved -> half-split
    inv_freq = base ** (-np.arange(0, D, 2) / D)
    ang = positions[:, None] * inv_freq[None, :]
    emb = np.concatenate([ang, ang], axis=-1)
    cos, sin = torch.from_numpy(np.cos(emb))[None], torch.from_numpy(np.sin(emb))[None]
    t = torch.from_numpy(x[..., perm]).permute(0, 2, 1, 3)                  # [B, H, N, D]
    out, _ = apply_rotary_pos_emb(t, t, cos, sin)
    out = out.permute(0, 2, 1, 3).numpy()
    res = np.empty_like(out)
    res[..., perm] = out
    return res


def test_order1_equals_library_rope():
    rng = np.random.default_rng(61)
    x = rng.standard_normal((2, 19, 3, 16))
    got = orc.tensorized_rope(x, [19], axis=0, base=10000.0)
    np.testing.assert_allclose(got, hf_rope(x, np.arange(19.0), 10000.0), rtol=0, atol=1e-12)
    # with one axis the block-split form is the same thing
    np.testing.assert_allclose(orc.tensorized_rope(x, [19], axis=-1), got, rtol=0, atol=1e-15)


def test_per_axis_form_uses_that_axis_coordinate():
    rng = np.random.default_rng(62)
    dims = (3, 4, 2)
    x = rng.standard_normal((1, 24, 2, 8))
    coords = np.stack(np.unravel_index(np.arange(24), dims), axis=1)
    for ax in range(3):
        got = orc.tensorized_rope(x, dims, axis=ax, base=100.0)
        np.testing.assert_allclose(got, hf_rope(x, coords[:, ax].astype(float), 100.0), rtol=0, atol=1e-12)


def test_block_split_form_rotates_block_i_with_coordinate_i():
    rng = np.random.default_rng(63)
    dims, D = (3, 4, 2), 20                       # blocks of 2*floor(20/6) = 6 features, 2 left over
    x = rng.standard_normal((1, 24, 1, D))
    got = orc.tensorized_rope(x, dims, axis=-1, base=50.0)
    coords = np.stack(np.unravel_index(np.arange(24), dims), axis=1)
    for i in range(3):
        blk = slice(6 * i, 6 * i + 6)
        np.testing.assert_allclose(got[..., blk], hf_rope(x[..., blk], coords[:, i].astype(float), 50.0), atol=1e-12)
    np.testing.assert_array_equal(got[..., 18:], x[..., 18:])


@pytest.mark.parametrize("axis", [-1, 0, 1])
def test_rotation_properties(axis):
    """Norm-preserving, inverse undoes it, and scores depend on coordinate differences only."""
    rng = np.random.default_rng(64)
    dims, D = (4, 5), 12
    q = rng.standard_normal((1, 20, 1, D))
    k = rng.standard_normal((1, 20, 1, D))
    rq, rk = orc.tensorized_rope(q, dims, axis), orc.tensorized_rope(k, dims, axis)
    np.testing.assert_allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), atol=1e-12)
    np.testing.assert_allclose(orc.tensorized_rope(rq, dims, axis, inverse=True), q, atol=1e-12)
    # same content at every token: score(t, u) must be a function of coords(t) - coords(u)
    q1 = np.broadcast_to(q[:, :1], q.shape)
    k1 = np.broadcast_to(k[:, :1], k.shape)
    s = np.einsum("td,ud->tu", orc.tensorized_rope(q1, dims, axis)[0, :, 0], orc.tensorized_rope(k1, dims, axis)[0, :, 0])
    coords = np.stack(np.unravel_index(np.arange(20), dims), axis=1)
    seen = {}
    for t in range(20):
        for u in range(20):
            d = tuple(coords[t] - coords[u]) if axis < 0 else (coords[t, axis] - coords[u, axis],)
            seen.setdefault(d, []).append(s[t, u])
    for vals in seen.values():
        assert np.ptp(vals) < 1e-12


# ---- the encoding inside the hops (tensorized_attention_forward / backward with rope_base) -------------------

def scalar_rotate(x, pos, base):
    """Rotary embedding of one feature vector at integer position `pos`, with scalar arithmetic from the
    definition: pair (2p, 2p+1) turned by pos * base^(-2p/D)."""
    import math
    D = len(x)
    out = list(x)
    for p in range(D // 2):
        ang = pos * base ** (-2.0 * p / D)
        c, s = math.cos(ang), math.sin(ang)
        out[2 * p] = x[2 * p] * c - x[2 * p + 1] * s
        out[2 * p + 1] = x[2 * p] * s + x[2 * p + 1] * c
    return out


@pytest.mark.parametrize("causal", [False, True])
def test_encoded_hops_equal_the_scalar_loop_operator(causal):
    """Algorithm 1 with the hop along axis i scoring with Q, K rotated by the coordinate j_i: the N x N
    operator is the product of the per-hop matrices, each built with scalar loops from its own rotated
    Q and K (tests/bruteforce.py), first hop rightmost."""
    import bruteforce as bf
    dims, D, base = (2, 3, 2), 4, 50.0
    N = 12
    rng = np.random.default_rng(65)
    q, k, v = rng.standard_normal((N, D)), rng.standard_normal((N, D)), rng.standard_normal((N, 3))
    W = None
    for axis in range(3):
        qa = [scalar_rotate(list(q[t]), bf.unravel(t, dims)[axis], base) for t in range(N)]
        ka = [scalar_rotate(list(k[t]), bf.unravel(t, dims)[axis], base) for t in range(N)]
        P = bf.hop_matrix(qa, ka, dims, axis, 0.5, causal)
        W = P if W is None else bf.matmul(P, W)
    got = orc.tensorized_attention_forward(q[None, :, None], k[None, :, None], v[None, :, None], dims, causal, scale=0.5, rope_base=base)
    np.testing.assert_allclose(got[0, :, 0], np.array(W) @ v, rtol=0, atol=1e-12)
    plain = orc.tensorized_attention_forward(q[None, :, None], k[None, :, None], v[None, :, None], dims, causal, scale=0.5)
    assert np.abs(plain - got).max() > 1e-3                     # the encoding does change the result


def test_order1_encoded_attention_equals_library_rope_plus_library_attention():
    rng = np.random.default_rng(66)
    B, N, H, D = 2, 23, 2, 8
    q, k, v = (rng.standard_normal((B, N, H, D)) for _ in range(3))
    got = orc.tensorized_attention_forward(q, k, v, (N,), True, rope_base=10000.0)
    rq, rk = hf_rope(q, np.arange(float(N)), 10000.0), hf_rope(k, np.arange(float(N)), 10000.0)
    t = lambda a: torch.from_numpy(a).permute(0, 2, 1, 3)
    ref = torch.nn.functional.scaled_dot_product_attention(t(rq), t(rk), t(v), is_causal=True).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_encoded_hop_attention_depends_on_coordinate_differences_only():
    """With the same content at every token, the hop along axis i attends by j_i - k_i alone: its
    attention is the same in every fibre, and the logit of (row a, key c) relative to the row's own
    diagonal is one function of a - c for all rows (what a relative encoding along that axis means)."""
    rng = np.random.default_rng(67)
    dims, D = (4, 5), 6
    q = np.broadcast_to(rng.standard_normal(D), (1, 20, 1, D))
    k = np.broadcast_to(rng.standard_normal(D), (1, 20, 1, D))
    v = rng.standard_normal((1, 20, 1, 3))
    _, _, probs = orc.tensorized_attention_forward(q, k, v, dims, False, rope_base=30.0, return_intermediates=True)
    for pos, n in enumerate(dims):
        A = probs[pos][0, 0]                                    # [fibres, n, n]
        np.testing.assert_allclose(A, np.broadcast_to(A[0], A.shape), atol=1e-14)
        logits = np.log(A[0])
        by_offset = {}
        for a in range(n):
            for c in range(n):
                by_offset.setdefault(a - c, []).append(logits[a, c] - logits[a, a])
        assert all(np.ptp(vals) < 1e-12 for vals in by_offset.values())
        assert max(abs(vals[0]) for d, vals in by_offset.items() if d != 0) > 1e-3     # and it is not flat


@pytest.mark.parametrize("dims,causal,Hq,Hkv", [((4, 2, 3), True, 2, 1), ((5, 4), False, 2, 2)])
def test_encoded_backward_matches_finite_differences(dims, causal, Hq, Hkv):
    N, D = int(np.prod(dims)), 8
    rng = np.random.default_rng(68)
    q, k, v, d_o = (rng.standard_normal((1, N, Hq, D)), rng.standard_normal((1, N, Hkv, D)),
                    rng.standard_normal((1, N, Hkv, D)), rng.standard_normal((1, N, Hq, D)))
    dq, dk, dv = orc.tensorized_attention_backward(q, k, v, d_o, dims, causal, rope_base=40.0)

    def loss():
        return float(np.sum(orc.tensorized_attention_forward(q, k, v, dims, causal, rope_base=40.0) * d_o))

    for x, g in ((q, dq), (k, dk), (v, dv)):
        flat = x.reshape(-1)
        for i in rng.choice(x.size, size=10, replace=False):
            old = flat[i]
            flat[i] = old + 1e-5; fp = loss()
            flat[i] = old - 1e-5; fm = loss()
            flat[i] = old
            fd = (fp - fm) / 2e-5
            assert abs(fd - g.reshape(-1)[i]) <= 1e-6 * max(abs(fd), 1e-3), (fd, g.reshape(-1)[i])
    # the trace's per-hop terms add up to the totals
    tr = {}
    orc.tensorized_attention_backward(q, k, v, d_o, dims, causal, rope_base=40.0, trace=tr)
    np.testing.assert_allclose(sum(tr["dq_hops"]), dq, atol=1e-13)
    G = Hq // Hkv
    np.testing.assert_allclose(sum(tr["dk_hops"]).reshape(1, N, Hkv, G, D).sum(3), dk, atol=1e-13)
    np.testing.assert_allclose(tr["dv_heads"].reshape(1, N, Hkv, G, D).sum(3), dv, atol=1e-13)
