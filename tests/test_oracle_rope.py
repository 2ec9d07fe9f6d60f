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
