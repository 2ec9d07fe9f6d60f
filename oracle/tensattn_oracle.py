"""CPU oracle for Tensorized Attention (arXiv 2410.20926).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, float64 definition
that the GPU library is checked against.  Only the test-suite, the smoke
check and the benchmark's `cpu_baseline` leg may import it; the product path
never does.  It shares no code with the HIP path and imports nothing from it.

What it implements, in the paper's own order and notation:

* Eq. 1               -- `attention`: vector-space softmax attention.
* Eq. 4               -- `axis_attention`: mode-i flattening, batched
                         softmax(Q_i K_i^T / sqrt(d) o M_i), value update,
                         mode-i folding.
* Algorithm 1         -- `tensorized_attention_forward`: O = V, one hop per
                         tensor axis with the same Q and K, vectorise.
* chain rule of Alg. 1 -- `tensorized_attention_backward` (the paper only says
                         that a backward exists, Sec. 3.2; this is the plain
                         derivative of the forward, hop by hop in reverse).

Readings taken where the paper is silent:
  - the mask "o M" excludes positions (logit -inf), it does not multiply;
  - causal means M_i[a, c] = 1 iff c <= a along every axis;
  - reshape is row-major, first axis slowest (Sec. 4.3: with {32,32,32}, one
    more step on the first axis adds 1,024 tokens);
  - hops run in Algorithm 1's order, first axis first, unless told otherwise;
  - d under the square root is the per-head feature width;
  - grouped-query heads: query head h uses key/value head h // (H_q / H_kv);
  - further per-axis masks M_i (Eq. 3 allows any; Sec. 2.1 mentions sparsity masks): a
    band of width w_i along axis i (key c visible from row a iff |a - c| < w_i, and
    c <= a when causal) and padding (tokens at or past `valid_len` are never attended
    to; their own rows see nothing and come out as zero), and an explicit n_i x n_i
    boolean table per axis (`axis_masks`), shared by the axis's fibres or one per fibre as in
    Eq. 3, all of them intersected; a row left with no visible key comes out as zero.  `valid_len` may also be one length per batch element
    (Eq. 3's M_i is one table per fibre: sequences of different lengths in one batch);
  - tensorized positional encoding inside the hops (Sec. 3.2), `rope_base`: the hop along
    axis i scores with Q and K rotated by their coordinate on that axis (`tensorized_rope`
    with axis = i), so that its attention depends on j_i - k_i; the value path is untouched.

Parity pins (tests/test_oracle_*.py): d=1 against a library attention
routine, row sums, brute-force N x N Kronecker-form operator built with scalar
loops, numpy.kron in the separable regime, Q = 0 closed forms, no-leak
invariant, unit-axis no-ops, finite differences for the backward.
Nothing in the attention functions is "parity unpinned".  `tensorized_rope` is pinned
for its rotary mechanics (a library routine at m = 1, relative-position property, norm and
inverse) but the paper does not say which features get which axis position: that
assignment is a reading, so its parity is "parity unpinned" to that extent.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence

import numpy as np

__all__ = [
    "axis_strides",
    "band_mask",
    "attention",
    "axis_attention",
    "axis_attention_by_fibres",
    "tensorized_attention_forward",
    "tensorized_attention_backward",
    "tensorized_rope",
]


def axis_strides(dims: Sequence[int]) -> list:
    """Token stride of every tensor axis for the row-major reshape of
    Sec. 3.1 / App. C.1: token t = sum_i j_i * stride_i, last axis contiguous."""
    strides = [1] * len(dims)
    for i in range(len(dims) - 2, -1, -1):
        strides[i] = strides[i + 1] * int(dims[i + 1])
    return strides


def _softmax_rows(s: np.ndarray, allowed: Optional[np.ndarray]) -> np.ndarray:
    """Row-wise softmax over the last axis (Eq. 1); positions where `allowed`
    is False are excluded from the normalisation and get probability 0.  A row
    with no allowed position gets all-zero probabilities."""
    if allowed is not None:
        s = np.where(allowed, s, -np.inf)
    mx = np.max(s, axis=-1, keepdims=True)
    mx = np.where(np.isfinite(mx), mx, 0.0)
    e = np.exp(s - mx)
    z = np.sum(e, axis=-1, keepdims=True)
    return e / np.where(z > 0, z, 1.0)


def band_mask(n: int, causal: bool, window: int = 0) -> Optional[np.ndarray]:
    """M_i for one axis: [a, c] True iff key c is visible from row a: c <= a when
    causal, and |a - c| < window when window > 0.  None when nothing is masked."""
    if not causal and window <= 0:
        return None
    a = np.arange(n)[:, None]
    c = np.arange(n)[None, :]
    m = np.ones((n, n), dtype=bool)
    if causal:
        m &= c <= a
    if window > 0:
        m &= np.abs(a - c) < window
    return m


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float,
              causal: bool, window: int = 0) -> np.ndarray:
    """Eq. 1 for one head: A = softmax(q k^T * scale o M), o = A v.
    q, k: [n, D]; v: [n, Dv]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    s = (q @ k.T) * scale
    return _softmax_rows(s, band_mask(q.shape[0], causal, window)) @ v


def axis_attention(q: np.ndarray, k: np.ndarray, o_prev: np.ndarray,
                   dims: Sequence[int], axis: int, scale: float, causal: bool,
                   return_probs: bool = False, window: int = 0, valid_len: Optional[int] = None,
                   mask: Optional[np.ndarray] = None):
    """One hop of Eq. 4 for one head.

    q, k: [N, D]; o_prev: [N, Dv]; N = prod(dims).  Mode-`axis` flattening
    turns each tensor into a batch of N / n_axis fibres of n_axis rows; every
    fibre gets its own n_axis x n_axis row-softmax attention, applied to the
    fibre's rows of o_prev; the result is folded back.  Returns o_new [N, Dv]
    and, on request, A_axis with shape dims[:axis] + dims[axis+1:] + (n, n)
    (batch axes in tensor order, then query index, then key index).
    `window` and `valid_len` add the band and padding masks described above; `mask`
    is an explicit M_i (Eq. 3), True where query row a may attend key c: boolean [n, n], the
    same table for every fibre, or [F, n, n] with F = N / n, one table per fibre, the fibres
    numbered in row-major order of their coordinates on the other axes."""
    dims = [int(n) for n in dims]
    N = int(np.prod(dims)) if dims else 1
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    o_prev = np.asarray(o_prev, dtype=np.float64)
    assert q.shape[0] == N and k.shape[0] == N and o_prev.shape[0] == N
    n = dims[axis]
    # tensorise (reshape) and mode-i flatten: move axis i next to the features
    Qi = np.moveaxis(q.reshape(dims + [q.shape[1]]), axis, -2)      # [..., n, D]
    Ki = np.moveaxis(k.reshape(dims + [k.shape[1]]), axis, -2)
    Oi = np.moveaxis(o_prev.reshape(dims + [o_prev.shape[1]]), axis, -2)
    S = np.matmul(Qi, np.swapaxes(Ki, -1, -2)) * scale                # [..., n, n]
    allowed = band_mask(n, causal, window)
    if valid_len is not None and valid_len < N:
        # a token is real iff its index is below valid_len; a padded token is no key and its own row sees nothing
        real = np.moveaxis((np.arange(N) < valid_len).reshape(dims + [1]), axis, -2)[..., 0]   # [..., n]
        pad = real[..., :, None] & real[..., None, :]
        allowed = pad if allowed is None else (allowed & pad)
    if mask is not None:
        mask = np.asarray(mask, dtype=bool)
        if mask.ndim == 3:                                            # one table per fibre: S's leading axes are the fibres in that order
            assert mask.shape == (N // n, n, n)
            mask = mask.reshape(S.shape)
        else:
            assert mask.shape == (n, n)
        allowed = mask if allowed is None else (allowed & mask)
    A = _softmax_rows(S, allowed)
    Onew = np.matmul(A, Oi)                                           # [..., n, Dv]
    # mode-i folding
    o_new = np.moveaxis(Onew, -2, axis).reshape(N, o_prev.shape[1])
    if return_probs:
        return o_new, A
    return o_new


def axis_attention_by_fibres(q: np.ndarray, k: np.ndarray, o_prev: np.ndarray, dims: Sequence[int], axis: int,
                             scale: float, causal: bool, window: int = 0, valid_len: Optional[int] = None,
                             mask: Optional[np.ndarray] = None) -> np.ndarray:
    """The same hop as `axis_attention`, written fibre by fibre (Eq. 4 read literally: fix every
    coordinate but the one on `axis`, take the n rows of that fibre, attend, put the rows back).
    Slow; the tests hold the batched form above to it."""
    dims = [int(n) for n in dims]
    N = int(np.prod(dims)) if dims else 1
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    o_prev = np.asarray(o_prev, dtype=np.float64)
    n = dims[axis]
    stride = axis_strides(dims)[axis]
    band = band_mask(n, causal, window)
    mask = None if mask is None else np.asarray(mask, dtype=bool)
    o_new = np.empty_like(o_prev)
    seen = np.zeros(N, dtype=bool)
    for t0 in range(N):
        if (t0 // stride) % n != 0:            # not the first token of its fibre
            continue
        rows = t0 + stride * np.arange(n)      # the fibre through t0: same coordinates on every other axis
        ok = band
        if mask is not None:
            # the fibre's number: its coordinates on the other axes read as one row-major index
            table = mask[(t0 // (stride * n)) * stride + t0 % stride] if mask.ndim == 3 else mask
            ok = table if ok is None else (ok & table)
        if valid_len is not None and valid_len < N:
            real = rows < valid_len
            pad = real[:, None] & real[None, :]
            ok = pad if ok is None else (ok & pad)
        A = _softmax_rows((q[rows] @ k[rows].T) * scale, ok)
        o_new[rows] = A @ o_prev[rows]
        seen[rows] = True
    assert seen.all()
    return o_new


def _hop_order(m: int, hop_order: Optional[Sequence[int]]) -> list:
    if hop_order is None:
        return list(range(m))
    order = [int(a) for a in hop_order]
    assert sorted(order) == list(range(m)), "hop_order must be a permutation of the axes"
    return order


def _per_batch(valid_len, B: int) -> list:
    """valid_len as a list of B entries (None = no padding)."""
    if valid_len is None or np.isscalar(valid_len):
        return [valid_len] * B
    out = [int(x) for x in valid_len]
    assert len(out) == B, "one valid_len per batch element"
    return out


def tensorized_attention_forward(q: np.ndarray, k: np.ndarray, v: np.ndarray,
                                 dims: Sequence[int], causal: bool,
                                 scale: Optional[float] = None,
                                 hop_order: Optional[Sequence[int]] = None,
                                 return_intermediates: bool = False,
                                 window: Optional[Sequence[int]] = None,
                                 valid_len=None,
                                 axis_masks: Optional[Sequence[Optional[np.ndarray]]] = None,
                                 rope_base: Optional[float] = None):
    """Algorithm 1.

    q: [B, N, H_q, D]; k, v: [B, N, H_kv, D] (H_q a multiple of H_kv);
    N = prod(dims).  Returns o [B, N, H_q, D] in float64.  With
    `return_intermediates` also returns the list [O_0, O_1, ..., O_m] (O_0 is V
    expanded to H_q heads, O_j the value tensor after the j-th executed hop)
    and the list of attention tensors A per executed hop, each of shape
    [B, H_q] + batch dims + [n, n].
    `valid_len`: None, one length for every batch element, or a sequence of B lengths.
    `rope_base`: None, or the base of the per-axis rotary encoding applied to Q and K inside
    every hop (the hop along axis i uses tensorized_rope(., dims, axis=i, base))."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, N, Hq, D = q.shape
    Hkv = k.shape[2]
    assert k.shape == (B, N, Hkv, D) and v.shape[:3] == (B, N, Hkv)
    assert Hq % Hkv == 0
    dims = [int(n) for n in dims]
    assert int(np.prod(dims)) == N, "prod(dims) must equal the sequence length"
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    order = _hop_order(len(dims), hop_order)
    window = [0] * len(dims) if window is None else [int(x) for x in window]
    axis_masks = [None] * len(dims) if axis_masks is None else list(axis_masks)

    valid_lens = _per_batch(valid_len, B)
    # the Q and K every hop scores with: as given, or rotated by the coordinate on the hop's axis
    q_hop = {axis: q if rope_base is None else tensorized_rope(q, dims, axis, rope_base) for axis in order}
    k_hop = {axis: k if rope_base is None else tensorized_rope(k, dims, axis, rope_base) for axis in order}

    o = np.empty((B, N, Hq, v.shape[3]), dtype=np.float64)
    inter = [np.repeat(v, G, axis=2)] + [np.empty_like(o) for _ in order]
    probs = [None] * len(order)
    for b in range(B):
        valid_len = valid_lens[b]
        for h in range(Hq):
            g = h // G
            oh = v[b, :, g, :]                      # Initialise O = V
            for pos, axis in enumerate(order):
                qh, kh = q_hop[axis][b, :, h, :], k_hop[axis][b, :, g, :]
                if return_intermediates:
                    oh, A = axis_attention(qh, kh, oh, dims, axis, scale, causal, True, window[axis], valid_len, axis_masks[axis])
                    if probs[pos] is None:
                        probs[pos] = np.empty((B, Hq) + A.shape, dtype=np.float64)
                    probs[pos][b, h] = A
                    inter[pos + 1][b, :, h, :] = oh
                else:
                    oh = axis_attention(qh, kh, oh, dims, axis, scale, causal, False, window[axis], valid_len, axis_masks[axis])
            o[b, :, h, :] = oh                      # Vectorise
    if return_intermediates:
        return o, inter, probs
    return o


def tensorized_attention_backward(q: np.ndarray, k: np.ndarray, v: np.ndarray,
                                  d_o: np.ndarray, dims: Sequence[int],
                                  causal: bool, scale: Optional[float] = None,
                                  hop_order: Optional[Sequence[int]] = None,
                                  window: Optional[Sequence[int]] = None,
                                  valid_len=None,
                                  axis_masks: Optional[Sequence[Optional[np.ndarray]]] = None,
                                  trace: Optional[dict] = None,
                                  rope_base: Optional[float] = None):
    """Gradient of L = sum(O * d_o) through Algorithm 1 w.r.t. q, k, v.

    Hops are undone in reverse.  For one hop on one fibre with rows Qs, Ks,
    input rows X (= previous O) and upstream gradient G:
        A      = softmax(Qs Ks^T * scale, mask)
        dX     = A^T G
        dA     = G X^T
        dS     = A o (dA - rowsum(A o dA))
        dQs   += dS Ks * scale ;  dKs += dS^T Qs * scale
    The gradient reaching O_0 is dV; dK and dV of a key/value head are the sums
    over the query heads that share it.  Returns (dq, dk, dv) in float64.
    With `rope_base` the hop scores with rotated Q and K (see the forward): Qs, Ks above are the
    rotated rows, and the hop's dQs, dKs are rotated back (the rotation's transpose is its
    inverse) before they are added to dq, dk.

    `trace`, when a dict is given, receives the separate terms of those sums and changes
    nothing else: "dq_hops"[pos] and "dk_hops"[pos] ([B, N, H_q, D] each, per QUERY head) are
    what the hop executed at position pos adds to dq and dk, "dv_heads" [B, N, H_q, Dv] is the
    gradient reaching O_0 per query head, and "dq_sq", "dk_sq" ([B, N, H_q, D]) are the sums of
    the SQUARES of the individual products dS[a,c] K[c,x] scale and dS[a,c] Q[a,x] scale that
    make up dq and dk over all hops (the tests build error bounds from all of them)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    d_o = np.asarray(d_o, dtype=np.float64)
    B, N, Hq, D = q.shape
    Hkv = k.shape[2]
    G = Hq // Hkv
    dims = [int(n) for n in dims]
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    order = _hop_order(len(dims), hop_order)
    _, inter, probs = tensorized_attention_forward(
        q, k, v, dims, causal, scale, order, return_intermediates=True, window=window, valid_len=valid_len, axis_masks=axis_masks,
        rope_base=rope_base)
    q_hop = {axis: q if rope_base is None else tensorized_rope(q, dims, axis, rope_base) for axis in order}
    k_hop = {axis: k if rope_base is None else tensorized_rope(k, dims, axis, rope_base) for axis in order}

    def unrotate(x, axis):                      # [N, D] gradient w.r.t. rotated rows -> w.r.t. the rows as given
        if rope_base is None:
            return x
        return tensorized_rope(x[None, :, None, :], dims, axis, rope_base, inverse=True)[0, :, 0, :]

    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    if trace is not None:
        trace["dq_hops"] = [np.zeros_like(q) for _ in order]
        trace["dk_hops"] = [np.zeros_like(q) for _ in order]
        trace["dv_heads"] = np.zeros((B, N, Hq, v.shape[3]))
        trace["dq_sq"] = np.zeros_like(q)
        trace["dk_sq"] = np.zeros_like(q)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            grad = d_o[b, :, h, :]
            for pos in range(len(order) - 1, -1, -1):
                axis = order[pos]
                A = probs[pos][b, h]                                   # [..., n, n]
                shape_d = dims + [D]
                shape_v = dims + [v.shape[3]]
                Gi = np.moveaxis(grad.reshape(shape_v), axis, -2)
                Xi = np.moveaxis(inter[pos][b, :, h, :].reshape(shape_v), axis, -2)
                Qi = np.moveaxis(q_hop[axis][b, :, h, :].reshape(shape_d), axis, -2)
                Ki = np.moveaxis(k_hop[axis][b, :, g, :].reshape(shape_d), axis, -2)
                dA = np.matmul(Gi, np.swapaxes(Xi, -1, -2))
                dX = np.matmul(np.swapaxes(A, -1, -2), Gi)
                dS = A * (dA - np.sum(A * dA, axis=-1, keepdims=True))
                dQi = np.matmul(dS, Ki) * scale
                dKi = np.matmul(np.swapaxes(dS, -1, -2), Qi) * scale
                dq_hop = unrotate(np.moveaxis(dQi, -2, axis).reshape(N, D), axis)
                dk_hop = unrotate(np.moveaxis(dKi, -2, axis).reshape(N, D), axis)
                dq[b, :, h, :] += dq_hop
                dk[b, :, g, :] += dk_hop
                if trace is not None:
                    trace["dq_hops"][pos][b, :, h, :] = dq_hop
                    trace["dk_hops"][pos][b, :, h, :] = dk_hop
                    trace["dq_sq"][b, :, h, :] += np.moveaxis(np.matmul(dS ** 2, Ki ** 2) * scale ** 2, -2, axis).reshape(N, D)
                    trace["dk_sq"][b, :, h, :] += np.moveaxis(np.matmul(np.swapaxes(dS, -1, -2) ** 2, Qi ** 2) * scale ** 2, -2, axis).reshape(N, D)
                grad = np.moveaxis(dX, -2, axis).reshape(N, v.shape[3])
            dv[b, :, g, :] += grad
            if trace is not None:
                trace["dv_heads"][b, :, h, :] = grad
    return dq, dk, dv


def tensorized_rope(x: np.ndarray, dims: Sequence[int], axis: int = -1, base: float = 10000.0,
                    inverse: bool = False) -> np.ndarray:
    """Tensorized positional encoding (Sec. 3.2): the position of token t is the vector of
    its tensor coordinates (j_1..j_m), and rotary embedding is applied with per-axis positions.

    The paper gives no formula (its appendix on it is absent), so the mechanics are the
    rotary embedding's own definition - feature pair (2p, 2p+1) of a block of width W is
    rotated by the angle pos * base^(-2p/W) - and the assignment of positions to features is
    this reading:
      axis >= 0 : the whole feature vector (W = D) is rotated with pos = j_axis, the encoding
                  a hop along that axis uses (scores then depend on j_axis - k_axis only);
      axis = -1 : the features are split into m consecutive blocks of W = 2*floor(D/(2m)),
                  block i rotated with pos = j_i; left-over features stay as they are.
    `inverse` rotates by the negative angle (the transpose: what the backward applies).
    x: [B, N, H, D] -> same shape, float64."""
    x = np.asarray(x, dtype=np.float64)
    B, N, H, D = x.shape
    dims = [int(n) for n in dims]
    m = len(dims)
    assert int(np.prod(dims)) == N
    coords = np.stack(np.unravel_index(np.arange(N), dims), axis=1)          # [N, m], row-major reshape
    out = x.copy()

    def rotate(lo, width, pos):
        p = np.arange(width // 2)
        ang = pos[:, None] * base ** (-2.0 * p / width)[None, :]             # [N, width/2]
        if inverse:
            ang = -ang
        c, s = np.cos(ang)[None, :, None, :], np.sin(ang)[None, :, None, :]
        even = x[..., lo:lo + width:2]
        odd = x[..., lo + 1:lo + width:2]
        out[..., lo:lo + width:2] = even * c - odd * s
        out[..., lo + 1:lo + width:2] = even * s + odd * c

    if axis >= 0:
        rotate(0, D - D % 2, coords[:, axis].astype(np.float64))
    else:
        width = 2 * (D // (2 * m))
        for i in range(m):
            rotate(i * width, width, coords[:, i].astype(np.float64))
    return out
