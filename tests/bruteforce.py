"""Brute-force constructions of the N x N operator W with o = W v that the
multi-hop process of tensorized attention is equivalent to (abstract and
Sec. 3.3: "Kronecker decomposition of full attention").

Written with scalar Python loops and math.exp only, from the definitions, on
purpose: it must not share structure with the oracle it pins.  Tiny inputs only.
"""
import itertools
import math


def unravel(t, dims):
    """Row-major coordinates of token t (first axis slowest, Sec. 4.3)."""
    coords = []
    for n in reversed(dims):
        coords.append(t % n)
        t //= n
    return tuple(reversed(coords))


def ravel(coords, dims):
    t = 0
    for c, n in zip(coords, dims):
        t = t * n + c
    return t


def fibre_probs(q, k, dims, axis, fixed, scale, causal, window=0, valid_len=None, mask=None):
    """The n x n row-softmax attention of one mode-`axis` fibre (Eq. 4).
    `fixed` gives the coordinates on every axis; its entry at `axis` is ignored.
    q, k: nested lists [N][D].  window > 0: key c is hidden from row a unless
    |a - c| < window; valid_len: tokens at or past it are padding (never a key; their
    own rows see nothing and get all-zero probabilities); mask: nested list [n][n] of
    truth values, key c hidden from row a where mask[a][c] is false."""
    n = dims[axis]
    tok = []
    for a in range(n):
        c = list(fixed)
        c[axis] = a
        tok.append(ravel(c, dims))
    A = [[0.0] * n for _ in range(n)]
    for a in range(n):
        logits = []
        for c in range(n):
            hidden = (causal and c > a) or (window > 0 and abs(a - c) >= window)
            if valid_len is not None and (tok[a] >= valid_len or tok[c] >= valid_len):
                hidden = True
            if mask is not None and not mask[a][c]:
                hidden = True
            if hidden:
                logits.append(None)
                continue
            s = 0.0
            for x, y in zip(q[tok[a]], k[tok[c]]):
                s += x * y
            logits.append(s * scale)
        if all(l is None for l in logits):
            continue                                  # a padded row: all zeros
        mx = max(l for l in logits if l is not None)
        ex = [0.0 if l is None else math.exp(l - mx) for l in logits]
        z = sum(ex)
        for c in range(n):
            A[a][c] = ex[c] / z
    return A


def hop_matrix(q, k, dims, axis, scale, causal, window=0, valid_len=None, mask=None, masks_by_fibre=None):
    """P_axis [N][N]: P[t][u] = A^{(fibre)}[j_axis][k_axis] when tokens t = (j)
    and u = (k) agree on every other axis, else 0.  `masks_by_fibre`: one [n][n] table per
    fibre (Eq. 3), indexed by the fibre's coordinates on the other axes read as a row-major number."""
    N = 1
    for n in dims:
        N *= n
    P = [[0.0] * N for _ in range(N)]
    other = [range(n) if i != axis else range(1) for i, n in enumerate(dims)]
    for fixed in itertools.product(*other):
        if masks_by_fibre is not None:
            number = 0
            for i, n in enumerate(dims):
                if i != axis:
                    number = number * n + fixed[i]
            mask = masks_by_fibre[number]
        A = fibre_probs(q, k, dims, axis, fixed, scale, causal, window, valid_len, mask)
        for a in range(dims[axis]):
            ca = list(fixed)
            ca[axis] = a
            t = ravel(ca, dims)
            for c in range(dims[axis]):
                cc = list(fixed)
                cc[axis] = c
                P[t][ravel(cc, dims)] = A[a][c]
    return P


def matmul(X, Y):
    n, m, p = len(X), len(Y), len(Y[0])
    out = [[0.0] * p for _ in range(n)]
    for i in range(n):
        Xi = X[i]
        for l in range(m):
            x = Xi[l]
            if x == 0.0:
                continue
            Yl = Y[l]
            oi = out[i]
            for j in range(p):
                oi[j] += x * Yl[j]
    return out


def operator_by_products(q, k, dims, scale, causal, order=None, window=None, valid_len=None, axis_masks=None):
    """W = P_{last hop} ... P_{first hop}: the first executed hop is rightmost."""
    order = list(range(len(dims))) if order is None else list(order)
    window = [0] * len(dims) if window is None else list(window)
    axis_masks = [None] * len(dims) if axis_masks is None else list(axis_masks)
    W = None
    for axis in order:
        P = hop_matrix(q, k, dims, axis, scale, causal, window[axis], valid_len, axis_masks[axis])
        W = P if W is None else matmul(P, W)
    return W


def operator_by_paths(q, k, dims, scale, causal):
    """Closed form for Algorithm 1's hop order (axis 0 first): between source
    token k and destination token j there is exactly one multi-hop path, which
    corrects one coordinate per hop,
        (k_0,k_1,..) -> (j_0,k_1,..) -> (j_0,j_1,k_2,..) -> ... -> (j_0,..,j_{m-1}),
    so W[j][k] = prod_i A_i^{(j_0..j_{i-1}; k_{i+1}..k_{m-1})}[j_i][k_i]."""
    m = len(dims)
    N = 1
    for n in dims:
        N *= n
    cache = {}
    W = [[0.0] * N for _ in range(N)]
    for t in range(N):
        j = unravel(t, dims)
        for u in range(N):
            kk = unravel(u, dims)
            w = 1.0
            for i in range(m):
                fixed = tuple(j[:i]) + (0,) + tuple(kk[i + 1:])
                key = (i, fixed)
                if key not in cache:
                    cache[key] = fibre_probs(q, k, dims, i, fixed, scale, causal)
                w *= cache[key][j[i]][kk[i]]
                if w == 0.0:
                    break
            W[t][u] = w
    return W
