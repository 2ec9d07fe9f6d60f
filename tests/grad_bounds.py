"""Per-element error scales for the backward parity tests.

A gradient element is a sum of products; every bf16 rounding on the GPU path (the attention
weights and dS as matrix-core operands, the saved inter-hop O, the gradient that travels
between hops, the running dQ / dK sums, the final store) perturbs it by at most 2^-8 times the
sum of the ABSOLUTE values of those products.  `gradient_magnitudes` evaluates exactly that
sum with the oracle's own attention matrices: the chain rule of Algorithm 1's hops (the paper
states no backward, Sec. 3.2) with every factor replaced by its absolute value, so that no
cancellation hides the size of the terms.  It is a bound's ingredient, not a reference value."""
import math

import numpy as np

from oracle import tensattn_oracle as orc


def gradient_magnitudes(q, k, v, d_o, dims, causal, scale=None, hop_order=None, **mask_kw):
    """Returns (Mq, Mk, Mv), shaped like (q, k, v): for every element the sum over hops (and
    over the query heads of a group for Mk, Mv) of the absolute values of the terms of
    dS K * scale, dS^T Q * scale and A^T G, with
       |G_prev| <- A^T |G|,   |dA| <- |G| |X|^T,   |dS| <- A o (|dA| + rowsum(A o |dA|))."""
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64); d_o = np.asarray(d_o, dtype=np.float64)
    B, N, Hq, D = q.shape
    Hkv = k.shape[2]
    G = Hq // Hkv
    dims = [int(n) for n in dims]
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    order = list(range(len(dims))) if hop_order is None else [int(a) for a in hop_order]
    _, inter, probs = orc.tensorized_attention_forward(q, k, v, dims, causal, scale, order, return_intermediates=True, **mask_kw)
    Mq, Mk, Mv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    sd, sv = dims + [D], dims + [v.shape[3]]
    for b in range(B):
        for h in range(Hq):
            g = h // G
            ga = np.abs(d_o[b, :, h, :])
            for pos in range(len(order) - 1, -1, -1):
                ax = order[pos]
                A = probs[pos][b, h]
                Gi = np.moveaxis(ga.reshape(sv), ax, -2)
                Xi = np.abs(np.moveaxis(inter[pos][b, :, h, :].reshape(sv), ax, -2))
                Qi = np.abs(np.moveaxis(q[b, :, h, :].reshape(sd), ax, -2))
                Ki = np.abs(np.moveaxis(k[b, :, g, :].reshape(sd), ax, -2))
                dA = np.matmul(Gi, np.swapaxes(Xi, -1, -2))
                dS = A * (dA + np.sum(A * dA, axis=-1, keepdims=True))
                Mq[b, :, h, :] += np.moveaxis(np.matmul(dS, Ki) * scale, -2, ax).reshape(N, D)
                Mk[b, :, g, :] += np.moveaxis(np.matmul(np.swapaxes(dS, -1, -2), Qi) * scale, -2, ax).reshape(N, D)
                ga = np.moveaxis(np.matmul(np.swapaxes(A, -1, -2), Gi), -2, ax).reshape(N, v.shape[3])
            Mv[b, :, g, :] += ga
    return Mq, Mk, Mv
