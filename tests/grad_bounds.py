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


HALF_ULP_BF16 = 2.0 ** -8          # largest relative error of one rounding to bfloat16 (8 significant bits)


def backward_reference_and_tolerance(q, k, v, d_o, dims, causal, dtype, launch_heads=None, scale=None, hop_order=None, **mask_kw):
    """The oracle's (dq, dk, dv) and, for each, a per-element tolerance for the HIP path.

    bf16:  tol = 2e-2 + 2^-8 * (R + 2 E).  R sums the absolute values of every quantity that the path
    stores in bf16 on the way to that element:
      dq  its running sum after each processed hop (hops are undone last to first; each adds
          its share to the stored dq and rounds), the last of which is the result itself;
      dk  the same, per launch: a launch covers up to `launch_heads` query heads of a group,
          sums them in fp32, adds the stored dk and rounds (None: what the library does, 8 heads per
          launch, 4 on an axis of 33 to 64 positions when the group is a multiple of 4 above 4 and the
          head width is 64 or 128);
      dv  the group sum per launch, plus (m - 1) times the magnitude sum of the gradient chain
          (gradient_magnitudes), for the m - 1 inter-hop gradients stored in bf16.
    E is the root of the sum of squares of the element's individual products dS K scale (dq) or
    dS Q scale (dk, over the group's heads) over all hops: dS enters the matrix cores rounded to bf16,
    one independent relative error of at most 2^-9 per product, so the sum of those errors has a
    standard deviation below 2^-9 E and 2^-7 E is more than four of them.
    The absolute 2e-2 is the forward's bound and covers what is left (the rounded attention weights
    in dX, the saved inter-hop O).
    fp32:  tol = 1e-5 + 2^-20 * M with M from gradient_magnitudes (fp32 sums of up to n_i * D terms)."""
    trace = {}
    ref = orc.tensorized_attention_backward(q, k, v, d_o, dims, causal, scale, hop_order, trace=trace, **mask_kw)
    Mq, Mk, Mv = gradient_magnitudes(q, k, v, d_o, dims, causal, scale, hop_order, **mask_kw)
    if dtype == "f32":
        return ref, tuple(1e-5 + 2.0 ** -20 * m for m in (Mq, Mk, Mv))
    B, N, Hq, D = np.asarray(q).shape
    Hkv = np.asarray(k).shape[2]
    G = Hq // Hkv
    m = len(dims)
    Rq, Rk, Rv = np.zeros_like(ref[0]), np.zeros_like(ref[1]), (m - 1) * Mv
    Eq = np.sqrt(trace["dq_sq"])
    Ek = np.sqrt(trace["dk_sq"].reshape(B, N, Hkv, G, D).sum(3))
    run_q = np.zeros_like(ref[0])
    run_k = np.zeros_like(ref[1])
    order = list(range(m)) if hop_order is None else [int(a) for a in hop_order]

    def heads_per_launch(pos):
        if launch_heads is not None:
            return launch_heads
        n = int(dims[order[pos]])
        return 4 if (32 < n <= 64 and G > 4 and G % 4 == 0 and D in (64, 128)) else 8

    for pos in range(m - 1, -1, -1):
        run_q = run_q + trace["dq_hops"][pos]
        Rq += np.abs(run_q)
        for base in range(0, G, heads_per_launch(pos)):
            hs = np.arange(base, min(base + heads_per_launch(pos), G))
            run_k = run_k + trace["dk_hops"][pos].reshape(B, N, Hkv, G, D)[:, :, :, hs].sum(3)
            Rk += np.abs(run_k)
    run_v = np.zeros_like(ref[2])
    for base in range(0, G, heads_per_launch(0)):
        hs = np.arange(base, min(base + heads_per_launch(0), G))
        run_v = run_v + trace["dv_heads"].reshape(B, N, Hkv, G, -1)[:, :, :, hs].sum(3)
        Rv = Rv + np.abs(run_v)
    return ref, (2e-2 + HALF_ULP_BF16 * (Rq + 2 * Eq), 2e-2 + HALF_ULP_BF16 * (Rk + 2 * Ek), 2e-2 + HALF_ULP_BF16 * Rv)


def check_gradient(got, ref, tol, what, report=None):
    """Element-wise |got - ref| <= tol; returns (and optionally records) the largest error / tolerance."""
    assert np.isfinite(got).all(), f"{what}: non-finite gradient"
    err = np.abs(got - ref)
    ratio = float((err / tol).max())
    line = (f"{what}: max|err| {err.max():.3e}, max|ref| {np.abs(ref).max():.3e}, "
            f"largest error / tolerance {ratio:.3f}")
    print(line)
    if report is not None:
        report.append(line)
    assert ratio <= 1.0, line
    return ratio


def check_backward(got, q, k, v, d_o, dims, causal, dtype, what="", **oracle_kw):
    """(dq, dk, dv) of the HIP path against the oracle, element by element, to the tolerance above."""
    ref, tol = backward_reference_and_tolerance(q, k, v, d_o, dims, causal, dtype, **oracle_kw)
    return max(check_gradient(g_, r_, t_, f"{what} {name}".strip()) for g_, r_, t_, name in zip(got, ref, tol, ("dq", "dk", "dv")))
