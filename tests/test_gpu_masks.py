"""GPU parity for the per-axis band mask (window), the padding mask (valid_len) and explicit
per-axis bit tables, forward and backward, across every kernel variant, against the masked
oracle."""
import numpy as np
import pytest
import torch

import paper_2410_20926_amd as ta
from gpu_util import TOL, multihop_backward, multihop_forward, to_host
from oracle import tensattn_oracle as orc
from paper_2410_20926_amd.workloads import make_inputs
from grad_bounds import check_backward

pytestmark = pytest.mark.gpu

CASES = [
    # dims, B, Hq, Hkv, D, causal, dtype, window, valid_len
    ((5, 3, 7), 2, 4, 2, 40, True, "f32", (2, 0, 3), None),            # generic kernels
    ((6, 10), 1, 2, 1, 64, False, "f32", (0, 4), 47),
    ((70,), 1, 2, 2, 64, True, "f32", (9,), 50),
    ((32, 16), 1, 2, 2, 128, True, "bf16", (5, 0), None),              # MFMA, plain variant
    ((16, 32), 2, 2, 1, 128, False, "bf16", (0, 7), 300),
    ((8, 32, 4), 1, 4, 1, 128, True, "bf16", (0, 6, 2), 801),          # MFMA, group-shared variant, packed fibres
    ((32, 32), 1, 8, 2, 64, False, "bf16", (3, 0), 700),
    ((64, 8), 1, 4, 1, 128, True, "bf16", (20, 0), 411),               # two key tiles
    ((48, 6), 1, 2, 2, 128, False, "bf16", (40, 2), None),
    ((200, 3), 1, 4, 1, 128, True, "bf16", (70, 0), 500),              # streaming kernel, band skips key tiles
    ((3, 130), 1, 2, 2, 64, False, "bf16", (0, 33), 333),
    ((100, 4), 1, 4, 1, 128, True, "bf16", (30, 0), 377),              # streaming kernel, all query tiles of a fibre in one workgroup
    ((2, 128), 2, 8, 2, 128, False, "bf16", (0, 40), 250),
    ((96, 2), 1, 4, 1, 64, True, "bf16", (0, 0), 150),
]


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype,window,valid_len", CASES)
def test_masked_forward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype, window, valid_len):
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=3000 + N + D, dtype=dtype)
    kw = dict(window=window)
    if valid_len is not None:
        kw["valid_len"] = valid_len
    got, plan, _ = multihop_forward(q, k, v, dims, dtype, causal, **kw)
    ref = orc.tensorized_attention_forward(q, k, v, dims, causal, window=window, valid_len=valid_len)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= TOL[dtype], f"max-abs error {err:.3e}"
    if valid_len is not None:
        assert (got[:, valid_len:] == 0).all()


BWD_CASES = [c for c in CASES if max(c[0]) <= (70 if c[6] == "f32" else 1024)]   # the generic (fp32) backward holds row statistics of the whole axis in LDS


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype,window,valid_len", BWD_CASES)
def test_masked_backward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype, window, valid_len):
    N = int(np.prod(dims))
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=4000 + N + D, dtype=dtype, with_grad=True)
    kw = dict(window=window)
    if valid_len is not None:
        kw["valid_len"] = valid_len
    _, plan, dev = multihop_forward(q, k, v, dims, dtype, causal, save=True, **kw)
    dq, dk, dv = multihop_backward(plan, dev, d_o, dtype)
    check_backward((dq, dk, dv), q, k, v, d_o, dims, causal, dtype, window=window, valid_len=valid_len)
    if valid_len is not None:
        assert (dq[:, valid_len:] == 0).all() and (dk[:, valid_len:] == 0).all() and (dv[:, valid_len:] == 0).all()


# ---- explicit per-axis tables ----------------------------------------------------------------

TABLE_CASES = [
    # dims, B, Hq, Hkv, D, causal, dtype, axes with a table, window, valid_len
    ((5, 3, 7), 2, 4, 2, 40, True, "f32", (0, 2), None, None),            # generic kernels
    ((6, 40), 1, 2, 1, 64, False, "f32", (1,), (0, 30), 230),             # two-word rows
    ((32, 16), 1, 2, 2, 128, True, "bf16", (0, 1), None, None),           # MFMA, plain variant, packed fibres on axis 1
    ((16, 32), 2, 3, 3, 128, False, "bf16", (1,), (0, 20), 300),
    ((8, 32, 4), 1, 4, 1, 128, True, "bf16", (0, 1, 2), None, 801),       # group-shared variant
    ((32, 32), 1, 8, 2, 64, False, "bf16", (0,), None, None),
    ((64, 8), 1, 4, 1, 128, True, "bf16", (0, 1), None, 411),             # two key tiles, two-word rows
    ((48, 6), 1, 2, 2, 128, False, "bf16", (0,), (40, 0), None),
    ((200, 3), 1, 4, 1, 128, True, "bf16", (0,), None, 500),              # streaming kernel, 7-word rows
    ((3, 130), 1, 2, 2, 64, False, "bf16", (1,), (0, 90), None),
    ((128, 3), 1, 4, 1, 128, True, "bf16", (0,), None, 300),              # streaming kernel, chunked over the query tiles
    ((2, 100), 1, 8, 2, 128, False, "bf16", (1,), (0, 70), None),
    ((2, 32, 32), 1, 4, 1, 128, True, "bf16", (1, 2), (0, 12, 0), 1900),  # the fused pair with tables on both of its axes
    ((4, 32, 8), 1, 24, 2, 100, True, "bf16", (0, 1, 2), None, None),     # head width 100, 12 heads per group, tables everywhere
]


def make_tables(dims, axes, seed):
    """Random tables at 60 % density with the diagonal kept, plus one fully hidden row on the
    first masked axis (its outputs must be zero after that hop)."""
    rng = np.random.default_rng(seed)
    host, dev = [], []
    for i, n in enumerate(dims):
        if i not in axes:
            host.append(None); dev.append(None)
            continue
        m = (rng.random((n, n)) < 0.6) | np.eye(n, dtype=bool)
        if i == axes[0] and n > 2:
            m[n // 2, :] = False
        host.append(m)
        dev.append(torch.from_numpy(ta.pack_axis_mask(m)).cuda())
    return host, dev


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype,axes,window,valid_len", TABLE_CASES)
def test_table_forward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype, axes, window, valid_len):
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=5000 + N + D, dtype=dtype)
    host, dev = make_tables(dims, axes, 5100 + N)
    kw = dict(axis_masks=dev)
    if window is not None:
        kw["window"] = window
    if valid_len is not None:
        kw["valid_len"] = valid_len
    got, plan, _ = multihop_forward(q, k, v, dims, dtype, causal, **kw)
    ref = orc.tensorized_attention_forward(q, k, v, dims, causal, window=window, valid_len=valid_len, axis_masks=host)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= TOL[dtype], f"max-abs error {err:.3e}"


TABLE_BWD_CASES = [c for c in TABLE_CASES if max(c[0]) <= (70 if c[6] == "f32" else 1024)]


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype,axes,window,valid_len", TABLE_BWD_CASES)
def test_table_backward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype, axes, window, valid_len):
    N = int(np.prod(dims))
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=6000 + N + D, dtype=dtype, with_grad=True)
    host, dev = make_tables(dims, axes, 6100 + N)
    kw = dict(axis_masks=dev)
    if window is not None:
        kw["window"] = window
    if valid_len is not None:
        kw["valid_len"] = valid_len
    _, plan, devt = multihop_forward(q, k, v, dims, dtype, causal, save=True, **kw)
    dq, dk, dv = multihop_backward(plan, devt, d_o, dtype)
    check_backward((dq, dk, dv), q, k, v, d_o, dims, causal, dtype, window=window, valid_len=valid_len, axis_masks=host)


def test_table_spelling_causal_is_bit_identical_to_the_causal_flag():
    dims, B, Hq, Hkv, D = (32, 32, 32), 1, 8, 2, 128
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=7000, dtype="bf16")
    tril = [torch.from_numpy(ta.pack_axis_mask(np.tril(np.ones((n, n), dtype=bool)))).cuda() for n in dims]
    a, _, _ = multihop_forward(q, k, v, dims, "bf16", True)
    b, _, _ = multihop_forward(q, k, v, dims, "bf16", False, axis_masks=tril)
    assert np.array_equal(a, b)


# ---- one padding length per batch element ------------------------------------------------------------------------

LENS_CASES = [
    # dims, Hq, Hkv, D, causal, dtype, lengths
    ((5, 7, 3), 4, 2, 64, False, "bf16", [105, 37, 0, 1]),
    ((2, 32, 32), 8, 2, 128, False, "bf16", [2048, 1500, 1024, 31]),      # fused pair: whole slabs of padding, ragged slabs
    ((3, 50), 2, 2, 128, True, "bf16", [150, 149, 51]),                   # two key tiles
    ((130, 3), 4, 1, 128, False, "bf16", [390, 200, 3]),                  # streaming forward, blocked backward
    ((64, 4), 4, 1, 64, False, "bf16", [256, 100]),
    ((4, 2, 3), 2, 1, 8, False, "f32", [24, 5, 0]),                       # generic kernels
    ((5, 37), 4, 1, 40, True, "f32", [185, 90]),
]


@pytest.mark.parametrize("dims,Hq,Hkv,D,causal,dtype,lens", LENS_CASES)
def test_valid_len_per_batch_element(dims, Hq, Hkv, D, causal, dtype, lens):
    N, B = int(np.prod(dims)), len(lens)
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=8800 + N + D, dtype=dtype, with_grad=True)
    tl = torch.tensor(lens, dtype=torch.int64, device="cuda")
    for save in (False, True):
        got, plan, dev = multihop_forward(q, k, v, dims, dtype, causal, save=save, valid_lens=tl)
        ref = orc.tensorized_attention_forward(q, k, v, dims, causal, valid_len=lens)
        assert np.isfinite(got).all() and np.abs(got - ref).max() <= TOL[dtype]
        for b, L in enumerate(lens):
            assert (got[b, L:] == 0).all()
    dq, dk, dv = multihop_backward(plan, dev, d_o, dtype)
    check_backward((dq, dk, dv), q, k, v, d_o, dims, causal, dtype, valid_len=lens)
    for b, L in enumerate(lens):
        assert (dq[b, L:] == 0).all() and (dk[b, L:] == 0).all() and (dv[b, L:] == 0).all()
    # the lengths are read when a kernel runs: the same plan follows a change of the array
    tl.copy_(torch.tensor(lens[::-1], dtype=torch.int64))
    o2 = torch.full_like(dev["o"], float("nan"))
    ta.ta_multihop_forward(plan, dev["q"], dev["k"], dev["v"], o2, dev["ws"], dev["wsb"], True)
    torch.cuda.synchronize()
    ref2 = orc.tensorized_attention_forward(q, k, v, dims, causal, valid_len=lens[::-1])
    assert np.abs(to_host(o2) - ref2).max() <= TOL[dtype]


def test_valid_lens_combine_with_valid_len_and_are_clamped():
    dims, B, Hq, Hkv, D = (6, 16), 3, 2, 1, 64
    N = 96
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=8900, dtype="bf16")
    tl = torch.tensor([1000, -5, 50], dtype=torch.int64, device="cuda")         # beyond N, negative, ordinary
    got, _, _ = multihop_forward(q, k, v, dims, "bf16", False, valid_len=70, valid_lens=tl)
    ref = orc.tensorized_attention_forward(q, k, v, dims, False, valid_len=[70, 0, 50])
    assert np.abs(got - ref).max() <= TOL["bf16"]


# ---- one table per fibre (Eq. 3) ------------------------------------------------------------------

def make_fibre_tables(dims, axes, seed):
    """A random table for every fibre of the masked axes (60 % density, diagonal kept), one row of one
    fibre fully hidden on the first masked axis."""
    rng = np.random.default_rng(seed)
    N = int(np.prod(dims))
    host, dev = [], []
    for i, n in enumerate(dims):
        if i not in axes:
            host.append(None); dev.append(None)
            continue
        m = (rng.random((N // n, n, n)) < 0.6) | np.eye(n, dtype=bool)[None]
        if i == axes[0] and n > 2:
            m[(N // n) // 2, n // 2, :] = False
        host.append(m)
        dev.append(torch.from_numpy(ta.pack_axis_mask(m)).cuda())
    return host, dev


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype,axes,window,valid_len", TABLE_CASES)
def test_fibre_table_forward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype, axes, window, valid_len):
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=5500 + N + D, dtype=dtype)
    host, dev = make_fibre_tables(dims, axes, 5600 + N)
    kw = dict(axis_masks=dev)
    if window is not None:
        kw["window"] = window
    if valid_len is not None:
        kw["valid_len"] = valid_len
    got, plan, _ = multihop_forward(q, k, v, dims, dtype, causal, **kw)
    ref = orc.tensorized_attention_forward(q, k, v, dims, causal, window=window, valid_len=valid_len, axis_masks=host)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= TOL[dtype], f"max-abs error {err:.3e}"
    # the tables do differ between fibres: the first fibre's table for all of them gives another result
    shared = orc.tensorized_attention_forward(q, k, v, dims, causal, window=window, valid_len=valid_len,
                                              axis_masks=[None if m is None else m[0] for m in host])
    assert np.abs(shared - ref).max() > 10 * TOL[dtype]


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,causal,dtype,axes,window,valid_len", TABLE_BWD_CASES)
def test_fibre_table_backward_matches_oracle(dims, B, Hq, Hkv, D, causal, dtype, axes, window, valid_len):
    N = int(np.prod(dims))
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=6500 + N + D, dtype=dtype, with_grad=True)
    host, dev = make_fibre_tables(dims, axes, 6600 + N)
    kw = dict(axis_masks=dev)
    if window is not None:
        kw["window"] = window
    if valid_len is not None:
        kw["valid_len"] = valid_len
    _, plan, devt = multihop_forward(q, k, v, dims, dtype, causal, save=True, **kw)
    dq, dk, dv = multihop_backward(plan, devt, d_o, dtype)
    check_backward((dq, dk, dv), q, k, v, d_o, dims, causal, dtype, window=window, valid_len=valid_len, axis_masks=host)


def test_equal_fibre_tables_are_bit_identical_to_the_shared_table():
    dims, B, Hq, Hkv, D = (64, 32, 32), 1, 8, 2, 128          # two-tile first hop, then the fused pair
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=7100, dtype="bf16")
    rng = np.random.default_rng(7101)
    tables = [(rng.random((n, n)) < 0.7) | np.eye(n, dtype=bool) for n in dims]
    shared = [torch.from_numpy(ta.pack_axis_mask(t)).cuda() for t in tables]
    each = [torch.from_numpy(ta.pack_axis_mask(np.broadcast_to(t, (N // t.shape[0],) + t.shape))).cuda() for t in tables]
    a, _, _ = multihop_forward(q, k, v, dims, "bf16", True, axis_masks=shared)
    b, _, _ = multihop_forward(q, k, v, dims, "bf16", True, axis_masks=each)
    assert np.array_equal(a, b)
