"""GPU parity for the fused pair of hops (the two innermost axes, both of length 32, in one
launch): against the float64 oracle's two hops of Eq. 4, and against the library's own two
single-hop launches."""
import numpy as np
import pytest
import torch

import paper_2410_20926_amd as ta
from gpu_util import TOL, multihop_backward, multihop_forward, to_dev, to_host
from grad_bounds import check_backward
from oracle import tensattn_oracle as orc
from paper_2410_20926_amd.workloads import make_inputs, round_to_bf16

pytestmark = pytest.mark.gpu


def oracle_two_hops(q, k, x, dims, axis, causal, window=None, masks=None):
    """Hop along `axis` then along `axis + 1` per (batch, head), value input x with H_q or H_kv heads."""
    B, N, Hq, D = q.shape
    G = Hq // k.shape[2]
    scale = 1.0 / np.sqrt(D)
    window = [0] * len(dims) if window is None else window
    masks = [None] * len(dims) if masks is None else masks
    out = np.empty((B, N, Hq, D))
    for b in range(B):
        for h in range(Hq):
            xh = x[b, :, h if x.shape[2] == Hq else h // G]
            for a in (axis, axis + 1):
                xh = orc.axis_attention(q[b, :, h], k[b, :, h // G], xh, list(dims), a, scale, causal,
                                        window=window[a], mask=masks[a])
            out[b, :, h] = xh
    return out


PAIR_CASES = [
    # dims, B, Hq, Hkv, causal, value input heads ("kv" or "o")
    ((32, 32), 1, 4, 1, True, "kv"),
    ((32, 32), 2, 2, 2, False, "kv"),
    ((3, 32, 32), 1, 8, 2, True, "o"),
    ((2, 32, 32), 1, 3, 3, False, "o"),          # 6 workgroup groups: the last block of 8 is partly empty
    ((5, 32, 32), 1, 16, 2, True, "o"),          # 8 heads per key/value head
    ((2, 2, 32, 32), 1, 4, 2, True, "o"),
    ((3, 32, 32), 1, 14, 2, True, "o"),          # 7 heads per key/value head
]


@pytest.mark.parametrize("dims,B,Hq,Hkv,causal,vin", PAIR_CASES)
def test_pair_matches_oracle_and_the_two_single_hops(dims, B, Hq, Hkv, causal, vin):
    N, D, m = int(np.prod(dims)), 128, len(dims)
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=8000 + N + Hq, dtype="bf16")
    rng = np.random.default_rng(8100 + N)
    x = v if vin == "kv" else round_to_bf16(rng.standard_normal((B, N, Hq, D)).astype(np.float32))
    kind = ta.TA_VIN_KV if vin == "kv" else ta.TA_VIN_O
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, causal)
    assert plan.pair_kernel(m - 2, kind) == "mfma_bf16_pair_n32"
    dq, dk, dx = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(x, "bf16")
    o = torch.full((B, N, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    ta.ta_axis_pair_attn_forward(plan, m - 2, dq, dk, dx, kind, o)
    torch.cuda.synchronize()
    got = to_host(o)
    ref = oracle_two_hops(q, k, x, dims, m - 2, causal)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= TOL["bf16"], f"fused pair vs oracle: max-abs error {err:.3e}"
    # the same two hops as separate launches: equal up to the rounding of the intermediate O
    mid = torch.empty_like(o)
    two = torch.empty_like(o)
    ta.ta_axis_attn_forward(plan, m - 2, dq, dk, dx, kind, mid)
    ta.ta_axis_attn_forward(plan, m - 1, dq, dk, mid, ta.TA_VIN_O, two)
    torch.cuda.synchronize()
    assert np.abs(got - to_host(two)).max() <= TOL["bf16"]
    # with o_mid the launch also hands out the first hop's output, and o_out does not change
    o2 = torch.full_like(o, float("nan"))
    got_mid = torch.full_like(o, float("nan"))
    ta.ta_axis_pair_attn_forward(plan, m - 2, dq, dk, dx, kind, o2, o_mid=got_mid)
    torch.cuda.synchronize()
    assert torch.equal(o2, o)
    assert np.abs(to_host(got_mid) - to_host(mid)).max() <= 2.0 ** -8 * max(1.0, float(np.abs(to_host(mid)).max()))


def test_pair_with_bands_and_tables():
    dims, B, Hq, Hkv, D = (2, 32, 32), 1, 4, 1, 128
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=8200, dtype="bf16")
    rng = np.random.default_rng(8201)
    x = round_to_bf16(rng.standard_normal((B, N, Hq, D)).astype(np.float32))
    t1 = (rng.random((32, 32)) < 0.6) | np.eye(32, dtype=bool)
    t1[7, :] = False                                     # a query position of the outer axis that sees nothing
    t2 = (rng.random((32, 32)) < 0.5) | np.eye(32, dtype=bool)
    dev = [None, torch.from_numpy(ta.pack_axis_mask(t1)).cuda(), torch.from_numpy(ta.pack_axis_mask(t2)).cuda()]
    window = (0, 9, 20)
    for causal in (False, True):
        plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, causal, window=window, axis_masks=dev)
        o = torch.full((B, N, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        ta.ta_axis_pair_attn_forward(plan, 1, to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(x, "bf16"), ta.TA_VIN_O, o)
        torch.cuda.synchronize()
        ref = oracle_two_hops(q, k, x, dims, 1, causal, window=window, masks=[None, t1, t2])
        err = np.abs(to_host(o) - ref).max()
        assert err <= TOL["bf16"], f"causal={causal}: max-abs error {err:.3e}"


def test_multihop_forward_and_backward_with_the_pair():
    dims, B, Hq, Hkv, D = (4, 32, 32), 1, 8, 2, 128
    N = int(np.prod(dims))
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=8300, dtype="bf16", with_grad=True)
    ref = orc.tensorized_attention_forward(q, k, v, dims, True)
    fused, plan, _ = multihop_forward(q, k, v, dims, "bf16", True, save=False)
    assert plan.fused_position() == 1
    assert plan.workspace_bytes(False) == B * N * Hq * D * 2 and plan.workspace_bytes(True) == 2 * B * N * Hq * D * 2
    saved, plan_s, dev = multihop_forward(q, k, v, dims, "bf16", True, save=True)
    assert np.abs(fused - ref).max() <= TOL["bf16"] and np.array_equal(saved, fused)
    # the saving forward wrote both intermediate O tensors: the backward that reads them matches the oracle
    dq, dk, dv = multihop_backward(plan_s, dev, d_o, "bf16")
    check_backward((dq, dk, dv), q, k, v, d_o, dims, True, "bf16")
    # another hop order: the pair is not at the end, every hop runs on its own
    swapped, plan2, _ = multihop_forward(q, k, v, dims, "bf16", True, hop_order=(1, 0, 2))
    assert plan2.fused_position() == -1
    ref2 = orc.tensorized_attention_forward(q, k, v, dims, True, hop_order=(1, 0, 2))
    assert np.abs(swapped - ref2).max() <= TOL["bf16"]


def test_pair_with_sharp_softmax():
    """Logits with a standard deviation of 16: nearly one-hot attention rows, exercising the max subtraction."""
    dims, B, Hq, Hkv, D = (2, 32, 32), 1, 4, 2, 128
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=8500, dtype="bf16", qk_scale=4.0)
    for causal in (False, True):
        got, plan, _ = multihop_forward(q, k, v, dims, "bf16", causal)
        assert plan.fused_position() == 1
        ref = orc.tensorized_attention_forward(q, k, v, dims, causal)
        assert np.isfinite(got).all()
        assert np.abs(got - ref).max() <= TOL["bf16"]


def test_order_two_needs_no_workspace_when_fused():
    dims, B, Hq, Hkv, D = (32, 32), 2, 4, 1, 128
    q, k, v = make_inputs(B, 1024, Hq, Hkv, D, seed=8400, dtype="bf16")
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, False)
    assert plan.fused_position() == 0 and plan.workspace_bytes(False) == 0
    o = torch.full((B, 1024, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    ta.ta_multihop_forward(plan, to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16"), o, None, 0, False)
    torch.cuda.synchronize()
    ref = orc.tensorized_attention_forward(q, k, v, dims, False)
    assert np.abs(to_host(o) - ref).max() <= TOL["bf16"]


@pytest.mark.parametrize("valid_len", [2900, 2048 + 5, 1024, 37])
@pytest.mark.parametrize("causal", [False, True])
def test_pair_with_padding(valid_len, causal):
    """Tokens at or past valid_len are padding: a slab cut in the middle of a row, at a row, a whole
    padded slab, and a sequence of barely more than one row."""
    dims, B, Hq, Hkv, D = (3, 32, 32), 2, 4, 2, 128
    N = int(np.prod(dims))
    q, k, v = make_inputs(B, N, Hq, Hkv, D, seed=8600 + valid_len, dtype="bf16")
    got, plan, _ = multihop_forward(q, k, v, dims, "bf16", causal, valid_len=valid_len)
    assert plan.fused_position() == 1
    ref = orc.tensorized_attention_forward(q, k, v, dims, causal, valid_len=valid_len)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= TOL["bf16"]
    assert (got[:, valid_len:] == 0).all()
    saved, plan_s, dev = multihop_forward(q, k, v, dims, "bf16", causal, save=True, valid_len=valid_len)
    assert np.array_equal(saved, got)
    o_bytes = B * N * Hq * D * 2
    mid = dev["ws"][o_bytes:2 * o_bytes].view(torch.bfloat16).view(B, N, Hq, D)      # the O between the fused hops
    assert (to_host(mid)[:, valid_len:] == 0).all() and np.isfinite(to_host(mid)).all()


@pytest.mark.parametrize("causal,valid_len,Hq,Hkv,D", [(True, None, 8, 2, 64), (False, None, 8, 2, 64), (True, 1500, 8, 2, 64),
                                                     (True, None, 4, 4, 100),      # OpenLLaMA-3B's head width, in 128-wide tiles
                                                     (False, 1900, 8, 2, 96), (True, None, 4, 1, 40)])
def test_pair_at_other_head_widths(causal, valid_len, Hq, Hkv, D):
    dims, B = (2, 32, 32), 2
    N = int(np.prod(dims))
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=8700, dtype="bf16", qk_scale=0.125, with_grad=True)
    kw = {} if valid_len is None else dict(valid_len=valid_len)
    got, plan, _ = multihop_forward(q, k, v, dims, "bf16", causal, **kw)
    # the multi-hop call fuses only where the pair is the faster choice (rows that are whole 64-byte pieces)
    assert plan.fused_position() == (1 if D % 32 == 0 else -1) and plan.pair_kernel(1, ta.TA_VIN_O) == "mfma_bf16_pair_n32"
    ref = orc.tensorized_attention_forward(q, k, v, dims, causal, valid_len=valid_len)
    assert np.isfinite(got).all() and np.abs(got - ref).max() <= TOL["bf16"]
    saved, plan_s, dev = multihop_forward(q, k, v, dims, "bf16", causal, save=True, **kw)
    assert np.array_equal(saved, got)
    # the pair kernel itself at this width, called directly after a first hop of its own
    dq_, dk_, dv_ = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
    first = torch.empty_like(dq_)
    direct = torch.full_like(dq_, float("nan"))
    ta.ta_axis_attn_forward(plan, 0, dq_, dk_, dv_, ta.TA_VIN_KV, first)
    ta.ta_axis_pair_attn_forward(plan, 1, dq_, dk_, first, ta.TA_VIN_O, direct)
    torch.cuda.synchronize()
    assert np.abs(to_host(direct) - ref).max() <= TOL["bf16"]
    dq, dk, dv = multihop_backward(plan_s, dev, d_o, "bf16")
    check_backward((dq, dk, dv), q, k, v, d_o, dims, causal, "bf16", valid_len=valid_len)


@pytest.mark.parametrize("kw", [dict(dims=(32, 16)), dict(dims=(32, 32, 2)),
                                dict(dims=(32, 32), dtype=ta.TA_F32), dict(dims=(32, 32), D=256)])
def test_pair_refuses_what_it_does_not_cover(kw):
    dims = kw.pop("dims")
    D = kw.pop("D", 128)
    dtype = kw.pop("dtype", ta.TA_BF16)
    N = int(np.prod(dims))
    plan = ta.ta_plan_create(1, 2, 2, D, dims, dtype, True, **kw)
    assert plan.fused_position() == -1 and plan.pair_kernel(0, ta.TA_VIN_KV) == "unsupported"
    tdt = torch.float32 if dtype == ta.TA_F32 else torch.bfloat16
    t = [torch.zeros((1, N, 2, D), dtype=tdt, device="cuda") for _ in range(4)]
    with pytest.raises(ta.TaError) as e:
        ta.ta_axis_pair_attn_forward(plan, 0, t[0], t[1], t[2], ta.TA_VIN_KV, t[3])
    assert e.value.name == "TA_ERR_UNSUPPORTED"
