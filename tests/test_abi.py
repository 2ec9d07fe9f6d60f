"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and its host logic (plan, cost model, error paths) behaves as documented.
No kernel is launched here."""
import ctypes as C
import json
import os
import re

import numpy as np
import pytest

import paper_2410_20926_amd as ta
from paper_2410_20926_amd import tensattn as binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tensattn.h")
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_facts.json")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ta_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ta.load_library()
    names = declared_symbols()
    assert len(names) >= 21
    for name in names:
        assert hasattr(lib, name), f"{name} declared in tensattn.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_version_and_status_strings():
    assert ta.ta_version() == (0, 4)
    lib = ta.load_library()
    assert lib.ta_status_string(0) == b"TA_OK"
    assert lib.ta_status_string(5) == b"TA_ERR_ALIAS"


def test_plan_reshape_convention_matches_paper():
    fact = json.load(open(GOLDEN))["extrapolation_first_axis"]
    p = ta.ta_plan_create(1, 32, 8, 128, fact["dims"], ta.TA_BF16, True)
    assert p.seq_len() == fact["seq_len"]
    assert p.axis_stride(0) == fact["first_axis_increment_tokens"]
    assert [p.axis_stride(i) for i in range(3)] == [1024, 32, 1]
    assert [p.axis_fibres(i) for i in range(3)] == [1024, 1024, 1024]
    assert [p.hop_axis(i) for i in range(3)] == [0, 1, 2]          # Algorithm 1's order
    p = ta.ta_plan_create(1, 32, 8, 128, (64, 64, 32), ta.TA_BF16, True)
    assert [p.axis_stride(i) for i in range(3)] == [2048, 32, 1]
    assert [p.axis_fibres(i) for i in range(3)] == [2048, 2048, 4096]
    p = ta.ta_plan_create(1, 2, 2, 64, (4, 3), ta.TA_F32, False, hop_order=(1, 0))
    assert [p.hop_axis(i) for i in range(2)] == [1, 0]
    assert p.axis_stride(5) == -1 and p.hop_axis(2) == -1 and p.hop_kernel(0, 7) is None


def test_cost_model_closed_forms():
    B, Hq, Hkv, D, dims = 1, 32, 8, 128, (32, 32, 32)
    N = 32768
    p = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta.TA_BF16, True)
    assert p.hop_bytes(0, ta.TA_VIN_KV) == B * N * D * 2 * (Hq + Hkv + Hkv + Hq) == 671088640
    assert p.hop_bytes(1, ta.TA_VIN_O) == B * N * D * 2 * (Hq + Hkv + Hq + Hq) == 872415232
    assert p.hop_bytes(0, ta.TA_VIN_KV) / N == 20480 and p.hop_bytes(1, ta.TA_VIN_O) / N == 26624
    for ax in range(3):
        assert p.hop_flops(ax) == 4.0 * B * Hq * N * dims[ax] * D
        assert p.hop_flops(ax, True) == 2.5 * p.hop_flops(ax)
    # backward: first processed hop (axis 2, value input = an O) overwrites dQ, dK
    assert p.hop_bytes(2, ta.TA_VIN_O, True, False) / N == 2 * D * (Hq + Hkv + Hq + Hq + Hq + Hq + Hkv) == 45056
    assert p.hop_bytes(1, ta.TA_VIN_O, True, True) / N == 55296
    assert p.hop_bytes(0, ta.TA_VIN_KV, True, True) / N == 43008
    o_bytes = B * N * Hq * D * 2
    # 32 x 32 x 32 in bf16 at D = 128: the last two hops run fused in inference, so one intermediate O
    assert p.fused_position() == 1 and p.pair_kernel(1, ta.TA_VIN_O) == "mfma_bf16_pair_n32"
    assert p.pair_bytes(1, ta.TA_VIN_O) / N == 26624
    assert p.workspace_bytes(False) == o_bytes and p.workspace_bytes(True) == 2 * o_bytes
    pw = ta.ta_plan_create(B, Hq, Hkv, D, (32, 16, 64), ta.TA_BF16, True)
    assert pw.fused_position() == -1 and pw.pair_kernel(1, ta.TA_VIN_O) == "unsupported"
    assert pw.workspace_bytes(False) == 2 * o_bytes
    assert p.backward_scratch_bytes() == 2 * o_bytes
    p1 = ta.ta_plan_create(1, 1, 1, 64, (256,), ta.TA_F32, False)
    assert p1.workspace_bytes(False) == 0
    p2 = ta.ta_plan_create(1, 1, 1, 64, (16, 16), ta.TA_F32, False)
    assert p2.workspace_bytes(False) == 256 * 64 * 4 and p2.workspace_bytes(True) == 256 * 64 * 4


@pytest.mark.parametrize("kw,status", [
    (dict(dims=()), "TA_ERR_SHAPE"),
    (dict(dims=(2,) * 9), "TA_ERR_SHAPE"),
    (dict(dims=(4, 0)), "TA_ERR_SHAPE"),
    (dict(dims=(4, -3)), "TA_ERR_SHAPE"),
    (dict(n_q_heads=6, n_kv_heads=4), "TA_ERR_SHAPE"),
    (dict(batch=0), "TA_ERR_SHAPE"),
    (dict(head_dim=101), "TA_ERR_UNSUPPORTED"),
    (dict(head_dim=512), "TA_ERR_UNSUPPORTED"),
    (dict(dtype=7), "TA_ERR_INVALID_ARG"),
    (dict(hop_order=(0, 0)), "TA_ERR_INVALID_ARG"),
    (dict(hop_order=(0, 2)), "TA_ERR_INVALID_ARG"),
    (dict(scale=-1.0), "TA_ERR_INVALID_ARG"),
    (dict(scale=float("nan")), "TA_ERR_INVALID_ARG"),
    (dict(q_strides=(64, 64, 64)), "TA_ERR_SHAPE"),             # overlapping rows
    (dict(o_strides=(4 * 3 * 2 * 64, 2 * 64, 60)), "TA_ERR_SHAPE"),   # not a multiple of 8
    (dict(dims=(1 << 20, 1 << 20, 1 << 20)), "TA_ERR_SHAPE"),   # overflow
    (dict(window=(0, -2)), "TA_ERR_INVALID_ARG"),
    (dict(valid_len=-1), "TA_ERR_INVALID_ARG"),
    (dict(valid_len=13), "TA_ERR_SHAPE"),
])
def test_plan_rejects_bad_descriptors(kw, status):
    args = dict(batch=1, n_q_heads=2, n_kv_heads=2, head_dim=64, dims=(4, 3), dtype=ta.TA_F32, causal=False)
    args.update(kw)
    with pytest.raises(ta.TaError) as ei:
        ta.ta_plan_create(**args)
    assert ei.value.name == status
    assert ei.value.detail


def test_plan_create_null_pointers():
    lib = ta.load_library()
    h = C.c_void_p()
    assert lib.ta_plan_create(None, C.byref(h)) == 1
    d = binding.make_desc(1, 1, 1, 64, (4,), ta.TA_F32, False)
    assert lib.ta_plan_create(C.byref(d), None) == 1
    lib.ta_plan_destroy(None)
    assert lib.ta_plan_seq_len(None) == -1
    assert lib.ta_plan_workspace_bytes(None, 0) == 0


def test_strided_layouts_accepted():
    # head-major [B, H, N, D] for every tensor
    B, H, N, D = 2, 4, 12, 64
    s = (H * N * D, D, N * D)
    p = ta.ta_plan_create(B, H, H, D, (3, 4), ta.TA_BF16, True, q_strides=s, kv_strides=s, o_strides=s)
    assert p.seq_len() == 12


def test_entry_points_reject_bad_arguments_without_launching():
    """All of these return before any HIP call, so they run without a GPU.  The
    addresses are fabricated and never dereferenced."""
    p = ta.ta_plan_create(1, 2, 1, 64, (4, 3), ta.TA_F32, True)
    nbytes_q = 12 * 2 * 64 * 4
    Q, K, V, O, W = 0x10000000, 0x20000000, 0x30000000, 0x40000000, 0x50000000

    def status(fn, *a, **k):
        with pytest.raises(ta.TaError) as ei:
            fn(*a, **k)
        return ei.value.name

    S = 0xdead0   # never used: the calls fail first
    assert status(ta.ta_axis_attn_forward, p, 2, Q, K, V, 0, O, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_axis_attn_forward, p, -1, Q, K, V, 0, O, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_axis_attn_forward, p, 0, Q, K, V, 3, O, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_axis_attn_forward, p, 0, None, K, V, 0, O, S) == "TA_ERR_NULL"
    assert status(ta.ta_axis_attn_forward, p, 0, Q, K, V, 0, None, S) == "TA_ERR_NULL"
    assert status(ta.ta_axis_attn_forward, p, 0, Q + 4, K, V, 0, O, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_axis_attn_forward, p, 0, Q, K, V, 0, Q + nbytes_q - 16, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_axis_attn_forward, p, 0, Q, K, V, 0, V, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_axis_attn_forward, p, 0, Q, K, O, 1, O, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_forward, p, Q, K, V, O, None, 0, False, S) == "TA_ERR_NULL"
    assert status(ta.ta_multihop_forward, p, Q, K, V, O, W, 16, False, S) == "TA_ERR_WORKSPACE"
    assert status(ta.ta_multihop_forward, p, Q, K, V, O, W + 16, 1 << 20, False, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_multihop_forward, p, Q, K, V, O, O, 1 << 20, False, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_forward, p, None, K, V, O, W, 1 << 20, False, S) == "TA_ERR_NULL"
    assert status(ta.ta_axis_attn_backward, p, 0, Q, K, V, 0, O, Q, W, W + (1 << 20), False, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_axis_attn_backward, p, 0, Q, K, V, 0, O, W, W, W + (1 << 20), False, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_axis_attn_backward, p, 0, Q, K, V, 0, None, W, W, W, False, S) == "TA_ERR_NULL"
    assert status(ta.ta_multihop_backward, p, Q, K, V, O, W, 16, W, W, W, W, 0, S) == "TA_ERR_WORKSPACE"
    assert status(ta.ta_rope_apply, p, 2, 0, Q, O, 0.0, False, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_rope_apply, p, 0, 2, Q, O, 0.0, False, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_rope_apply, p, 0, -1, Q, Q + 32, 0.0, False, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_rope_apply, p, 0, -1, None, O, 0.0, False, S) == "TA_ERR_NULL"
    assert status(ta.ta_rope_apply, p, 1, 0, Q, O, -3.0, False, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_copy_bytes, Q, K, 24, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_copy_bytes, None, K, 32, S) == "TA_ERR_NULL"


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libtensattn.so")
    with pytest.raises(ImportError):
        ta.ta_plan_create(1, 1, 1, 64, (4,), ta.TA_F32, False)


def test_pack_axis_mask_layout():
    """Row a, word c // 32, bit c % 32 (the layout the descriptor's axis_mask documents)."""
    rng = np.random.default_rng(5)
    for n in (1, 5, 32, 33, 70):
        m = rng.random((n, n)) < 0.5
        words = ta.pack_axis_mask(m).view(np.uint32)
        assert words.shape == (n, (n + 31) // 32)
        for a in range(n):
            for c in range(n):
                assert ((int(words[a, c // 32]) >> (c % 32)) & 1) == int(m[a, c])
        # bits past the last column are zero
        if n % 32:
            assert (words[:, -1] >> np.uint32(n % 32) == 0).all()


def test_misaligned_axis_mask_is_rejected():
    with pytest.raises(ta.TaError) as e:
        ta.Plan(binding.make_desc(1, 2, 2, 64, (4, 4), ta.TA_F32, True, axis_masks=[6, None]))
    assert e.value.name == "TA_ERR_INVALID_ARG"


def test_kernels_for_other_head_widths():
    p = ta.ta_plan_create(1, 32, 32, 100, (32, 32), ta.TA_BF16, True)      # OpenLLaMA-3B geometry: a multiple of 4
    assert p.hop_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_n32" and p.hop_kernel(1, ta.TA_VIN_O) == "mfma_bf16_n32"
    assert p.fused_position() == 0 and p.pair_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_pair_n32"
    assert p.hop_backward_kernel(1, ta.TA_VIN_O) == "mfma_bf16_bwd_n32"
    two_tiles = ta.ta_plan_create(1, 32, 32, 100, (64, 16), ta.TA_BF16, True)
    assert two_tiles.hop_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_n64"
    assert two_tiles.hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_blocked"
    long_axis = ta.ta_plan_create(1, 8, 2, 96, (128, 4), ta.TA_BF16, True)
    assert long_axis.hop_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_stream_shared_kv"
    odd = ta.ta_plan_create(1, 4, 4, 90, (16, 16), ta.TA_BF16, True)       # even, not a multiple of 4
    assert odd.hop_kernel(0, ta.TA_VIN_KV) == "generic"
