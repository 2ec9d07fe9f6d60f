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
    assert ta.ta_version() == (0, 7)
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
    (dict(valid_lens=0x1004), "TA_ERR_INVALID_ARG"),            # not 8-byte aligned
    (dict(rope_base=-2.0), "TA_ERR_INVALID_ARG"),
    (dict(rope_base=float("inf")), "TA_ERR_INVALID_ARG"),
])
def test_plan_rejects_bad_descriptors(kw, status):
    args = dict(batch=1, n_q_heads=2, n_kv_heads=2, head_dim=64, dims=(4, 3), dtype=ta.TA_F32, causal=False)
    args.update(kw)
    with pytest.raises(ta.TaError) as ei:
        ta.ta_plan_create(**args)
    assert ei.value.name == status
    assert ei.value.detail


def test_per_fibre_mask_flag_must_be_0_or_1_and_packing_keeps_the_fibre_axis():
    import numpy as np
    d = binding.make_desc(1, 2, 2, 64, (4, 3), ta.TA_F32, False)
    d.axis_mask_per_fibre[1] = 3
    with pytest.raises(ta.TaError) as e:
        ta.Plan(d)
    assert e.value.name == "TA_ERR_INVALID_ARG"
    d.axis_mask_per_fibre[1] = 1
    d.axis_mask_per_fibre[5] = 9                       # entries at or beyond `order` are ignored
    ta.Plan(d)
    m = np.random.default_rng(3).random((7, 40, 40)) < 0.5
    packed = ta.pack_axis_mask(m).view(np.uint32)
    assert packed.shape == (7, 40, 2)
    for f, a, c in ((0, 0, 0), (6, 39, 39), (3, 17, 32), (2, 5, 31)):
        assert bool((packed[f, a, c // 32] >> (c % 32)) & 1) == bool(m[f, a, c])
    assert np.array_equal(ta.pack_axis_mask(m[4]), ta.pack_axis_mask(m)[4])


def test_rope_flag_must_be_0_or_1():
    d = binding.make_desc(1, 2, 2, 64, (4, 3), ta.TA_F32, False)
    d.rope = 2
    with pytest.raises(ta.TaError) as e:
        ta.Plan(d)
    assert e.value.name == "TA_ERR_INVALID_ARG"
    # the encoding rides on the same kernels, the fused pair of hops included
    p = ta.ta_plan_create(1, 32, 8, 128, (32, 32, 32), ta.TA_BF16, True, rope_base=10000.0)
    assert p.fused_position() == 1 and p.pair_kernel(1, ta.TA_VIN_O) == "mfma_bf16_pair_n32"
    assert p.workspace_bytes(False) == 32768 * 32 * 128 * 2
    assert p.hop_kernel(1, ta.TA_VIN_O) == "mfma_bf16_n32_shared" and p.hop_backward_kernel(1, ta.TA_VIN_O) == "mfma_bf16_bwd_n32"


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


def test_strides_whose_span_would_overflow_are_refused():
    """A stride so large that (extent - 1) * stride leaves the 64-bit range is a shape error, not an
    address wrap in the alias checks."""
    huge = (1 << 60, 64, 8 * 64)
    with pytest.raises(ta.TaError) as ei:
        ta.ta_plan_create(16, 8, 8, 64, (4, 4), ta.TA_BF16, True, q_strides=huge)
    assert ei.value.name == "TA_ERR_SHAPE"
    ok = (1 << 40, 8 * 64, 64)
    assert ta.ta_plan_create(16, 8, 8, 64, (4, 4), ta.TA_BF16, True, q_strides=ok).seq_len() == 16


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
    assert status(ta.ta_stream_mix, Q, K, 4, 5, 3, S) == "TA_ERR_UNSUPPORTED"      # no kernel for that mix
    assert status(ta.ta_stream_mix, None, K, 4, 1, 1, S) == "TA_ERR_NULL"
    assert status(ta.ta_stream_mix, Q + 8, K, 4, 1, 1, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_stream_slabs, Q, K, V, None, 1024, 4, 2, 1, S) == "TA_ERR_NULL"
    assert status(ta.ta_stream_slabs, Q, K, V, O, 1000, 4, 2, 1, S) == "TA_ERR_INVALID_ARG"   # not a multiple of 1024
    assert status(ta.ta_stream_slabs, Q, K, V, O, 1024, 4, 3, 1, S) == "TA_ERR_INVALID_ARG"   # heads do not divide
    assert status(ta.ta_stream_slabs, Q, K, V, O, 1024, 4, 2, 4, S) == "TA_ERR_INVALID_ARG"   # no such granule
    assert status(ta.ta_stream_slabs, Q, K, V, O + 8, 1024, 4, 2, 1, S) == "TA_ERR_INVALID_ARG"


def test_multihop_calls_validate_every_hop_before_the_first_launch():
    """Nothing may be enqueued when a call is going to fail: aliasing, alignment and the
    availability of a kernel for EVERY hop are checked up front.  There is no GPU here, so a
    call that got as far as a launch would come back as TA_ERR_DEVICE instead."""
    def status(fn, *a, **k):
        with pytest.raises(ta.TaError) as ei:
            fn(*a, **k)
        return ei.value.name

    S = 0xdead0
    Q, K, V, O, W, G = 0x10000000, 0x20000000, 0x30000000, 0x40000000, 0x50000000, 0x60000000
    DQ, DK, DV, SC = 0x70000000, 0x80000000, 0x90000000, 0xa0000000
    p = ta.ta_plan_create(1, 2, 1, 64, (4, 3), ta.TA_F32, True)
    big = 1 << 20
    # the output of the LAST hop overlaps an input: found before the first hop is enqueued
    assert status(ta.ta_multihop_forward, p, Q, K, V, Q + 64, W, big, False, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_forward, p, Q, K, V, V, W, big, False, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_forward, p, Q, K + 8, V, O, W, big, False, S) == "TA_ERR_INVALID_ARG"
    # backward: scratch and workspace are range-checked against every tensor and each other
    assert status(ta.ta_multihop_backward, p, Q, K, V, G, W, big, DQ, DK, DV, W, big, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_backward, p, Q, K, V, G, W, big, DQ, DK, DV, DQ, big, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_backward, p, Q, K, V, G, W, big, DQ, DK, DV, Q, big, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_backward, p, Q, K, V, G, W, big, W, DK, DV, SC, big, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_backward, p, Q, K, V, G, W, big, DQ, DQ, DV, SC, big, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_backward, p, Q, K, V, G, W, big, DQ, DK, K, SC, big, S) == "TA_ERR_ALIAS"
    assert status(ta.ta_multihop_backward, p, Q, K, V, G, W, big, DQ, DK, DV, SC + 16, big, S) == "TA_ERR_INVALID_ARG"
    assert status(ta.ta_multihop_backward, p, Q, K, V, G, W, big, DQ + 2, DK, DV, SC, big, S) == "TA_ERR_INVALID_ARG"
    # an fp32 axis too long for the backward's row statistics: the hop over axis 1 runs first in
    # the backward and is fine, the hop over axis 0 is not; the call must refuse before either
    long_axis = ta.ta_plan_create(1, 8, 1, 64, (4096, 2), ta.TA_F32, True)
    assert long_axis.hop_backward_kernel(1, ta.TA_VIN_O) == "generic"
    assert long_axis.hop_backward_kernel(0, ta.TA_VIN_KV) == "unsupported"
    huge = 1 << 28
    A = [i << 32 for i in range(1, 12)]
    assert status(ta.ta_multihop_backward, long_axis, A[0], A[1], A[2], A[3], A[4], huge, A[5], A[6], A[7], A[8], huge, S) == "TA_ERR_UNSUPPORTED"


def test_launch_geometry_is_settled_when_the_plan_is_made():
    """Whether a kernel's launch grid fits is decided by ta_plan_create, not at launch time."""
    ok = ta.ta_plan_create(32767, 1, 1, 64, (32769, 16), ta.TA_BF16, True)
    assert ok.hop_kernel(1, ta.TA_VIN_KV) == "mfma_bf16_n32" and ok.hop_backward_kernel(1, ta.TA_VIN_KV) == "mfma_bf16_bwd_n32"
    # 32,769 tiles need 2 grid rows per batch element: with 32,768 batch elements no grid holds the job, neither
    # the matrix-core kernel's nor the generic kernel's, and the plan says so (it used to surface as a failed launch)
    more = ta.ta_plan_create(32768, 1, 1, 64, (32769, 32), ta.TA_BF16, True)
    assert more.hop_kernel(1, ta.TA_VIN_KV) == "unsupported"
    assert more.hop_backward_kernel(1, ta.TA_VIN_KV) == "generic"        # one workgroup per fibre and group: that grid fits
    assert more.pair_kernel(0, ta.TA_VIN_KV) == "unsupported"
    none = ta.ta_plan_create(65535, 8, 1, 64, (32769, 32), ta.TA_BF16, True)         # more workgroups than any grid here holds
    assert none.hop_kernel(1, ta.TA_VIN_KV) == "unsupported"
    with pytest.raises(ta.TaError) as e:
        ta.ta_axis_attn_forward(none, 1, 1 << 50, 2 << 50, 3 << 50, ta.TA_VIN_KV, 4 << 50, 0xdead0)
    assert e.value.name == "TA_ERR_UNSUPPORTED"


def test_sequence_length_overflow_is_caught_before_multiplying():
    for dims in ((1 << 30, 1 << 30), (1 << 20, 1 << 20, 1 << 20), (2147483647, 2147483647, 2147483647, 2147483647)):
        with pytest.raises(ta.TaError) as e:
            ta.ta_plan_create(1, 1, 1, 64, dims, ta.TA_F32, False)
        assert e.value.name == "TA_ERR_SHAPE"
    assert ta.load_library().ta_status_string(8) == b"TA_ERR_NOMEM"


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
    # the fused kernel takes the width, but the multi-hop call uses it only for rows of whole 64-byte pieces (widths
    # that are a multiple of 32): elsewhere the two hops on their own are faster
    assert p.fused_position() == -1 and p.pair_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_pair_n32"
    assert ta.ta_plan_create(1, 32, 8, 96, (32, 32), ta.TA_BF16, True).fused_position() == 0
    assert p.hop_backward_kernel(1, ta.TA_VIN_O) == "mfma_bf16_bwd_n32"
    two_tiles = ta.ta_plan_create(1, 32, 32, 100, (64, 16), ta.TA_BF16, True)
    assert two_tiles.hop_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_n64"
    assert two_tiles.hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_blocked"      # narrow heads stay on the blocked kernel
    assert ta.ta_plan_create(1, 32, 8, 128, (64, 16), ta.TA_BF16, True).hop_backward_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_bwd_n64"
    long_axis = ta.ta_plan_create(1, 8, 2, 96, (128, 4), ta.TA_BF16, True)
    assert long_axis.hop_kernel(0, ta.TA_VIN_KV) == "mfma_bf16_stream_shared_kv"
    odd = ta.ta_plan_create(1, 4, 4, 90, (16, 16), ta.TA_BF16, True)       # even, not a multiple of 4
    assert odd.hop_kernel(0, ta.TA_VIN_KV) == "generic"
