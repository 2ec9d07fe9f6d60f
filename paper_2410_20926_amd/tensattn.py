"""ctypes binding of include/tensattn.h.  Argument marshalling only: every step of
the attention path runs inside the library's HIP kernels.  Tensors may be given as
torch tensors (their data_ptr() is passed) or as integer device addresses."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

TA_MAX_ORDER = 8
TA_F32, TA_BF16 = 0, 1
TA_VIN_KV, TA_VIN_O = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtensattn.so")
_lib = None

EXPORTS = [
    "ta_plan_create", "ta_plan_destroy", "ta_plan_seq_len", "ta_plan_axis_stride", "ta_plan_axis_fibres",
    "ta_plan_hop_axis", "ta_plan_hop_kernel", "ta_plan_hop_backward_kernel", "ta_plan_hop_bytes", "ta_plan_hop_flops",
    "ta_plan_workspace_bytes", "ta_plan_backward_scratch_bytes", "ta_axis_attn_forward",
    "ta_axis_attn_backward", "ta_multihop_forward", "ta_multihop_backward", "ta_rope_apply", "ta_copy_bytes", "ta_stream_mix", "ta_stream_slabs",
    "ta_status_string", "ta_last_error_detail", "ta_version",
    "ta_axis_pair_attn_forward", "ta_plan_pair_kernel", "ta_plan_pair_bytes", "ta_plan_fused_position",
    "ta_multihop_forward_static",
]
TA_STATIC_WORKSPACE_BYTES = 64 << 20


class TaDesc(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("order", C.c_int32), ("dims", C.c_int32 * TA_MAX_ORDER), ("dtype", C.c_int32), ("causal", C.c_int32),
        ("scale", C.c_float), ("hop_order", C.c_int32 * TA_MAX_ORDER),
        ("q_strides", C.c_int64 * 3), ("kv_strides", C.c_int64 * 3), ("o_strides", C.c_int64 * 3),
        ("window", C.c_int32 * TA_MAX_ORDER), ("valid_len", C.c_int64),
        ("axis_mask", C.c_void_p * TA_MAX_ORDER),
        ("valid_lens", C.c_void_p), ("rope", C.c_int32), ("rope_base", C.c_float),
        ("axis_mask_per_fibre", C.c_int32 * TA_MAX_ORDER),
    ]


class TaError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name}: {detail}" if detail else name)
        self.status = status
        self.name = name
        self.detail = detail


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the in-tree libtensattn.so.  There is no fallback of any kind: a missing
    library is an error (build it with `python -m paper_2410_20926_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2410_20926_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    vp, i, i64, sz, dbl = C.c_void_p, C.c_int, C.c_int64, C.c_size_t, C.c_double
    lib.ta_plan_create.argtypes = [C.POINTER(TaDesc), C.POINTER(vp)]
    lib.ta_plan_create.restype = i
    lib.ta_plan_destroy.argtypes = [vp]
    lib.ta_plan_destroy.restype = None
    lib.ta_plan_seq_len.argtypes = [vp]
    lib.ta_plan_seq_len.restype = i64
    for name in ("ta_plan_axis_stride", "ta_plan_axis_fibres"):
        getattr(lib, name).argtypes = [vp, i]
        getattr(lib, name).restype = i64
    lib.ta_plan_hop_axis.argtypes = [vp, i]
    lib.ta_plan_hop_axis.restype = i
    lib.ta_plan_hop_kernel.argtypes = [vp, i, i]
    lib.ta_plan_hop_kernel.restype = C.c_char_p
    lib.ta_plan_hop_backward_kernel.argtypes = [vp, i, i]
    lib.ta_plan_hop_backward_kernel.restype = C.c_char_p
    lib.ta_plan_hop_bytes.argtypes = [vp, i, i, i, i]
    lib.ta_plan_hop_bytes.restype = dbl
    lib.ta_plan_hop_flops.argtypes = [vp, i, i]
    lib.ta_plan_hop_flops.restype = dbl
    lib.ta_plan_workspace_bytes.argtypes = [vp, i]
    lib.ta_plan_workspace_bytes.restype = sz
    lib.ta_plan_backward_scratch_bytes.argtypes = [vp]
    lib.ta_plan_backward_scratch_bytes.restype = sz
    lib.ta_axis_attn_forward.argtypes = [vp, i, vp, vp, vp, i, vp, vp]
    lib.ta_axis_attn_forward.restype = i
    lib.ta_axis_pair_attn_forward.argtypes = [vp, i, vp, vp, vp, i, vp, vp, vp]
    lib.ta_axis_pair_attn_forward.restype = i
    lib.ta_plan_pair_kernel.argtypes = [vp, i, i]
    lib.ta_plan_pair_kernel.restype = C.c_char_p
    lib.ta_plan_pair_bytes.argtypes = [vp, i, i]
    lib.ta_plan_pair_bytes.restype = dbl
    lib.ta_plan_fused_position.argtypes = [vp]
    lib.ta_plan_fused_position.restype = i
    lib.ta_axis_attn_backward.argtypes = [vp, i, vp, vp, vp, i, vp, vp, vp, vp, i, vp]
    lib.ta_axis_attn_backward.restype = i
    lib.ta_multihop_forward.argtypes = [vp, vp, vp, vp, vp, vp, sz, i, vp]
    lib.ta_multihop_forward.restype = i
    lib.ta_multihop_forward_static.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.ta_multihop_forward_static.restype = i
    lib.ta_multihop_backward.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp, sz, vp]
    lib.ta_multihop_backward.restype = i
    lib.ta_rope_apply.argtypes = [vp, i, i, C.c_float, i, vp, vp, vp]
    lib.ta_rope_apply.restype = i
    lib.ta_copy_bytes.argtypes = [vp, vp, sz, vp]
    lib.ta_copy_bytes.restype = i
    lib.ta_stream_mix.argtypes = [vp, vp, sz, i, i, vp]
    lib.ta_stream_mix.restype = i
    lib.ta_stream_slabs.argtypes = [vp, vp, vp, vp, C.c_int64, i, i, i, vp]
    lib.ta_stream_slabs.restype = i
    lib.ta_status_string.argtypes = [i]
    lib.ta_status_string.restype = C.c_char_p
    lib.ta_last_error_detail.argtypes = []
    lib.ta_last_error_detail.restype = C.c_char_p
    lib.ta_version.argtypes = [C.POINTER(i), C.POINTER(i)]
    lib.ta_version.restype = None
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        lib = load_library()
        raise TaError(status, lib.ta_status_string(status).decode(), lib.ta_last_error_detail().decode())


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()            # torch tensor


def _stream(stream) -> Optional[int]:
    """A raw hipStream_t.  None = torch's current stream when torch is in use."""
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def make_desc(batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dims: Sequence[int], dtype: int,
              causal: bool, scale: float = 0.0, hop_order: Optional[Sequence[int]] = None,
              q_strides=None, kv_strides=None, o_strides=None, window: Optional[Sequence[int]] = None,
              valid_len: int = 0, axis_masks: Optional[Sequence] = None, valid_lens=None,
              rope_base: Optional[float] = None) -> TaDesc:
    """`axis_masks`: per axis None or a device tensor of packed bit rows (see pack_axis_mask), [n, words] for one
    table shared by the axis's fibres or [fibres, n, words] for one table per fibre;
    `valid_lens`: None or a device int64 tensor of B lengths; the descriptor keeps a reference to
    each so the memory outlives the plan.  `rope_base`: None = no encoding inside the hops, else
    the rotary base (0 = 10000)."""
    d = TaDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = batch, n_q_heads, n_kv_heads, head_dim
    d.order = len(dims)
    for j in range(TA_MAX_ORDER):
        d.dims[j] = int(dims[j]) if j < min(len(dims), TA_MAX_ORDER) else 0
        d.hop_order[j] = -1
    if hop_order is not None:
        for j, a in enumerate(hop_order[:TA_MAX_ORDER]):
            d.hop_order[j] = int(a)
    d.dtype, d.causal, d.scale = dtype, int(bool(causal)), float(scale)
    for j in range(TA_MAX_ORDER):
        d.window[j] = int(window[j]) if window is not None and j < len(window) else 0
    d.valid_len = int(valid_len)
    d._mask_refs = []
    for j in range(TA_MAX_ORDER):
        t = axis_masks[j] if axis_masks is not None and j < len(axis_masks) else None
        d.axis_mask[j] = _ptr(t) if t is not None else None
        d.axis_mask_per_fibre[j] = 1 if (t is not None and getattr(t, "ndim", 2) == 3) else 0   # [fibres, n, words]
        d._mask_refs.append(t)
    d.valid_lens = _ptr(valid_lens) if valid_lens is not None else None
    d._mask_refs.append(valid_lens)
    d.rope = 0 if rope_base is None else 1
    d.rope_base = 0.0 if rope_base is None else float(rope_base)
    for name, s in (("q_strides", q_strides), ("kv_strides", kv_strides), ("o_strides", o_strides)):
        arr = getattr(d, name)
        for j in range(3):
            arr[j] = int(s[j]) if s is not None else 0
    return d


def pack_axis_mask(mask):
    """Packs a boolean [n, n] table (row a, column c true = query position a may attend key
    position c), or [fibres, n, n] with one table per fibre, into the library's layout: uint32
    [..., n, ceil(n / 32)], bit c % 32 of word c / 32.  Returns a host array (viewed as int32, which
    torch can hold); move it to the device and pass it in `axis_masks`."""
    import numpy as np
    m = np.asarray(mask, dtype=bool)
    n = m.shape[-1]
    assert m.shape[-2:] == (n, n) and m.ndim in (2, 3)
    words = (n + 31) // 32
    padded = np.zeros(m.shape[:-1] + (words * 32,), dtype=bool)
    padded[..., :n] = m
    packed = np.packbits(padded.reshape(m.shape[:-1] + (words, 32)), axis=-1, bitorder="little")
    return np.ascontiguousarray(packed).view(np.uint32).reshape(m.shape[:-1] + (words,)).view(np.int32)


class Plan:
    """Owns a ta_plan_t*.  Immutable; destroyed with the object."""

    def __init__(self, desc: TaDesc):
        lib = load_library()
        h = C.c_void_p()
        _check(lib.ta_plan_create(C.byref(desc), C.byref(h)))
        self._h = h
        self.desc = desc
        self.order = desc.order
        self.dims = tuple(desc.dims[j] for j in range(desc.order))

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.ta_plan_destroy(h)

    @property
    def handle(self):
        return self._h

    def seq_len(self) -> int:
        return load_library().ta_plan_seq_len(self._h)

    def axis_stride(self, axis: int) -> int:
        return load_library().ta_plan_axis_stride(self._h, axis)

    def axis_fibres(self, axis: int) -> int:
        return load_library().ta_plan_axis_fibres(self._h, axis)

    def hop_axis(self, pos: int) -> int:
        return load_library().ta_plan_hop_axis(self._h, pos)

    def hop_kernel(self, axis: int, vin: int) -> Optional[str]:
        s = load_library().ta_plan_hop_kernel(self._h, axis, vin)
        return s.decode() if s is not None else None

    def hop_backward_kernel(self, axis: int, vin: int) -> Optional[str]:
        s = load_library().ta_plan_hop_backward_kernel(self._h, axis, vin)
        return s.decode() if s is not None else None

    def pair_kernel(self, axis: int, vin: int) -> Optional[str]:
        s = load_library().ta_plan_pair_kernel(self._h, axis, vin)
        return s.decode() if s is not None else None

    def pair_bytes(self, axis: int, vin: int) -> float:
        return load_library().ta_plan_pair_bytes(self._h, axis, vin)

    def fused_position(self) -> int:
        return load_library().ta_plan_fused_position(self._h)

    def hop_bytes(self, axis: int, vin: int, backward: bool = False, accumulate: bool = False) -> float:
        return load_library().ta_plan_hop_bytes(self._h, axis, vin, int(backward), int(accumulate))

    def hop_flops(self, axis: int, backward: bool = False) -> float:
        return load_library().ta_plan_hop_flops(self._h, axis, int(backward))

    def workspace_bytes(self, save_for_backward: bool = False) -> int:
        return load_library().ta_plan_workspace_bytes(self._h, int(save_for_backward))

    def backward_scratch_bytes(self) -> int:
        return load_library().ta_plan_backward_scratch_bytes(self._h)


def ta_plan_create(batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dims: Sequence[int], dtype: int,
                   causal: bool, **kw) -> Plan:
    return Plan(make_desc(batch, n_q_heads, n_kv_heads, head_dim, dims, dtype, causal, **kw))


def ta_axis_pair_attn_forward(plan: Plan, axis: int, q, k, v_in, vin: int, o_out, stream=None, o_mid=None) -> None:
    _check(load_library().ta_axis_pair_attn_forward(plan.handle, axis, _ptr(q), _ptr(k), _ptr(v_in), vin, _ptr(o_mid),
                                                    _ptr(o_out), _stream(stream)))


def ta_axis_attn_forward(plan: Plan, axis: int, q, k, v_in, vin: int, o_out, stream=None) -> None:
    _check(load_library().ta_axis_attn_forward(plan.handle, axis, _ptr(q), _ptr(k), _ptr(v_in), vin, _ptr(o_out),
                                               _stream(stream)))


def ta_axis_attn_backward(plan: Plan, axis: int, q, k, v_in, vin: int, d_o, d_v_in, dq, dk, accumulate: bool,
                          stream=None) -> None:
    _check(load_library().ta_axis_attn_backward(plan.handle, axis, _ptr(q), _ptr(k), _ptr(v_in), vin, _ptr(d_o),
                                                _ptr(d_v_in), _ptr(dq), _ptr(dk), int(accumulate), _stream(stream)))


def ta_multihop_forward(plan: Plan, q, k, v, o, workspace, workspace_bytes: int, save_for_backward: bool = False,
                        stream=None) -> None:
    _check(load_library().ta_multihop_forward(plan.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(workspace),
                                              workspace_bytes, int(save_for_backward), _stream(stream)))


def ta_multihop_forward_static(plan: Plan, q, k, v, o, stream=None) -> None:
    _check(load_library().ta_multihop_forward_static(plan.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _stream(stream)))


def ta_multihop_backward(plan: Plan, q, k, v, d_o, workspace, workspace_bytes: int, dq, dk, dv, scratch,
                         scratch_bytes: int, stream=None) -> None:
    _check(load_library().ta_multihop_backward(plan.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(workspace),
                                               workspace_bytes, _ptr(dq), _ptr(dk), _ptr(dv), _ptr(scratch),
                                               scratch_bytes, _stream(stream)))


def ta_rope_apply(plan: Plan, which: int, axis: int, x, y, base: float = 0.0, inverse: bool = False, stream=None) -> None:
    _check(load_library().ta_rope_apply(plan.handle, which, axis, float(base), int(inverse), _ptr(x), _ptr(y),
                                        _stream(stream)))


def ta_copy_bytes(src, dst, nbytes: int, stream=None) -> None:
    _check(load_library().ta_copy_bytes(_ptr(src), _ptr(dst), nbytes, _stream(stream)))


def ta_stream_mix(src, dst, units: int, reads: int, writes: int, stream=None) -> None:
    _check(load_library().ta_stream_mix(_ptr(src), _ptr(dst), units, reads, writes, _stream(stream)))


def ta_stream_slabs(q, k, x, o, tokens: int, n_q_heads: int, n_kv_heads: int, granule: int, stream=None) -> None:
    _check(load_library().ta_stream_slabs(_ptr(q), _ptr(k), _ptr(x), _ptr(o), tokens, n_q_heads, n_kv_heads, granule,
                                          _stream(stream)))


def ta_version():
    a, b = C.c_int(), C.c_int()
    load_library().ta_version(C.byref(a), C.byref(b))
    return a.value, b.value
