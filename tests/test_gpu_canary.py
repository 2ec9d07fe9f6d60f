"""Out-of-bounds guard: every buffer a call writes (outputs, workspace, scratch) sits between two
4 KB canary regions inside one larger allocation; after the call the canaries must be intact.
Covers the per-axis forward, the fused pair, the multi-hop forward and the multi-hop backward on
a ragged shape (tiles with padding rows, a ragged last tile), a strided head-major layout and a
shape with long axes (streaming forward, blocked backward)."""
import numpy as np
import pytest
import torch

import paper_2410_20926_amd as ta
from gpu_util import ta_dtype, to_dev, torch_dtype
from paper_2410_20926_amd.workloads import make_inputs

pytestmark = pytest.mark.gpu

CANARY = 4096
PATTERN = 0xA5


class Guarded:
    """`nbytes` usable bytes, 256-byte aligned, with CANARY bytes of a fixed pattern on both sides."""

    def __init__(self, nbytes: int):
        self.nbytes = int(nbytes)
        pad = (-self.nbytes) % 256
        self.raw = torch.full((CANARY + self.nbytes + pad + CANARY,), PATTERN, dtype=torch.uint8, device="cuda")
        assert self.raw.data_ptr() % 256 == 0
        self.body = self.raw[CANARY:CANARY + self.nbytes]
        self.body.fill_(0xFF)                      # NaN pattern for bf16 and fp32 alike

    def tensor(self, shape, dtype):
        return self.body.view(dtype).view(*shape)

    def check(self, what):
        head = self.raw[:CANARY]
        tail = self.raw[CANARY + self.nbytes:]
        assert bool((head == PATTERN).all()), f"{what}: bytes before the buffer were overwritten"
        assert bool((tail == PATTERN).all()), f"{what}: bytes after the buffer were overwritten"


def esize(dtype):
    return 4 if dtype == "f32" else 2


CASES = [
    # dims, B, Hq, Hkv, D, dtype, causal, head_major
    ((5, 7, 3), 2, 4, 2, 64, "bf16", True, False),       # ragged tiles with padding rows
    ((3, 50), 1, 4, 1, 128, "bf16", True, False),        # two-tile axis with a ragged second tile
    ((2, 32, 32), 1, 8, 2, 128, "bf16", True, False),    # fused last pair
    ((6, 32), 2, 4, 2, 64, "bf16", True, True),          # head-major strides
    ((130, 3), 1, 4, 1, 128, "bf16", False, False),      # streaming forward, blocked backward, ragged last tile
    ((6, 9), 1, 4, 4, 100, "bf16", True, False),         # narrow head: 8-byte-granular rows
    ((4, 2, 3), 1, 2, 1, 8, "f32", True, False),         # generic kernels
    ((5, 37), 1, 4, 1, 40, "f32", False, True),          # generic kernels, head-major
]


@pytest.mark.parametrize("dims,B,Hq,Hkv,D,dtype,causal,head_major", CASES)
def test_no_write_outside_outputs_workspace_and_scratch(dims, B, Hq, Hkv, D, dtype, causal, head_major):
    N = int(np.prod(dims))
    es, tdt = esize(dtype), torch_dtype(dtype)
    q, k, v, d_o = make_inputs(B, N, Hq, Hkv, D, seed=77 + N, dtype=dtype, with_grad=True)
    kw = {}
    if head_major:
        kw = dict(q_strides=(Hq * N * D, D, N * D), kv_strides=(Hkv * N * D, D, N * D), o_strides=(Hq * N * D, D, N * D))
        lay = lambda a: to_dev(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), dtype)
        shp_q, shp_kv = (B, Hq, N, D), (B, Hkv, N, D)
    else:
        lay = lambda a: to_dev(a, dtype)
        shp_q, shp_kv = (B, N, Hq, D), (B, N, Hkv, D)
    plan = ta.ta_plan_create(B, Hq, Hkv, D, dims, ta_dtype(dtype), causal, **kw)
    tq, tk, tv, tg = lay(q), lay(k), lay(v), lay(d_o)
    nq, nkv = B * N * Hq * D * es, B * N * Hkv * D * es

    # one hop on its own, value input V
    g_o = Guarded(nq)
    ta.ta_axis_attn_forward(plan, len(dims) - 1, tq, tk, tv, ta.TA_VIN_KV, g_o.tensor(shp_q, tdt))
    torch.cuda.synchronize()
    g_o.check("per-axis forward output")

    # the fused pair on its own, with and without the tensor between its hops
    if plan.pair_kernel(len(dims) - 2, ta.TA_VIN_O) == "mfma_bf16_pair_n32":
        g_o2, g_mid = Guarded(nq), Guarded(nq)
        x = g_o.tensor(shp_q, tdt)
        ta.ta_axis_pair_attn_forward(plan, len(dims) - 2, tq, tk, x, ta.TA_VIN_O, g_o2.tensor(shp_q, tdt), o_mid=g_mid.tensor(shp_q, tdt))
        torch.cuda.synchronize()
        g_o2.check("fused pair output"); g_mid.check("fused pair intermediate output")

    # multi-hop forward (inference workspace), then the training forward and the backward
    for save in (False, True):
        wsb = plan.workspace_bytes(save)
        g_ws, g_out = Guarded(max(wsb, 256)), Guarded(nq)
        ta.ta_multihop_forward(plan, tq, tk, tv, g_out.tensor(shp_q, tdt), g_ws.body, wsb, save)
        torch.cuda.synchronize()
        g_ws.check(f"multi-hop forward workspace (save={save})"); g_out.check(f"multi-hop forward output (save={save})")
    scb = plan.backward_scratch_bytes()
    g_sc, g_dq, g_dk, g_dv = Guarded(max(scb, 256)), Guarded(nq), Guarded(nkv), Guarded(nkv)
    ta.ta_multihop_backward(plan, tq, tk, tv, tg, g_ws.body, wsb, g_dq.tensor(shp_q, tdt), g_dk.tensor(shp_kv, tdt),
                            g_dv.tensor(shp_kv, tdt), g_sc.body, scb)
    torch.cuda.synchronize()
    for g_, name in ((g_sc, "scratch"), (g_dq, "dq"), (g_dk, "dk"), (g_dv, "dv"), (g_ws, "workspace (read-only in the backward)")):
        g_.check(f"multi-hop backward {name}")
    for t_, name in ((g_dq.tensor(shp_q, tdt), "dq"), (g_dk.tensor(shp_kv, tdt), "dk"), (g_dv.tensor(shp_kv, tdt), "dv"),
                     (g_out.tensor(shp_q, tdt), "o")):
        assert bool(torch.isfinite(t_.float()).all()), f"{name} holds values the call did not write"


@pytest.mark.parametrize("reads,writes", [(1, 1), (3, 2), (9, 4), (4, 3)])
def test_measurement_kernels_move_what_they_say(reads, writes):
    """The copy and the streaming kernel of the measurement aids: every byte they are meant to write is written
    with the expected value, and nothing outside (they calibrate the traffic counters and give the attainable rate)."""
    units = 37
    g = torch.Generator(device="cuda").manual_seed(5)
    src = torch.randint(0, 2 ** 31 - 1, (units * reads * 1024 + 8,), dtype=torch.int32, device="cuda", generator=g)
    dst = torch.full((units * writes * 1024 + 8,), -7, dtype=torch.int32, device="cuda")
    ta.ta_stream_mix(src[4:], dst[4:], units, reads, writes)
    torch.cuda.synchronize()
    x = src[4:4 + units * reads * 1024].view(units, reads, 1024)
    acc = x[:, 0]
    for r in range(1, reads):
        acc = acc ^ x[:, r]
    want = torch.stack([acc + w for w in range(writes)], dim=1).reshape(-1)
    assert torch.equal(dst[4:4 + units * writes * 1024], want)
    assert (dst[:4] == -7).all() and (dst[-4:] == -7).all()
    if reads == 1 and writes == 1:
        out = torch.full_like(src, -7)
        ta.ta_copy_bytes(src[4:-4], out[4:-4], (src.numel() - 8) * 4)
        torch.cuda.synchronize()
        assert torch.equal(out[4:-4], src[4:-4]) and (out[:4] == -7).all() and (out[-4:] == -7).all()


@pytest.mark.parametrize("granule", [1, 2, 3])
@pytest.mark.parametrize("heads", [(8, 2), (4, 4), (3, 1)])
def test_slab_streaming_kernel_moves_what_it_says(granule, heads):
    """The kernel that repeats the fused pair's traffic without its arithmetic: with zeros for Q and K the output
    is the value input, with anything else every output row is still written, and nothing outside the tensors is."""
    Hq, Hkv = heads
    tokens = 2048
    g = torch.Generator(device="cuda").manual_seed(9)
    nq, nk = tokens * Hq * 128, tokens * Hkv * 128
    x = torch.randint(-2 ** 15, 2 ** 15 - 1, (nq,), dtype=torch.int16, device="cuda", generator=g)
    for zeros in (True, False):
        q = torch.zeros(nq, dtype=torch.int16, device="cuda") if zeros else torch.randint(1, 2 ** 15 - 1, (nq,), dtype=torch.int16, device="cuda", generator=g)
        k = torch.zeros(nk, dtype=torch.int16, device="cuda") if zeros else torch.randint(1, 2 ** 15 - 1, (nk,), dtype=torch.int16, device="cuda", generator=g)
        o = torch.full((nq + 16,), -7, dtype=torch.int16, device="cuda")
        ta.ta_stream_slabs(q, k, x, o[8:], tokens, Hq, Hkv, granule)
        torch.cuda.synchronize()
        assert (o[:8] == -7).all() and (o[-8:] == -7).all()
        if zeros:
            assert torch.equal(o[8:-8], x)
        else:
            # every 16-byte unit is the input's unit xor one 32-bit word repeated four times
            d = (o[8:-8] ^ x).view(torch.int32).view(-1, 4)
            assert bool((d == d[:, :1]).all())
