"""The allocation-free KV quantizer (nvfp4_kv_quant_noalloc) against nvfp4_kv_quant, through the C ABI.

Runs last (file name) and must also pass alone in a fresh process: its first call on the device
is then the one that looks up the library's scratch array."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_18739_amd as nv
from paper_2605_18739_amd import workloads as wl
from .parity import dev_bf16, host_q

pytestmark = pytest.mark.gpu


def _same(a, b, what):
    (ca, sa, ga), (cb, sb, gb) = host_q(a), host_q(b)
    assert ga.view(np.uint32) == gb.view(np.uint32), f"{what}: global scale"
    assert (sa == sb).all(), f"{what}: scales"
    assert (ca == cb).all(), f"{what}: codes"


def test_kv_quant_noalloc_matches_kv_quant_two_calls_in_a_row():
    """Calls in a row on the library's own scratch array, each with a smaller input than the one before and each
    bit for bit what nvfp4_kv_quant gives.  The first two windows (141 MB and 126 MB of bf16) are too large to stay
    on the chip, so they take the two-pass kernels, whose partial maxima live in the scratch array; the third is
    small and takes the one-launch kernel, which leaves the array alone."""
    H, d = 24, 128
    shapes = [(23000, H, d), (20500, H, d), (37, H, d)]
    kvs = [dev_bf16(wl.kv_tensor(T, h, dd, 4, i)) for i, (T, h, dd) in enumerate(shapes)]
    # every tensor is much smaller in magnitude than the one before, so a stale maximum of an earlier call would show
    kvs[1] = (kvs[1].float() * 2.0 ** -6).to(torch.bfloat16)
    kvs[2] = (kvs[2].float() * 2.0 ** -12).to(torch.bfloat16)
    want = [nv.nvfp4_kv_quant(kv) for kv in kvs]
    outs = [nv.NVFP4Tensor(T * h, dd, "cuda") for (T, h, dd) in shapes]
    for o in outs:
        o.codes.fill_(0xEE)
        o.scales.fill_(0xEE)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for kv, o in zip(kvs, outs):                   # back to back on one stream, nothing in between
        nv.nvfp4_kv_quant_noalloc(kv, o)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for i, (o, w) in enumerate(zip(outs, want)):
        _same(o, w, f"call {i}")
    # and once more on a side stream, after the default stream's work is complete
    side = torch.cuda.Stream()
    o2 = nv.NVFP4Tensor(shapes[0][0] * H, d, "cuda")
    with torch.cuda.stream(side):
        nv.nvfp4_kv_quant_noalloc(kvs[0], o2, stream=side)
    side.synchronize()
    _same(o2, want[0], "side stream")


def test_kv_quant_noalloc_rejects_sizes_beyond_its_limit():
    L = nv.lib()
    t = nv.NVFP4Tensor(16, 128, "cuda")
    ct = t.c()
    x = torch.zeros(16 * 128, dtype=torch.bfloat16, device="cuda")
    big = nv.NOALLOC_MAX_ELEMENTS // 128 + 1      # rows that put T*H*d just past the limit
    ct.rows = big
    assert L.nvfp4_kv_quant_noalloc(ctypes.c_void_p(x.data_ptr()), big, 1, 128, ctypes.byref(ct), None) == -2
    assert L.nvfp4_kv_quant_noalloc(ctypes.c_void_p(x.data_ptr()), 1 << 40, 1 << 30, 128, ctypes.byref(ct), None) == -2
    assert L.nvfp4_kv_quant_noalloc(None, 1, 16, 128, ctypes.byref(t.c()), None) == -1
    assert L.nvfp4_kv_quant_noalloc(ctypes.c_void_p(x.data_ptr()), 0, 16, 128, ctypes.byref(t.c()), None) == -2
