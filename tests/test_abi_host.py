"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_18739_amd as nv
from paper_2605_18739_amd.binding import _CTensor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "nvfp4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nvfp4_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = nv.lib()
    names = _declared_symbols()
    assert {"nvfp4_quantize", "nvfp4_gemm", "nvfp4_gemm_act_quant", "nvfp4_kv_quant",
            "nvfp4_kv_dequant", "nvfp4_workspace_bytes", "nvfp4_status_string", "nvfp4_set_one_launch",
            "nvfp4_quantize_4over6", "nvfp4_kv_quant_4over6", "nvfp4_kv_quant_k",
            "nvfp4_kv_dequant_gather", "nvfp4_quantize_2d", "nvfp4_quantize_rht",
            "nvfp4_quantize_for_all_to_all", "nvfp4_lora_down", "nvfp4_gemm_lora",
            "nvfp4_kv_quant_noalloc", "nvfp4_gemm_scale_out"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    L = nv.lib()
    assert L.nvfp4_status_string(0) == b"ok"
    for rc in (-1, -2, -3, -4, -5):
        assert len(L.nvfp4_status_string(rc)) > 5
    assert L.nvfp4_status_string(-99) == b"unknown status"


def test_one_launch_mode_is_validated_on_the_host():
    L = nv.lib()
    for mode in (nv.ONE_LAUNCH_ALWAYS, nv.ONE_LAUNCH_NEVER, nv.ONE_LAUNCH_AUTO):
        assert L.nvfp4_set_one_launch(mode) == 0
    assert L.nvfp4_set_one_launch(3) == -2 and L.nvfp4_set_one_launch(-1) == -2         # NVFP4_ERR_SHAPE
    assert L.nvfp4_set_one_launch(nv.ONE_LAUNCH_AUTO) == 0


def test_workspace_sizes():
    assert nv.nvfp4_workspace_bytes(nv.OP_QUANTIZE, 128, 256) == 4096
    assert nv.nvfp4_workspace_bytes(nv.OP_KV_QUANT, 10, 24, 128) == 4096
    # the Hadamard quantizer: the partial maxima plus one byte per lane of every 128 x 256 tile (pass 1 -> pass 2)
    assert nv.nvfp4_workspace_bytes(nv.OP_QUANTIZE_RHT, 128, 256) == 4096 + 256
    assert nv.nvfp4_workspace_bytes(nv.OP_QUANTIZE_RHT, 17600, 14336) == 4096 + 138 * 56 * 256
    assert nv.nvfp4_workspace_bytes(nv.OP_QUANTIZE_RHT, 144, 264) == 4096 + 2 * 2 * 256
    with_h = nv.nvfp4_workspace_bytes(nv.OP_GEMM_ACT_QUANT, 3520, 14336, 0)
    without_h = nv.nvfp4_workspace_bytes(nv.OP_GEMM_ACT_QUANT, 3520, 14336, 1)
    assert with_h - without_h == 3520 * 14336 * 2
    assert nv.nvfp4_workspace_bytes(99, 1, 1, 1) == 0


def _t(codes=0x1000, scales=0x2000, gs=0x3000, rows=4, K=32):
    return _CTensor(codes, scales, gs, rows, K)


def test_quantize_rejects_bad_arguments_on_the_host():
    """Pointers below are fake but never dereferenced: validation fails first."""
    L = nv.lib()
    x, ws = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x20000)
    ok = _t()
    q = lambda xp, R, C, ld, ax, t, w, wb: L.nvfp4_quantize(xp, R, C, ld, ax, None, ctypes.byref(t), w, wb, None)
    assert q(None, 4, 32, 32, 0, ok, ws, 4096) == -1                 # NULL input
    assert q(x, 4, 32, 32, 0, _t(codes=None), ws, 4096) == -1        # NULL output plane
    assert q(x, 4, 24, 24, 0, _t(K=24), ws, 4096) == -2              # K % 16
    assert q(x, 4, 32, 32, 0, _t(rows=5), ws, 4096) == -2            # out shape mismatch
    assert q(x, 4, 32, 16, 0, ok, ws, 4096) == -2                    # ld < C
    assert q(x, 4, 32, 32, 2, ok, ws, 4096) == -2                    # bad axis
    assert q(ctypes.c_void_p(0x10002), 4, 32, 32, 0, ok, ws, 4096) == -3   # misaligned x
    assert q(x, 4, 32, 36, 0, ok, ws, 4096) == -3                    # ld % 8
    assert q(x, 4, 32, 32, 0, _t(codes=0x1001), ws, 4096) == -3      # misaligned codes
    assert q(x, 4, 32, 32, 0, ok, None, 0) == -4                     # workspace missing
    assert q(x, 4, 32, 32, 0, ok, ws, 100) == -4                     # workspace too small
    # transposed: rows = C, K = R
    assert q(x, 32, 8, 8, 1, _t(rows=8, K=32), ws, 100) == -4
    assert q(x, 24, 8, 8, 1, _t(rows=8, K=24), ws, 4096) == -2


def test_gemm_and_kv_reject_bad_arguments_on_the_host():
    L = nv.lib()
    y = ctypes.c_void_p(0x40000)
    a, w = _t(rows=4, K=32), _t(rows=8, K=32)
    assert L.nvfp4_gemm(ctypes.byref(a), ctypes.byref(w), None, 8, 0, None) == -1
    assert L.nvfp4_gemm(ctypes.byref(a), ctypes.byref(_t(rows=8, K=64)), y, 8, 0, None) == -2   # K mismatch
    assert L.nvfp4_gemm(ctypes.byref(a), ctypes.byref(w), y, 4, 0, None) == -2                  # ldy < N
    assert L.nvfp4_gemm(ctypes.byref(a), ctypes.byref(w), y, 8, 7, None) == -2                  # bad dtype
    assert L.nvfp4_gemm(ctypes.byref(a), ctypes.byref(w), y, 10, 0, None) == -3                 # ldy % 4
    a64, w64 = _t(rows=4, K=64), _t(rows=8, K=64)                                                 # a shape the tiled kernels take
    assert L.nvfp4_gemm(ctypes.byref(a64), ctypes.byref(w64), y, 12, 1, None) == -3              # bf16 rows must stay 16-byte aligned: ldy % 8
    # GEMM that also returns the tensor scale of its output
    gs, ws = ctypes.c_void_p(0x50000), ctypes.c_void_p(0x60000)
    need = nv.nvfp4_workspace_bytes(nv.OP_GEMM_SCALE_OUT, 4, 8)
    assert need >= 4096 and need % 256 == 0
    assert L.nvfp4_gemm_scale_out(ctypes.byref(a64), ctypes.byref(w64), None, 8, gs, ws, need, None) == -1
    assert L.nvfp4_gemm_scale_out(ctypes.byref(a64), ctypes.byref(w64), y, 8, None, ws, need, None) == -1
    assert L.nvfp4_gemm_scale_out(ctypes.byref(a64), ctypes.byref(w64), y, 4, gs, ws, need, None) == -2       # ldy < N
    assert L.nvfp4_gemm_scale_out(ctypes.byref(a64), ctypes.byref(w64), y, 12, gs, ws, need, None) == -3      # ldy % 8
    assert L.nvfp4_gemm_scale_out(ctypes.byref(a64), ctypes.byref(w64), y, 8, gs, ws, need - 1, None) == -4   # workspace
    assert L.nvfp4_gemm_scale_out(ctypes.byref(a64), ctypes.byref(w64), y, 8, gs, None, need, None) == -4
    # LoRA branch: rank-128 operands are required; the fused call only takes tiled shapes
    tb = ctypes.c_void_p(0x80000)
    lw = ctypes.c_void_p(0x90000)
    assert nv.nvfp4_workspace_bytes(nv.OP_LORA_DOWN, 3520, 3072) == 8 * 3584 * 128 * 4          # 28 row tiles x 8 K ranges
    assert L.nvfp4_lora_down(None, 4, 32, 32, tb, tb, lw, 1 << 20, None) == -1
    assert L.nvfp4_lora_down(y, 4, 24, 24, tb, tb, lw, 1 << 20, None) == -2                      # K % 16
    assert L.nvfp4_lora_down(y, 4, 32, 36, tb, tb, lw, 1 << 20, None) == -3                      # ldx % 8
    assert L.nvfp4_lora_down(y, 4, 32, 32, tb, tb, lw, 100, None) == -4
    assert L.nvfp4_gemm_lora(ctypes.byref(a), ctypes.byref(w), None, tb, 1.0, y, 8, 0, None) == -1
    assert L.nvfp4_gemm_lora(ctypes.byref(a), ctypes.byref(w), tb, tb, 1.0, y, 8, 0, None) == -2  # K = 32 is not a multiple of 64
    a64, w64 = _t(rows=4, K=64), _t(rows=8, K=64)
    assert L.nvfp4_gemm_lora(ctypes.byref(a64), ctypes.byref(w64), tb, tb, 1.0, y, 4, 0, None) == -2   # ldy < N
    assert L.nvfp4_gemm_lora(ctypes.byref(a64), ctypes.byref(w64), tb, tb, 1.0, y, 8, 3, None) == -2   # bad dtype
    out = _t(rows=4, K=16)
    ws = ctypes.c_void_p(0x50000)
    assert L.nvfp4_gemm_act_quant(ctypes.byref(a), ctypes.byref(w), 1, None, ctypes.byref(out), None, ws, 1 << 20, None) == -2
    out = _t(rows=4, K=8)
    assert L.nvfp4_gemm_act_quant(ctypes.byref(a), ctypes.byref(w), 1, None, ctypes.byref(out), None, ws, 1 << 20, None) == -2
    w16 = _t(rows=16, K=32)
    out = _t(rows=4, K=16)
    assert L.nvfp4_gemm_act_quant(ctypes.byref(a), ctypes.byref(w16), 5, None, ctypes.byref(out), None, ws, 1 << 20, None) == -2
    assert L.nvfp4_gemm_act_quant(ctypes.byref(a), ctypes.byref(w16), 1, None, ctypes.byref(out), None, ws, 16, None) == -4
    kv = ctypes.c_void_p(0x60000)
    t = _t(rows=6, K=32)
    # all-to-all packer: the heads must divide over the peers
    a2a = lambda T_, H_, d_, P_, o: L.nvfp4_quantize_for_all_to_all(kv, T_, H_, d_, P_, None, ctypes.byref(o), ws, 4096, None)
    assert a2a(2, 3, 32, 2, t) == -2
    assert a2a(2, 3, 32, 0, t) == -2
    assert a2a(2, 4, 32, 2, t) == -2                                                  # rows != T*H
    # Hadamard-transformed weight-gradient operand: out is [C, R]; the sign mask has 16 bits
    rt = _t(rows=48, K=32)
    qr = lambda R, C, mask, o, wsp, wb: L.nvfp4_quantize_rht(kv, R, C, C, mask, None, ctypes.byref(o), wsp, wb, None)
    assert qr(32, 48, 0x1FFFF, rt, ws, 4096) == -2
    assert qr(32, 48, 0x5A5A, w2 if False else _t(rows=32, K=48), ws, 4096) == -2      # out not transposed
    assert qr(24, 48, 0x5A5A, _t(rows=48, K=24), ws, 4096) == -2                      # R % 16
    assert qr(32, 48, 0x5A5A, rt, None, 0) == -4
    # 2-D weight scaling: both sides multiples of 16, shapes of both outputs
    w2 = _t(rows=32, K=48)
    w2t = _t(rows=48, K=32)
    q2 = lambda R, C, o, ot, wsp, wb: L.nvfp4_quantize_2d(kv, R, C, C, None, ctypes.byref(o), ctypes.byref(ot) if ot else None, wsp, wb, None)
    assert q2(32, 48, w2, _t(rows=32, K=48), ws, 4096) == -2         # transposed output has the wrong shape
    assert q2(24, 48, _t(rows=24, K=48), None, ws, 4096) == -2       # R % 16
    assert q2(32, 48, w2, w2t, None, 0) == -4
    assert L.nvfp4_quantize_2d(None, 32, 48, 48, None, ctypes.byref(w2), None, ws, 4096, None) == -1
    # smoothed keys: d / 16 must be a power of two <= 64; the means are required
    mean = ctypes.c_void_p(0x70000)
    t48 = _t(rows=6, K=48)
    assert L.nvfp4_kv_quant_k(kv, 2, 3, 48, ctypes.byref(t48), mean, ws, 4096, None) == -2
    assert L.nvfp4_kv_quant_k(kv, 2, 3, 32, ctypes.byref(t), None, ws, 4096, None) == -1
    assert L.nvfp4_kv_quant_k(kv, 2, 3, 32, ctypes.byref(t), mean, ws, 8, None) == -4
    assert L.nvfp4_kv_quant_k(kv, 2, 4, 32, ctypes.byref(t), mean, ws, 4096, None) == -2          # rows != T*H
    # gathered reconstruction: chunk count and per-chunk shapes
    from paper_2605_18739_amd.binding import _CKvChunk
    ch = (_CKvChunk * 2)()
    ch[0].q, ch[0].row_mean_bf16, ch[0].T = t, None, 2
    ch[1].q, ch[1].row_mean_bf16, ch[1].T = t, 0x70000, 2
    assert L.nvfp4_kv_dequant_gather(ch, 0, kv, 3, 32, None) == -2
    assert L.nvfp4_kv_dequant_gather(ch, 65, kv, 3, 32, None) == -2
    assert L.nvfp4_kv_dequant_gather(ch, 2, None, 3, 32, None) == -1
    assert L.nvfp4_kv_dequant_gather(ch, 2, kv, 4, 32, None) == -2                                # rows != T*H
    ch[1].T = 3
    assert L.nvfp4_kv_dequant_gather(ch, 2, kv, 3, 32, None) == -2
    # the scale-search variants validate like their plain counterparts
    assert L.nvfp4_kv_quant_4over6(kv, 0, 3, 32, ctypes.byref(t), ws, 4096, None) == -2
    assert L.nvfp4_kv_quant_4over6(kv, 2, 3, 32, ctypes.byref(t), None, 0, None) == -4
    assert L.nvfp4_quantize_4over6(None, 6, 32, 32, None, ctypes.byref(t), ws, 4096, None) == -1
    assert L.nvfp4_quantize_4over6(kv, 6, 32, 16, None, ctypes.byref(t), ws, 4096, None) == -2     # ld < C
    assert L.nvfp4_quantize_4over6(kv, 6, 32, 32, None, ctypes.byref(t), ws, 16, None) == -4
    assert L.nvfp4_kv_quant(kv, 0, 3, 32, ctypes.byref(t), ws, 4096, None) == -2
    assert L.nvfp4_kv_quant(kv, 2, 3, 24, ctypes.byref(_t(rows=6, K=24)), ws, 4096, None) == -2
    assert L.nvfp4_kv_dequant(ctypes.byref(t), None, 2, 3, 32, None) == -1
    assert L.nvfp4_kv_dequant(ctypes.byref(t), kv, 2, 4, 32, None) == -2


def test_gemm_launch_plan():
    """Host logic of the GEMM tiling: whole waves of large tiles on the 256 compute units, the
    leftover rectangle on smaller tiles, every output covered exactly once."""
    # the DiT FFN pair of the benchmark: 784 tiles of 256x256 = 3 waves + 16; the last 16 tile
    # positions (192 valid rows x 4096 columns) run as 3 x 64 tiles of 64x64
    assert nv.nvfp4_gemm_plan(3520, 14336, 3072) == [("256x256", 768), ("64x64", 192)]
    assert nv.nvfp4_gemm_plan(3520, 3072, 14336) == [("256x192", 224)]
    # the training layer's weight gradient: 672 tiles = 2.6 waves; 42 whole tile rows (two waves, the
    # second 97 % full), then the 14 tile rows below as one wave of 256x192 tiles
    assert nv.nvfp4_gemm_plan(14336, 3072, 17600) == [("256x256", 504), ("256x192", 224)]
    assert nv.nvfp4_gemm_plan(64, 64, 48) == [("generic", 0)]          # K % 64 != 0
    assert nv.nvfp4_gemm_plan(130, 260, 128) == [("generic", 0)]       # N % 8 != 0
    rng = np.random.default_rng(5)
    seen = set()
    for _ in range(300):
        M, N = int(rng.integers(1, 20000)), int(rng.integers(1, 2500)) * 8
        K = int(rng.integers(1, 64)) * 64
        plan = nv.nvfp4_gemm_plan(M, N, K)
        bm, bn = (int(v) for v in plan[0][0].split("x"))
        tiles_n = -(-N // bn)
        main = plan[0][1]
        assert main <= -(-M // bm) * tiles_n
        if len(plan) == 1:
            assert main == -(-M // bm) * tiles_n
        else:
            # the main launch is a whole number of waves and stops inside tile row q at column c,
            # or it ends with tile row q - 1 (c = 0); the other launches tile [row q, from column c]
            # and [rows below] completely
            assert main % 256 == 0 or main % tiles_n == 0
            q, c = divmod(main, tiles_n)
            rects = []
            if c:
                rects.append((min(M, (q + 1) * bm) - q * bm, N - c * bn))
            below = M - (q + (1 if c else 0)) * bm
            if below > 0:
                rects.append((below, N))
            assert len(rects) == len(plan) - 1
            for (rm, rn), (tile, wgs) in zip(rects, plan[1:]):
                tm, tn = (int(v) for v in tile.split("x"))
                assert wgs == -(-rm // tm) * -(-rn // tn)
        seen.update(t for t, _ in plan)
        # the fused call keeps one partial maximum per workgroup in its workspace
        assert nv.nvfp4_workspace_bytes(nv.OP_GEMM_ACT_QUANT, M, N, 1) >= 4 * sum(w for _, w in plan)
    assert seen == {"256x256", "256x192", "128x128", "64x64"}
    for M, N, K in [(300100, 264, 14336), (72, 300104, 14336), (1, 8, 64), (65, 72, 64)]:
        assert nv.nvfp4_workspace_bytes(nv.OP_GEMM_ACT_QUANT, M, N, 1) >= 4 * sum(w for _, w in nv.nvfp4_gemm_plan(M, N, K))
    text = ctypes.create_string_buffer(4)
    assert nv.lib().nvfp4_gemm_plan(3520, 14336, 3072, text, 4) == -4    # text does not fit
    assert nv.lib().nvfp4_gemm_plan(3520, 14336, 3072, None, 64) == -1
    assert nv.lib().nvfp4_gemm_plan(3520, 14336, 3070, text, 4) == -2


def test_binding_fails_loudly_without_the_library(monkeypatch):
    from paper_2605_18739_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libnvfp4_hip.so")
    with pytest.raises(binding.NVFP4Error):
        binding.lib()
