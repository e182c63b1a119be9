"""ctypes binding of the NVFP4 HIP library: argument marshalling only.

Function names mirror the C ABI in include/nvfp4.h.  torch supplies device
memory and the current stream; every step of the path runs in the library's
kernels.  There is no CPU fallback: if the shared library is missing, importing
this module's entry points raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnvfp4_hip.so")
_lib = None

OUT_F32, OUT_BF16 = 0, 1
ACT_NONE, ACT_GELU_TANH = 0, 1
OP_QUANTIZE, OP_KV_QUANT, OP_GEMM_ACT_QUANT, OP_GEMM, OP_KV_DEQUANT, OP_GEMM_ACT_QUANT_GEMM = 0, 1, 2, 3, 4, 5
OP_QUANTIZE_4OVER6, OP_KV_QUANT_4OVER6, OP_KV_QUANT_K, OP_KV_DEQUANT_GATHER = 6, 7, 8, 9
KV_MAX_CHUNKS = 64
NOALLOC_MAX_ELEMENTS = 1 << 32
OP_QUANTIZE_2D, OP_QUANTIZE_RHT, OP_QUANTIZE_A2A, OP_LORA_DOWN, OP_GEMM_LORA, OP_PROBE = 10, 11, 12, 13, 14, 15
OP_GEMM_SCALE_OUT = 16
LORA_RANK = 128


class _CTensor(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("global_scale", ctypes.c_void_p), ("rows", ctypes.c_int64), ("K", ctypes.c_int64)]


class _CKvChunk(ctypes.Structure):
    _fields_ = [("q", _CTensor), ("row_mean_bf16", ctypes.c_void_p), ("T", ctypes.c_int64)]


class NVFP4Error(RuntimeError):
    pass


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise NVFP4Error(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2605_18739_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(_LIB_PATH)
        c = ctypes
        vp, i64, sz = c.c_void_p, c.c_int64, c.c_size_t
        tp = c.POINTER(_CTensor)
        L.nvfp4_quantize.restype = c.c_int
        L.nvfp4_quantize.argtypes = [vp, i64, i64, i64, c.c_int, vp, tp, vp, sz, vp]
        L.nvfp4_gemm.restype = c.c_int
        L.nvfp4_gemm.argtypes = [tp, tp, vp, i64, c.c_int, vp]
        L.nvfp4_gemm_scale_out.restype = c.c_int
        L.nvfp4_gemm_scale_out.argtypes = [tp, tp, vp, i64, vp, vp, sz, vp]
        L.nvfp4_lora_down.restype = c.c_int
        L.nvfp4_lora_down.argtypes = [vp, i64, i64, i64, vp, vp, vp, sz, vp]
        L.nvfp4_gemm_lora.restype = c.c_int
        L.nvfp4_gemm_lora.argtypes = [tp, tp, vp, vp, c.c_float, vp, i64, c.c_int, vp]
        L.nvfp4_gemm_act_quant.restype = c.c_int
        L.nvfp4_gemm_act_quant.argtypes = [tp, tp, c.c_int, vp, tp, vp, vp, sz, vp]
        L.nvfp4_kv_quant.restype = c.c_int
        L.nvfp4_kv_quant.argtypes = [vp, i64, i64, i64, tp, vp, sz, vp]
        L.nvfp4_kv_quant_noalloc.restype = c.c_int
        L.nvfp4_kv_quant_noalloc.argtypes = [vp, i64, i64, i64, tp, vp]
        L.nvfp4_kv_dequant.restype = c.c_int
        L.nvfp4_kv_dequant.argtypes = [tp, vp, i64, i64, i64, vp]
        L.nvfp4_quantize_4over6.restype = c.c_int
        L.nvfp4_quantize_4over6.argtypes = [vp, i64, i64, i64, vp, tp, vp, sz, vp]
        L.nvfp4_kv_quant_4over6.restype = c.c_int
        L.nvfp4_kv_quant_4over6.argtypes = [vp, i64, i64, i64, tp, vp, sz, vp]
        L.nvfp4_quantize_for_all_to_all.restype = c.c_int
        L.nvfp4_quantize_for_all_to_all.argtypes = [vp, i64, i64, i64, i64, vp, tp, vp, sz, vp]
        L.nvfp4_quantize_rht.restype = c.c_int
        L.nvfp4_quantize_rht.argtypes = [vp, i64, i64, i64, c.c_uint32, vp, tp, vp, sz, vp]
        L.nvfp4_quantize_2d.restype = c.c_int
        L.nvfp4_quantize_2d.argtypes = [vp, i64, i64, i64, vp, tp, tp, vp, sz, vp]
        L.nvfp4_kv_quant_k.restype = c.c_int
        L.nvfp4_kv_quant_k.argtypes = [vp, i64, i64, i64, tp, vp, vp, sz, vp]
        L.nvfp4_kv_dequant_gather.restype = c.c_int
        L.nvfp4_kv_dequant_gather.argtypes = [c.POINTER(_CKvChunk), c.c_int, vp, i64, i64, vp]
        L.nvfp4_workspace_bytes.restype = sz
        L.nvfp4_workspace_bytes.argtypes = [c.c_int, i64, i64, i64]
        L.nvfp4_status_string.restype = c.c_char_p
        L.nvfp4_status_string.argtypes = [c.c_int]
        L.nvfp4_gemm_plan.restype = c.c_int
        L.nvfp4_gemm_plan.argtypes = [i64, i64, i64, c.c_char_p, sz]
        L.nvfp4_set_timing.restype = None
        L.nvfp4_set_timing.argtypes = [c.c_int]
        L.nvfp4_set_timing_ops.restype = None
        L.nvfp4_set_timing_ops.argtypes = [c.c_uint32]
        L.nvfp4_timing_read.restype = c.c_int
        L.nvfp4_timing_read.argtypes = [c.c_int, c.POINTER(c.c_int), c.POINTER(c.c_float)]
        L.nvfp4_timing_read_all.restype = c.c_int
        L.nvfp4_timing_read_all.argtypes = [c.c_int, c.POINTER(c.c_float), c.c_int]
        L.nvfp4_set_one_launch.restype = c.c_int
        L.nvfp4_set_one_launch.argtypes = [c.c_int]
        L.nvfp4_set_sync_spin_limit.restype = None
        L.nvfp4_set_sync_spin_limit.argtypes = [c.c_uint32]
        L.nvfp4_probe.restype = c.c_int
        L.nvfp4_probe.argtypes = [c.c_int, vp, vp, sz, c.c_int, vp]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise NVFP4Error(f"nvfp4 status {rc}: {lib().nvfp4_status_string(rc).decode()}")


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


class NVFP4Tensor:
    """Device NVFP4 tensor: codes [rows, K/2] u8, scales [rows, K/16] u8, global_scale [1] f32."""

    def __init__(self, rows, K, device="cuda", codes=None, scales=None, global_scale=None):
        self.rows, self.K = int(rows), int(K)
        self.codes = codes if codes is not None else torch.empty((rows, K // 2), dtype=torch.uint8, device=device)
        self.scales = scales if scales is not None else torch.empty((rows, K // 16), dtype=torch.uint8, device=device)
        self.global_scale = (global_scale if global_scale is not None
                             else torch.empty(1, dtype=torch.float32, device=device))

    def c(self):
        return _CTensor(self.codes.data_ptr(), self.scales.data_ptr(), self.global_scale.data_ptr(),
                        self.rows, self.K)

    @staticmethod
    def from_host(codes_np, scales_np, global_scale, device="cuda"):
        codes = torch.from_numpy(codes_np).to(device)
        scales = torch.from_numpy(scales_np).to(device)
        gs = torch.tensor([float(global_scale)], dtype=torch.float32, device=device)
        return NVFP4Tensor(codes.shape[0], codes.shape[1] * 2, device, codes, scales, gs)


def nvfp4_workspace_bytes(op, a, b=0, c=0):
    return int(lib().nvfp4_workspace_bytes(op, a, b, c))


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def nvfp4_quantize(x, block_axis=0, global_scale_in=None, out=None, workspace=None, stream=None):
    """x: bf16 [R, C] device tensor with unit stride along C. Returns an NVFP4Tensor."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1
    R, C = x.shape
    ld = x.stride(0)
    rows, K = (R, C) if block_axis == 0 else (C, R)
    if out is None:
        out = NVFP4Tensor(rows, K, x.device)
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_QUANTIZE, R, C), x.device)
    ct = out.c()
    _check(lib().nvfp4_quantize(_ptr(x), R, C, ld, block_axis, _ptr(global_scale_in), ctypes.byref(ct),
                                _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def nvfp4_gemm(A, W, out_dtype=OUT_F32, Y=None, stream=None):
    M, N = A.rows, W.rows
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.float32 if out_dtype == OUT_F32 else torch.bfloat16,
                        device=A.codes.device)
    ca, cw = A.c(), W.c()
    _check(lib().nvfp4_gemm(ctypes.byref(ca), ctypes.byref(cw), _ptr(Y), Y.stride(0), out_dtype,
                            _stream(stream)))
    return Y


def nvfp4_gemm_scale_out(A, W, Y=None, scale_out=None, workspace=None, stream=None):
    """bf16 Y = A W^T together with the NVFP4 tensor scale of Y (one float on the device).  Returns (Y, scale_out)."""
    M, N = A.rows, W.rows
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=A.codes.device)
    if scale_out is None:
        scale_out = torch.empty(1, dtype=torch.float32, device=A.codes.device)
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_GEMM_SCALE_OUT, M, N), A.codes.device)
    ca, cw = A.c(), W.c()
    _check(lib().nvfp4_gemm_scale_out(ctypes.byref(ca), ctypes.byref(cw), _ptr(Y), Y.stride(0), _ptr(scale_out),
                                      _ptr(workspace), workspace.numel(), _stream(stream)))
    return Y, scale_out


def nvfp4_lora_down(x, a, out=None, workspace=None, stream=None):
    """T = bf16(x a^T): x bf16 [M, K] (unit stride along K), a bf16 [128, K] contiguous."""
    assert x.dtype == torch.bfloat16 and a.dtype == torch.bfloat16 and x.stride(1) == 1 and a.is_contiguous()
    M, K = x.shape
    assert a.shape == (LORA_RANK, K)
    if out is None:
        out = torch.empty((M, LORA_RANK), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_LORA_DOWN, M, K), x.device)
    _check(lib().nvfp4_lora_down(_ptr(x), M, K, x.stride(0), _ptr(a), _ptr(out), _ptr(workspace), workspace.numel(),
                                 _stream(stream)))
    return out


def nvfp4_gemm_lora(A, W, t, b, lora_scale, out_dtype=OUT_F32, Y=None, stream=None):
    """nvfp4_gemm(A, W) + lora_scale * t b^T, fused; t bf16 [M, 128], b bf16 [N, 128], both contiguous."""
    M, N = A.rows, W.rows
    assert t.is_contiguous() and b.is_contiguous() and t.shape == (M, LORA_RANK) and b.shape == (N, LORA_RANK)
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.float32 if out_dtype == OUT_F32 else torch.bfloat16,
                        device=A.codes.device)
    ca, cw = A.c(), W.c()
    _check(lib().nvfp4_gemm_lora(ctypes.byref(ca), ctypes.byref(cw), _ptr(t), _ptr(b), float(lora_scale), _ptr(Y),
                                 Y.stride(0), out_dtype, _stream(stream)))
    return Y


def nvfp4_gemm_act_quant(A, W, act=ACT_GELU_TANH, global_scale_in=None, out=None, h_bf16=None,
                         workspace=None, stream=None):
    M, N = A.rows, W.rows
    dev = A.codes.device
    if out is None:
        out = NVFP4Tensor(M, N, dev)
    if workspace is None:
        flags = (1 if h_bf16 is not None else 0) | (2 if (global_scale_in is not None and A.K % 64 == 0) else 0)
        workspace = _workspace(nvfp4_workspace_bytes(OP_GEMM_ACT_QUANT, M, N, flags), dev)
    ca, cw, co = A.c(), W.c(), out.c()
    _check(lib().nvfp4_gemm_act_quant(ctypes.byref(ca), ctypes.byref(cw), act, _ptr(global_scale_in),
                                      ctypes.byref(co), _ptr(h_bf16), _ptr(workspace), workspace.numel(),
                                      _stream(stream)))
    return out


def nvfp4_kv_quant(kv, out=None, workspace=None, stream=None):
    """kv: contiguous bf16 [T, H, d]."""
    assert kv.dtype == torch.bfloat16 and kv.dim() == 3 and kv.is_contiguous()
    T, H, d = kv.shape
    if out is None:
        out = NVFP4Tensor(T * H, d, kv.device)
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_KV_QUANT, T, H, d), kv.device)
    ct = out.c()
    _check(lib().nvfp4_kv_quant(_ptr(kv), T, H, d, ctypes.byref(ct), _ptr(workspace), workspace.numel(),
                                _stream(stream)))
    return out


def nvfp4_kv_quant_noalloc(kv, out, stream=None):
    """kv: contiguous bf16 [T, H, d]; `out` must be given: this entry point (and this wrapper) allocates nothing."""
    assert kv.dtype == torch.bfloat16 and kv.dim() == 3 and kv.is_contiguous()
    T, H, d = kv.shape
    ct = out.c()
    _check(lib().nvfp4_kv_quant_noalloc(_ptr(kv), T, H, d, ctypes.byref(ct), _stream(stream)))
    return out


def nvfp4_quantize_4over6(x, global_scale_in=None, out=None, workspace=None, stream=None):
    """x: bf16 [R, C] device tensor with unit stride along C; blocks along C, scale search per block."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1
    R, C = x.shape
    if out is None:
        out = NVFP4Tensor(R, C, x.device)
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_QUANTIZE_4OVER6, R, C), x.device)
    ct = out.c()
    _check(lib().nvfp4_quantize_4over6(_ptr(x), R, C, x.stride(0), _ptr(global_scale_in), ctypes.byref(ct),
                                       _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def nvfp4_kv_quant_4over6(kv, out=None, workspace=None, stream=None):
    """kv: contiguous bf16 [T, H, d]; scale search per block."""
    assert kv.dtype == torch.bfloat16 and kv.dim() == 3 and kv.is_contiguous()
    T, H, d = kv.shape
    if out is None:
        out = NVFP4Tensor(T * H, d, kv.device)
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_KV_QUANT_4OVER6, T, H, d), kv.device)
    ct = out.c()
    _check(lib().nvfp4_kv_quant_4over6(_ptr(kv), T, H, d, ctypes.byref(ct), _ptr(workspace), workspace.numel(),
                                       _stream(stream)))
    return out


def nvfp4_quantize_for_all_to_all(x, P, global_scale_in=None, out=None, workspace=None, stream=None):
    """x: contiguous bf16 [T, H, d]; NVFP4 along d, rows regrouped into P per-destination slabs of H/P heads."""
    assert x.dtype == torch.bfloat16 and x.dim() == 3 and x.is_contiguous()
    T, H, d = x.shape
    if out is None:
        out = NVFP4Tensor(T * H, d, x.device)
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_QUANTIZE_A2A, T, H, d), x.device)
    ct = out.c()
    _check(lib().nvfp4_quantize_for_all_to_all(_ptr(x), T, H, d, P, _ptr(global_scale_in), ctypes.byref(ct),
                                               _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def nvfp4_quantize_rht(x, sign_mask, global_scale_in=None, out=None, workspace=None, stream=None):
    """x: bf16 [R, C], contracted over R.  Random Hadamard transform along R (groups of 16) with the
    16-bit sign mask, then the transposed quantizer: returns NVFP4Tensor [C, R]."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1
    R, C = x.shape
    if out is None:
        out = NVFP4Tensor(C, R, x.device)
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_QUANTIZE_RHT, R, C), x.device)
    ct = out.c()
    _check(lib().nvfp4_quantize_rht(_ptr(x), R, C, x.stride(0), int(sign_mask), _ptr(global_scale_in),
                                    ctypes.byref(ct), _ptr(workspace), workspace.numel(), _stream(stream)))
    return out


def nvfp4_quantize_2d(w, global_scale_in=None, transposed=True, workspace=None, stream=None):
    """w: bf16 [R, C] weights (R, C multiples of 16), one scale per 16x16 tile.
    Returns (NVFP4Tensor [R, C], NVFP4Tensor [C, R] or None)."""
    assert w.dtype == torch.bfloat16 and w.dim() == 2 and w.stride(1) == 1
    R, C = w.shape
    out = NVFP4Tensor(R, C, w.device)
    out_t = NVFP4Tensor(C, R, w.device) if transposed else None
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_QUANTIZE_2D, R, C), w.device)
    co = out.c()
    ct = out_t.c() if transposed else None
    _check(lib().nvfp4_quantize_2d(_ptr(w), R, C, w.stride(0), _ptr(global_scale_in), ctypes.byref(co),
                                   ctypes.byref(ct) if transposed else None, _ptr(workspace), workspace.numel(),
                                   _stream(stream)))
    return out, out_t


def nvfp4_kv_quant_k(k, out=None, row_mean=None, workspace=None, stream=None):
    """k: contiguous bf16 [T, H, d] keys; K-smoothing then scale search.  Returns (NVFP4Tensor, row means bf16 [T*H])."""
    assert k.dtype == torch.bfloat16 and k.dim() == 3 and k.is_contiguous()
    T, H, d = k.shape
    if out is None:
        out = NVFP4Tensor(T * H, d, k.device)
    if row_mean is None:
        row_mean = torch.empty(T * H, dtype=torch.bfloat16, device=k.device)
    if workspace is None:
        workspace = _workspace(nvfp4_workspace_bytes(OP_KV_QUANT_K, T, H, d), k.device)
    ct = out.c()
    _check(lib().nvfp4_kv_quant_k(_ptr(k), T, H, d, ctypes.byref(ct), _ptr(row_mean), _ptr(workspace),
                                  workspace.numel(), _stream(stream)))
    return out, row_mean


def nvfp4_kv_dequant_gather(chunks, H, d, out=None, stream=None):
    """chunks: list of (NVFP4Tensor, row_mean or None, T).  Returns bf16 [sum T, H, d]."""
    n = len(chunks)
    arr = (_CKvChunk * n)()
    total = 0
    for i, (q, mean, T) in enumerate(chunks):
        arr[i].q = q.c()
        arr[i].row_mean_bf16 = mean.data_ptr() if mean is not None else None
        arr[i].T = T
        total += T
    if out is None:
        out = torch.empty((total, H, d), dtype=torch.bfloat16, device=chunks[0][0].codes.device)
    _check(lib().nvfp4_kv_dequant_gather(arr, n, _ptr(out), H, d, _stream(stream)))
    return out


def nvfp4_kv_dequant(q, T, H, d, out=None, stream=None):
    if out is None:
        out = torch.empty((T, H, d), dtype=torch.bfloat16, device=q.codes.device)
    ct = q.c()
    _check(lib().nvfp4_kv_dequant(ctypes.byref(ct), _ptr(out), T, H, d, _stream(stream)))
    return out


def nvfp4_gemm_plan(M, N, K):
    """-> list of (tile, workgroups) per launch, e.g. [("256x256", 768), ("64x64", 192)]; host only."""
    buf = ctypes.create_string_buffer(256)
    _check(min(lib().nvfp4_gemm_plan(M, N, K, buf, len(buf)), 0))
    return [(item.split(":")[0], int(item.split(":")[1])) if ":" in item else (item, 0)
            for item in buf.value.decode().split()]


def nvfp4_set_timing(enabled):
    lib().nvfp4_set_timing(1 if enabled else 0)


def nvfp4_set_timing_ops(ops):
    """Record events only around the entry points listed in `ops` (OP_* ids); an empty list: none."""
    mask = 0
    for op in ops:
        mask |= 1 << op
    lib().nvfp4_set_timing_ops(mask)


def nvfp4_timing_read(op):
    """-> (calls, total_ms) recorded for entry point `op` since timing was enabled."""
    n, ms = ctypes.c_int(0), ctypes.c_float(0)
    _check(lib().nvfp4_timing_read(op, ctypes.byref(n), ctypes.byref(ms)))
    return n.value, ms.value


ONE_LAUNCH_AUTO, ONE_LAUNCH_ALWAYS, ONE_LAUNCH_NEVER = 0, 1, 2


def nvfp4_set_one_launch(mode=ONE_LAUNCH_AUTO):
    """Form of the row quantizers for tensors that fit on the chip (see include/nvfp4.h)."""
    _check(lib().nvfp4_set_one_launch(int(mode)))


def nvfp4_set_sync_spin_limit(ticks_10ns=0xFFFFFFFF):
    """Bound of the grid-wide wait of the one-launch quantizers (10 ns ticks; 0: give up at once; default: restore)."""
    lib().nvfp4_set_sync_spin_limit(ticks_10ns)


def nvfp4_timing_read_all(op, max_records=8192):
    """-> list of the recorded durations (ms) of entry point `op`, in call order."""
    buf = (ctypes.c_float * max_records)()
    n = lib().nvfp4_timing_read_all(op, buf, max_records)
    _check(min(n, 0))
    return [buf[i] for i in range(n)]


PROBE_READ, PROBE_WRITE, PROBE_COPY, PROBE_MFMA = 0, 1, 2, 3
PROBE_MFMA_FLOPS_PER_ITER = 256 * 4 * 64 * 32768


def nvfp4_probe(kind, a, b, nbytes=0, iters=0, stream=None):
    """Ceiling probe (see include/nvfp4.h): a, b device tensors (a may be None for write / mfma)."""
    _check(lib().nvfp4_probe(kind, _ptr(a), _ptr(b), int(nbytes), int(iters), _stream(stream)))


def bf16_from_bits(bits_np, device="cuda"):
    """uint16 numpy bit patterns -> bf16 device tensor (a copy, no arithmetic)."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(bits_np).view(np.int16)).to(device)
    return t.view(torch.bfloat16)


def bits_from_bf16(t):
    import numpy as np
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
