"""ctypes loader for the NVFP4 CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Thin numpy marshalling around nvfp4_oracle.c (compiled with gcc by build());
no arithmetic of the method lives here.  Only tests, the smoke check and the
bench's cpu_baseline leg may import this module.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nvfp4_oracle.c")
_LIB = os.path.join(_HERE, "libnvfp4_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2 -fopenmp, no fused multiply-add: every fp64 operation
    rounds on its own, as written); returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        c = ctypes
        u8p, u16p, f32p, f64p, i64p = (c.POINTER(t) for t in
                                       (c.c_uint8, c.c_uint16, c.c_float, c.c_double, c.c_int64))
        i64 = c.c_int64
        L.nvfp4o_e2m1_decode.restype = c.c_double
        L.nvfp4o_e2m1_decode.argtypes = [c.c_uint]
        L.nvfp4o_e4m3_decode.restype = c.c_double
        L.nvfp4o_e4m3_decode.argtypes = [c.c_uint]
        L.nvfp4o_bf16_decode.restype = c.c_double
        L.nvfp4o_bf16_decode.argtypes = [c.c_uint16]
        L.nvfp4o_bf16_rne.restype = c.c_uint16
        L.nvfp4o_bf16_rne.argtypes = [c.c_double]
        L.nvfp4o_e4m3_cast_ratio.restype = c.c_int
        L.nvfp4o_e4m3_cast_ratio.argtypes = [c.c_double, c.c_double]
        L.nvfp4o_e2m1_cast_ratio.restype = c.c_int
        L.nvfp4o_e2m1_cast_ratio.argtypes = [c.c_double, c.c_double]
        L.nvfp4o_global_scale.restype = c.c_float
        L.nvfp4o_global_scale.argtypes = [u16p, i64, i64, i64]
        L.nvfp4o_quantize.restype = None
        L.nvfp4o_quantize.argtypes = [u16p, i64, i64, i64, c.c_int, f32p, u8p, u8p, f32p]
        L.nvfp4o_quantize_2d.restype = None
        L.nvfp4o_quantize_2d.argtypes = [u16p, i64, i64, i64, f32p, u8p, u8p, u8p, u8p, f32p]
        L.nvfp4o_quantize_4over6.restype = None
        L.nvfp4o_quantize_4over6.argtypes = [u16p, i64, i64, i64, f32p, u8p, u8p, f32p]
        L.nvfp4o_dequant_f64.restype = None
        L.nvfp4o_dequant_f64.argtypes = [u8p, u8p, c.c_float, i64, i64, f64p]
        L.nvfp4o_dequant_bf16.restype = None
        L.nvfp4o_dequant_bf16.argtypes = [u8p, u8p, c.c_float, i64, i64, u16p]
        L.nvfp4o_lora_down.restype = None
        L.nvfp4o_lora_down.argtypes = [u16p, u16p, i64, i64, i64, u16p]
        L.nvfp4o_lora_up_add.restype = None
        L.nvfp4o_lora_up_add.argtypes = [u16p, u16p, i64, i64, c.c_double, c.POINTER(c.c_int64), i64,
                                         c.POINTER(c.c_double), c.POINTER(c.c_double)]
        L.nvfp4o_rht_rows.restype = None
        L.nvfp4o_rht_rows.argtypes = [u16p, i64, i64, i64, c.c_uint, u16p]
        L.nvfp4o_kv_smooth.restype = None
        L.nvfp4o_kv_smooth.argtypes = [u16p, i64, i64, u16p, u16p]
        L.nvfp4o_dequant_bf16_smooth.restype = None
        L.nvfp4o_dequant_bf16_smooth.argtypes = [u8p, u8p, c.c_float, u16p, i64, i64, u16p]
        L.nvfp4o_gemm.restype = None
        L.nvfp4o_gemm.argtypes = [u8p, u8p, c.c_float, u8p, u8p, c.c_float, i64, i64, i64,
                                  i64p, i64, f64p, f64p]
        L.nvfp4o_gelu_tanh.restype = c.c_double
        L.nvfp4o_gelu_tanh.argtypes = [c.c_double]
        L.nvfp4o_gelu_tanh_bf16.restype = None
        L.nvfp4o_gelu_tanh_bf16.argtypes = [f64p, i64, u16p]
        L.nvfp4o_num_threads.restype = c.c_int
        L.nvfp4o_num_threads.argtypes = []
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _u16(x):
    x = np.ascontiguousarray(x)
    assert x.dtype == np.uint16 and x.ndim == 2
    return x


class Q:
    """Host NVFP4 tensor: codes [rows, K/2] u8, scales [rows, K/16] u8, global_scale f32."""

    def __init__(self, codes, scales, global_scale):
        self.codes, self.scales, self.global_scale = codes, scales, np.float32(global_scale)
        self.rows, self.K = codes.shape[0], codes.shape[1] * 2


def global_scale(x_bits):
    x = _u16(x_bits)
    return np.float32(lib().nvfp4o_global_scale(_p(x, ctypes.c_uint16), x.shape[0], x.shape[1], x.shape[1]))


def quantize(x_bits, block_axis=0, global_scale_in=None, four_over_six=False):
    """x_bits: uint16 [R, C] bf16 bit patterns."""
    x = _u16(x_bits)
    R, C = x.shape
    rows, K = (R, C) if block_axis == 0 else (C, R)
    assert K % 16 == 0
    codes = np.empty((rows, K // 2), np.uint8)
    scales = np.empty((rows, K // 16), np.uint8)
    gs_out = ctypes.c_float(0)
    gs_in = None
    if global_scale_in is not None:
        gs_in = ctypes.pointer(ctypes.c_float(float(global_scale_in)))
    if four_over_six:
        assert block_axis == 0
        lib().nvfp4o_quantize_4over6(_p(x, ctypes.c_uint16), R, C, C, gs_in,
                                     _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8),
                                     ctypes.byref(gs_out))
    else:
        lib().nvfp4o_quantize(_p(x, ctypes.c_uint16), R, C, C, block_axis, gs_in,
                              _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8),
                              ctypes.byref(gs_out))
    return Q(codes, scales, gs_out.value)


def dequant_f64(q):
    out = np.empty((q.rows, q.K), np.float64)
    lib().nvfp4o_dequant_f64(_p(np.ascontiguousarray(q.codes), ctypes.c_uint8),
                             _p(np.ascontiguousarray(q.scales), ctypes.c_uint8),
                             ctypes.c_float(float(q.global_scale)), q.rows, q.K,
                             _p(out, ctypes.c_double))
    return out


def quantize_2d(x_bits, global_scale_in=None):
    """Weights with one scale per 16x16 tile (Sec. 2.2 training recipe): returns (Q of [R, C], Q of [C, R])."""
    x = _u16(x_bits)
    R, C = x.shape
    assert R % 16 == 0 and C % 16 == 0
    codes, scales = np.empty((R, C // 2), np.uint8), np.empty((R, C // 16), np.uint8)
    codes_t, scales_t = np.empty((C, R // 2), np.uint8), np.empty((C, R // 16), np.uint8)
    gs_out = ctypes.c_float(0)
    gs_in = None
    if global_scale_in is not None:
        gs_in = ctypes.pointer(ctypes.c_float(float(global_scale_in)))
    lib().nvfp4o_quantize_2d(_p(x, ctypes.c_uint16), R, C, C, gs_in, _p(codes, ctypes.c_uint8),
                             _p(scales, ctypes.c_uint8), _p(codes_t, ctypes.c_uint8),
                             _p(scales_t, ctypes.c_uint8), ctypes.byref(gs_out))
    return Q(codes, scales, gs_out.value), Q(codes_t, scales_t, gs_out.value)


def rht_rows(x_bits, sign_mask):
    """Random Hadamard transform along the rows (groups of 16) of x_bits [R, C]; returns bf16 bits [R, C]."""
    x = _u16(x_bits)
    R, C = x.shape
    assert R % 16 == 0
    out = np.empty((R, C), np.uint16)
    lib().nvfp4o_rht_rows(_p(x, ctypes.c_uint16), R, C, C, int(sign_mask) & 0xFFFF, _p(out, ctypes.c_uint16))
    return out


def kv_smooth(x_bits):
    """K-smoothing (Sec. 3.2, Eq. 6): x_bits uint16 [rows, d] -> (mean bits [rows], smoothed bits [rows, d])."""
    x = _u16(x_bits)
    rows, d = x.shape
    mean = np.empty(rows, np.uint16)
    xbar = np.empty((rows, d), np.uint16)
    lib().nvfp4o_kv_smooth(_p(x, ctypes.c_uint16), rows, d, _p(mean, ctypes.c_uint16), _p(xbar, ctypes.c_uint16))
    return mean, xbar


def dequant_bf16(q, mean_bits=None):
    out = np.empty((q.rows, q.K), np.uint16)
    if mean_bits is not None:
        mean = np.ascontiguousarray(mean_bits, dtype=np.uint16)
        assert mean.shape == (q.rows,)
        lib().nvfp4o_dequant_bf16_smooth(_p(np.ascontiguousarray(q.codes), ctypes.c_uint8),
                                         _p(np.ascontiguousarray(q.scales), ctypes.c_uint8),
                                         ctypes.c_float(float(q.global_scale)), _p(mean, ctypes.c_uint16),
                                         q.rows, q.K, _p(out, ctypes.c_uint16))
        return out
    lib().nvfp4o_dequant_bf16(_p(np.ascontiguousarray(q.codes), ctypes.c_uint8),
                              _p(np.ascontiguousarray(q.scales), ctypes.c_uint8),
                              ctypes.c_float(float(q.global_scale)), q.rows, q.K,
                              _p(out, ctypes.c_uint16))
    return out


def gemm(qa, qw, rows=None, want_abs=True):
    """Returns (Y, S) float64 [len(rows) or M, N]."""
    assert qa.K == qw.K
    M, N, K = qa.rows, qw.rows, qa.K
    rp, nr = None, 0
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rp, nr = _p(rows, ctypes.c_int64), len(rows)
    n_out = nr if rows is not None else M
    Y = np.empty((n_out, N), np.float64)
    S = np.empty((n_out, N), np.float64) if want_abs else None
    lib().nvfp4o_gemm(_p(np.ascontiguousarray(qa.codes), ctypes.c_uint8),
                      _p(np.ascontiguousarray(qa.scales), ctypes.c_uint8),
                      ctypes.c_float(float(qa.global_scale)),
                      _p(np.ascontiguousarray(qw.codes), ctypes.c_uint8),
                      _p(np.ascontiguousarray(qw.scales), ctypes.c_uint8),
                      ctypes.c_float(float(qw.global_scale)),
                      M, N, K, rp, nr, _p(Y, ctypes.c_double),
                      _p(S, ctypes.c_double) if want_abs else None)
    return Y, S


def lora_down(x_bits, a_bits):
    """T = RN_bf16(X A^T): x_bits [M, K], a_bits [r, K] bf16 bit patterns -> [M, r]."""
    x, a = _u16(x_bits), _u16(a_bits)
    (M, K), (r, K2) = x.shape, a.shape
    assert K == K2
    t = np.empty((M, r), np.uint16)
    lib().nvfp4o_lora_down(_p(x, ctypes.c_uint16), _p(a, ctypes.c_uint16), M, K, r, _p(t, ctypes.c_uint16))
    return t


def gemm_lora(qa, qw, t_bits, b_bits, scale, rows=None):
    """GEMM of the quantized operands plus scale * T B^T (T [M, r], B [N, r] bf16 bits). Returns (Y, S)."""
    Y, S = gemm(qa, qw, rows=rows)
    t, b = _u16(t_bits), _u16(b_bits)
    assert t.shape[0] == qa.rows and b.shape[0] == qw.rows and t.shape[1] == b.shape[1]
    rp, nr = None, qa.rows
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rp, nr = _p(rows, ctypes.c_int64), len(rows)
    lib().nvfp4o_lora_up_add(_p(t, ctypes.c_uint16), _p(b, ctypes.c_uint16), qw.rows, t.shape[1], float(scale),
                             rp, nr, _p(Y, ctypes.c_double), _p(S, ctypes.c_double))
    return Y, S


def gelu_tanh_bf16(y):
    y = np.ascontiguousarray(y, dtype=np.float64)
    h = np.empty(y.shape, np.uint16)
    lib().nvfp4o_gelu_tanh_bf16(_p(y, ctypes.c_double), y.size, _p(h, ctypes.c_uint16))
    return h


def bf16_rne(v):
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(v.shape, np.uint16)
    f = lib().nvfp4o_bf16_rne
    flat_in, flat_out = v.ravel(), out.ravel()
    for i in range(flat_in.size):
        flat_out[i] = f(float(flat_in[i]))
    return out


def num_threads():
    return int(lib().nvfp4o_num_threads())
