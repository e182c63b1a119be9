"""Arithmetic facts the HIP kernels rely on, checked on the CPU with IEEE fp32 / fp64 (numpy)."""
import numpy as np


def _bf16_to_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _rne_f32_to_bf16(f):
    u = f.view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint32)


def _rne_f64_to_bf16(v):
    """One rounding (nearest even) of a float64 with a normal bf16 result, in integer arithmetic."""
    u = v.view(np.uint64)
    sign = (u >> 63).astype(np.uint32)
    e = ((u >> 52) & 0x7FF).astype(np.int64)
    m = (u & ((1 << 52) - 1)) | (1 << 52)
    q, rem, half = m >> 45, m & ((1 << 45) - 1), 1 << 44
    q = q + ((rem > half) | ((rem == half) & ((q & 1) == 1)))
    over = q >= 256
    q, e = np.where(over, q >> 1, q), e + over
    bits = (sign << 15) | ((e - 1023 + 127).astype(np.uint32) << 7) | (q.astype(np.uint32) & 0x7F)
    return np.where(v == 0, sign << 15, bits).astype(np.uint32)


def test_fp32_difference_of_bf16_rounds_like_the_exact_one():
    """K-smoothing (Sec. 3.2, Eq. 6) on the GPU subtracts the row mean in fp32 and rounds to bf16.
    For every pair of bf16 numbers that equals the single rounding of the exact difference: all
    mantissa pairs and signs, exponents up to 2^30 apart (fp64 holds those differences exactly)."""
    mant = np.arange(128, dtype=np.uint32)
    bad = total = 0
    for ex in (90, 127, 140):
        for gap in range(-30, 31):
            em = ex + gap
            for sx in (0, 1):
                for sm in (0, 1):
                    xb = ((sx << 15) | (ex << 7) | mant)[:, None] + np.zeros((1, 128), np.uint32)
                    mb = ((sm << 15) | (em << 7) | mant)[None, :] + np.zeros((128, 1), np.uint32)
                    x, mu = _bf16_to_f32(xb.ravel()), _bf16_to_f32(mb.ravel())
                    fast = _rne_f32_to_bf16((x - mu).astype(np.float32))
                    exact = _rne_f64_to_bf16(x.astype(np.float64) - mu.astype(np.float64))
                    bad += int((fast != exact).sum())
                    total += fast.size
    assert total > 10_000_000 and bad == 0
