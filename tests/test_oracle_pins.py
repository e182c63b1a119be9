"""Pins for the CPU oracle: everything here runs without a GPU and checks the
oracle against things other than itself -- values the paper prints, torch's
own float8/bfloat16 casts, exact rational brute force, closed forms."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2605_18739_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold_constants():
    out = {}
    for line in open(os.path.join(GOLD, "format_constants.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v)
    return out


def _gold_e2m1():
    for line in open(os.path.join(GOLD, "e2m1_values.txt")):
        if not line.startswith("#"):
            return [float(t) for t in line.split()]


E4M3_VALUES = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def bits(x):
    return wl.to_bf16_bits(np.asarray(x, dtype=np.float32))


# ------------------------------------------------------------------ formats

def test_e2m1_value_set_matches_paper(oracle):
    mags = _gold_e2m1()
    L = oracle.lib()
    assert [L.nvfp4o_e2m1_decode(c) for c in range(8)] == mags
    assert [L.nvfp4o_e2m1_decode(c | 8) for c in range(8)] == [-m for m in mags]
    assert max(mags) == _gold_constants()["M_FP4"]


def test_e4m3_decode_matches_torch_float8(oracle):
    L = oracle.lib()
    for b in range(256):
        v = L.nvfp4o_e4m3_decode(b)
        if np.isnan(E4M3_VALUES[b]):
            assert np.isnan(v)
        else:
            assert v == E4M3_VALUES[b], b
    assert L.nvfp4o_e4m3_decode(0x7E) == _gold_constants()["M_FP8"]


def test_e4m3_cast_matches_torch_and_identity(oracle):
    L = oracle.lib()
    # encode(decode(b)) = b on the 127 non-negative finite values
    for b in range(127):
        assert L.nvfp4o_e4m3_cast_ratio(float(E4M3_VALUES[b]), 1.0) == b
    # against torch's own round-to-nearest-even cast on random fp32 in range
    g = np.random.default_rng(7)
    q = np.concatenate([g.uniform(0, 448, 4000), np.exp(g.uniform(np.log(2.0 ** -11), np.log(448), 4000)),
                        # every midpoint between neighbours: ties
                        0.5 * (E4M3_VALUES[:126] + E4M3_VALUES[1:127])]).astype(np.float32)
    want = torch.from_numpy(q).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([L.nvfp4o_e4m3_cast_ratio(float(v), 1.0) for v in q])
    assert (got == want).all()
    # saturation above 448 (torch would give NaN there, the format reading saturates)
    assert L.nvfp4o_e4m3_cast_ratio(1e9, 1.0) == 0x7E
    assert L.nvfp4o_e4m3_cast_ratio(464.0, 1.0) == 0x7E
    # ratio form: same answer when numerator and denominator are scaled together
    for v in q[:500]:
        assert L.nvfp4o_e4m3_cast_ratio(float(v) * 3.0, 3.0) == L.nvfp4o_e4m3_cast_ratio(float(v), 1.0)


def test_bf16_rne_matches_torch(oracle):
    L = oracle.lib()
    g = np.random.default_rng(11)
    v = np.concatenate([g.standard_normal(3000) * 10.0 ** g.uniform(-30, 30, 3000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 2.0 ** -133, 2.0 ** -127 * 1.5,
                         -3.0 * 2.0 ** -134]]).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([L.nvfp4o_bf16_rne(float(x)) for x in v], dtype=np.uint16)
    assert (got == want).all()
    # decode is the inverse on every finite pattern sampled
    for h in range(0, 0x7F80, 97):
        assert L.nvfp4o_bf16_rne(L.nvfp4o_bf16_decode(h)) == h


def _nearest_brute(values, q):
    """argmin |v - q| over `values` with exact rationals; tie -> even index."""
    best, best_d = None, None
    for i, v in enumerate(values):
        d = abs(Fraction(v) - q)
        if best is None or d < best_d or (d == best_d and i % 2 == 0 and best % 2 == 1):
            best, best_d = i, d
    return best


def test_e2m1_cast_ties_and_brute_force(oracle):
    L = oracle.lib()
    mags = _gold_e2m1()
    # tie cases on a unit scale: halfway points go to the neighbour with mantissa bit 0
    ties = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for x, want in ties.items():
        assert mags[L.nvfp4o_e2m1_cast_ratio(x, 1.0)] == want
    # saturation
    for x in (6.0, 6.37, 8.4, 1e30):
        assert mags[L.nvfp4o_e2m1_cast_ratio(x, 1.0)] == 6.0
    # zero scale
    assert L.nvfp4o_e2m1_cast_ratio(3.0, 0.0) == 0
    # brute force with exact rationals on awkward denominators
    g = np.random.default_rng(3)
    for _ in range(3000):
        num = float(np.float32(abs(g.standard_normal()) * 4))
        den = float(np.float32(g.uniform(0.1, 3.0)))
        want = _nearest_brute(mags, Fraction(num) / Fraction(den))
        assert L.nvfp4o_e2m1_cast_ratio(num, den) == want


# ---------------------------------------------------------------- quantizer

def _fp32_nearest(fr):
    """Nearest float32 to an exact Fraction (ties to even) by brute force over neighbours."""
    c = np.float32(float(fr))
    cands = [np.nextafter(c, np.float32(-np.inf)), c, np.nextafter(c, np.float32(np.inf))]
    best = min(cands, key=lambda v: (abs(Fraction(float(v)) - fr), int(np.float32(v).view(np.uint32)) & 1))
    return np.float32(best)


def _quantize_brute(xb, gs_in=None):
    """Independent whole-quantizer in exact rational arithmetic, distance-argmin form."""
    x = wl.bf16_bits_to_f32(xb).astype(np.float64)
    R, K = x.shape
    amax = Fraction(float(np.abs(x).max()))
    if gs_in is not None:
        sg = np.float32(gs_in)
    else:
        sg = np.float32(1.0) if amax == 0 else _fp32_nearest(amax / 2688)
    sgF = Fraction(float(sg))
    e4 = [Fraction(float(v)) for v in E4M3_VALUES[:127]]
    mags = [Fraction(v) for v in _gold_e2m1()]
    codes = np.zeros((R, K // 2), np.uint8)
    scales = np.zeros((R, K // 16), np.uint8)
    for r in range(R):
        for b in range(K // 16):
            blk = x[r, b * 16:(b + 1) * 16]
            bmax = Fraction(float(np.abs(blk).max()))
            sb = _nearest_brute(e4, bmax / (6 * sgF))
            scales[r, b] = sb
            den = e4[sb] * sgF
            for j in range(16):
                idx = 0 if den == 0 else _nearest_brute(mags, Fraction(float(abs(blk[j]))) / den)
                c = idx | (8 if np.signbit(blk[j]) else 0)
                codes[r, b * 8 + j // 2] |= c << (4 * (j % 2))
    return codes, scales, sg


@pytest.mark.parametrize("seed,scale", [(0, 1.0), (1, 0.02), (2, 37.0), (3, 1e-3)])
def test_quantize_matches_rational_brute_force(oracle, seed, scale):
    g = np.random.default_rng(seed)
    x = (g.standard_normal((6, 48)) * scale).astype(np.float32)
    x[1, 5] *= 20
    x[2, 16:32] = 0                     # an all-zero block
    x[3, :] *= 1e-3                     # small rows -> subnormal / zero block scales
    x[4, 3] = -0.0
    xb = wl.to_bf16_bits(x)
    q = oracle.quantize(xb)
    codes, scales, sg = _quantize_brute(xb)
    assert q.global_scale == sg
    assert (q.scales == scales).all()
    assert (q.codes == codes).all()


def test_quantize_given_global_scale_brute(oracle):
    g = np.random.default_rng(5)
    xb = wl.to_bf16_bits(g.standard_normal((3, 32)).astype(np.float32))
    for gs in (2.0 ** -9, 0.001953125 * 1.5, 0.01):
        q = oracle.quantize(xb, global_scale_in=gs)
        codes, scales, sg = _quantize_brute(xb, gs_in=gs)
        assert q.global_scale == sg and (q.scales == scales).all() and (q.codes == codes).all()


@pytest.mark.parametrize("k", [-96, -24, 7, 96])
def test_quantize_commutes_with_power_of_two_scaling(oracle, k):
    """Eq. 2 / Eq. 12-13 only compare ratios: multiplying the tensor AND its scale by 2^k leaves every scale byte and
    every code unchanged (plain rule, scale search, both block axes).  The GPU uses this for tensor scales outside the
    range where fp32 quotients are safe.  Magnitudes chosen so that nothing overflows or becomes subnormal."""
    g = np.random.default_rng(300 + k)
    x = (g.standard_normal((48, 64)) * 3.0).astype(np.float32)
    x[g.random((48, 64)) < 0.1] *= np.float32(2.0 ** -9)                  # some blocks far below the maximum
    xb = wl.to_bf16_bits(x)
    xs = wl.to_bf16_bits((wl.bf16_bits_to_f32(xb).astype(np.float64) * 2.0 ** k).astype(np.float32))   # exact in bf16
    base_gs = oracle.global_scale(xb)
    assert np.float32(oracle.global_scale(xs)) == np.float32(np.float64(base_gs) * 2.0 ** k)
    for kw in ({}, {"four_over_six": True}, {"block_axis": 1}):
        a, b = oracle.quantize(xb, **kw), oracle.quantize(xs, **kw)
        assert (a.codes == b.codes).all() and (a.scales == b.scales).all(), kw


def test_global_scale_closed_forms(oracle):
    x = np.zeros((2, 16), np.float32)
    assert oracle.global_scale(bits(x)) == np.float32(1.0)        # all-zero tensor
    x[1, 3] = -2688.0
    assert oracle.global_scale(bits(x)) == np.float32(1.0)        # amax = 448*6
    x[1, 3] = 5.25                                                 # 5.25/2688 = 2^-9
    assert oracle.global_scale(bits(x)) == np.float32(2.0 ** -9)
    x[1, 3] = 1.0                                                  # 1/2688: nearest fp32 by brute force
    assert oracle.global_scale(bits(x)) == _fp32_nearest(Fraction(1, 2688))


def test_round_trip_of_representable_inputs(oracle):
    """X = code * scale * 2^p with a +-6 in every block and 6*448*2^p in the tensor
    must come back as exactly those codes, scales and s_g = 2^p."""
    g = np.random.default_rng(9)
    mags = np.array(_gold_e2m1())
    for p in (0, -9, 3):
        R, K = 8, 64
        sb = g.integers(1, 127, size=(R, K // 16)).astype(np.uint8)   # any positive E4M3 scale
        sb[0, 0] = 0x7E                                               # 448 somewhere
        idx = g.integers(0, 8, size=(R, K))
        sign = g.integers(0, 2, size=(R, K))
        pos = g.integers(0, 16, size=(R, K // 16))
        for r in range(R):
            for b in range(K // 16):
                idx[r, b * 16 + pos[r, b]] = 7                        # a 6 in every block
        val = mags[idx] * np.where(sign == 1, -1.0, 1.0)
        x = val * np.repeat(E4M3_VALUES[sb], 16, axis=1) * 2.0 ** p
        xb = bits(x)
        assert (wl.bf16_bits_to_f32(xb).astype(np.float64) == x).all()   # bf16-exact by construction
        q = oracle.quantize(xb)
        assert q.global_scale == np.float32(2.0 ** p)
        assert (q.scales == sb).all()
        code = (idx | (np.signbit(val) << 3)).astype(np.uint8)
        want = code[:, 0::2] | (code[:, 1::2] << 4)                  # even element in the low nibble
        assert (q.codes == want).all()
        assert (oracle.dequant_f64(q) == x).all()
        assert (oracle.dequant_bf16(q) == xb).all()


def test_ties_saturation_zero_blocks(oracle):
    # tensor with amax = 2688 (s_g = 1) and a block whose max is 6 (s_b = 1): unit grid
    x = np.zeros((1, 48), np.float32)
    x[0, 0] = 2688.0
    x[0, 16:32] = [6, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -0.25, -0.75, -1.25, -1.75, -2.5, -3.5, -5.0, 0]
    # third block: all zero
    q = oracle.quantize(bits(x))
    assert q.global_scale == np.float32(1.0)
    assert list(q.scales[0]) == [0x7E, 0x38, 0x00]                    # 448, 1.0, 0
    d = oracle.dequant_f64(q)[0]
    assert list(d[16:32]) == [6, 0, 1, 1, 2, 2, 4, 4, -0.0, -1, -1, -2, -2, -4, -4, 0]
    assert (q.codes[0, 16:24] == 0).all()
    # negative values that round to zero keep their sign bit: element 24 is -0.25 -> code 0x8
    assert q.codes[0, 8 + 4] & 0x0F == 0x8
    # E4M3 tie: bmax/(6 s_g) exactly between 1.0 (0x38) and 1.125 (0x39) -> even mantissa 0x38
    x2 = np.zeros((1, 32), np.float32)
    x2[0, 0] = 2688.0
    x2[0, 16] = 6 * 1.0625
    q2 = oracle.quantize(bits(x2))
    assert q2.scales[0, 1] == 0x38
    # ... and the block max then sits at 6.375 on that scale and saturates to 6
    assert oracle.dequant_f64(q2)[0, 16] == 6.0
    # between 1.125 (0x39) and 1.25 (0x3A) -> even mantissa 0x3A
    x2[0, 16] = 6 * 1.1875
    assert oracle.quantize(bits(x2)).scales[0, 1] == 0x3A
    # block whose true scale 1.4*2^-9 rounds to 2^-9: quotient 8.4 -> saturates at 6
    x3 = np.zeros((1, 32), np.float32)
    x3[0, 0] = 2688.0
    x3[0, 16] = 6 * 1.40625 * 2.0 ** -9
    q3 = oracle.quantize(bits(x3))
    assert q3.scales[0, 1] == 0x01 and (q3.codes[0, 8] & 7) == 7
    # bmax/(6 s_g) = 2^-10 exactly: tie between 0 and 2^-9 -> 0x00, all codes magnitude 0
    x3[0, 16] = 6 * 2.0 ** -10
    q3 = oracle.quantize(bits(x3))
    assert q3.scales[0, 1] == 0x00 and (q3.codes[0, 8:] & 0x77 == 0).all()


def test_gap_claim_and_error_invariant(oracle):
    """With the maximum mapped to 6, anything between 4/6 and 1 of the block maximum can
    only become 4 or 6 (appendix on scale search); and |x - x^| <= half the local step."""
    cfg = wl.config2(seed=1, M=64)
    xb = cfg["A"]
    q = oracle.quantize(xb)
    x = wl.bf16_bits_to_f32(xb).astype(np.float64)
    d = oracle.dequant_f64(q)
    lo = (q.codes & 7).astype(np.int64)
    hi = ((q.codes >> 4) & 7).astype(np.int64)
    idx = np.empty(x.shape, np.int64)
    idx[:, 0::2], idx[:, 1::2] = lo, hi
    sb = np.repeat(E4M3_VALUES[q.scales], 16, axis=1)
    den = sb * float(q.global_scale)
    bmax = np.repeat(np.abs(x).reshape(x.shape[0], -1, 16).max(-1), 16, axis=1)
    # block scale times 6 is within one E4M3 rounding (2^-4 relative) of the block maximum
    normal = (sb >= 2.0 ** -6) & (sb < 448)
    assert (np.abs(den * 6 - bmax)[normal] <= bmax[normal] * 2.0 ** -4).all()
    ratio = np.abs(x) / bmax
    # stay clear of the one-E4M3-rounding wiggle of the scale (a factor 1 +- 2^-4) around the bounds
    in_gap = (ratio > (4.0 / 6.0) * (1 + 2.0 ** -4)) & (ratio < 1.0)
    assert in_gap.sum() > 100
    assert np.isin(idx[in_gap], (6, 7)).all()
    gap = np.array([0.5, 0.5, 0.5, 0.5, 1.0, 1.0, 2.0, 2.0])[idx]      # step to the next value up
    gap_dn = np.array([0.5, 0.5, 0.5, 0.5, 0.5, 1.0, 1.0, 2.0])[idx]   # step to the next value down
    unsat = np.abs(x) <= 6 * den
    err = np.abs(x) - np.abs(d)
    assert (err[unsat] <= 0.5 * gap[unsat] * den[unsat]).all()
    assert (-err[unsat] <= 0.5 * gap_dn[unsat] * den[unsat]).all()


def test_storage_accounting(oracle):
    c = _gold_constants()
    xb = wl.config1()["A"]
    q = oracle.quantize(xb)
    n = xb.size
    assert q.codes.nbytes * 8 + q.scales.nbytes * 8 == c["BITS_PER_ELEM"] * n
    assert q.scales.shape[1] * c["BLOCK"] == xb.shape[1]
    # K+V in bf16: 4 bytes per (t,h,d) position; in NVFP4: 9/8 bytes
    assert 2 * 2 == c["KV_BYTES_PER_ELEM_BF16_KV"]
    assert 2 * (q.codes.nbytes + q.scales.nbytes) / n == c["KV_BYTES_PER_ELEM_NVFP4_KV"]


def test_transposed_quantize_is_quantize_of_transpose(oracle):
    g = np.random.default_rng(21)
    xb = wl.to_bf16_bits(g.standard_normal((48, 24)).astype(np.float32))
    qt = oracle.quantize(xb, block_axis=1)
    q = oracle.quantize(np.ascontiguousarray(xb.T), block_axis=0)
    assert qt.global_scale == q.global_scale
    assert (qt.codes == q.codes).all() and (qt.scales == q.scales).all()
    assert qt.rows == 24 and qt.K == 48


# ------------------------------------------------------------------ dequant

def _py_dequant(q):
    """Independent decode: torch float8 table for scales, the paper's value set for codes."""
    mags = np.array(_gold_e2m1())
    lo, hi = q.codes & 15, q.codes >> 4
    c = np.empty((q.rows, q.K), np.uint8)
    c[:, 0::2], c[:, 1::2] = lo, hi
    v = mags[c & 7] * np.where(c & 8, -1.0, 1.0)
    return v * np.repeat(E4M3_VALUES[q.scales], 16, axis=1) * np.float64(q.global_scale)


def test_dequant_matches_independent_decode_and_single_rounding(oracle):
    cfg = wl.config4(seed=3, T=16, H=4, d=128)
    xb = cfg["K"].reshape(-1, 128)
    q = oracle.quantize(xb)
    d = oracle.dequant_f64(q)
    assert (d == _py_dequant(q)).all()
    # bf16 output: nearest bf16 to the exact product, checked with exact rationals
    out = oracle.dequant_bf16(q)
    o = wl.bf16_bits_to_f32(out).astype(np.float64)
    flat_d, flat_o, flat_b = d.ravel(), o.ravel(), out.ravel()
    for i in range(0, flat_d.size, 7):
        exact = Fraction(flat_d[i])
        got = Fraction(flat_o[i])
        up = Fraction(float(wl.bf16_bits_to_f32(np.array([flat_b[i] + 1], np.uint16))[0]))
        dn = Fraction(float(wl.bf16_bits_to_f32(np.array([flat_b[i] - 1], np.uint16))[0])) if flat_b[i] & 0x7FFF else -up
        e = abs(exact - got)
        assert e <= abs(exact - up) and e <= abs(exact - dn)
        if e == abs(exact - up) or e == abs(exact - dn):
            assert flat_b[i] % 2 == 0      # a tie went to the even significand


# --------------------------------------------------------------------- GEMM

@pytest.mark.parametrize("M,N,K", [(3, 5, 16), (8, 8, 32), (7, 4, 48)])
def test_gemm_tiny_against_numpy_matmul(oracle, M, N, K):
    g = np.random.default_rng(M * 100 + N * 10 + K)
    qa = oracle.quantize(wl.to_bf16_bits(g.standard_normal((M, K)).astype(np.float32)))
    qw = oracle.quantize(wl.to_bf16_bits((g.standard_normal((N, K)) * 0.02).astype(np.float32)))
    Y, S = oracle.gemm(qa, qw)
    A, W = _py_dequant(qa), _py_dequant(qw)
    ref = A @ W.T
    refS = np.abs(A) @ np.abs(W).T
    assert np.allclose(Y, ref, rtol=0, atol=1e-13 * refS.max())
    assert np.allclose(S, refS, rtol=1e-13, atol=0)
    # a transposed operand or swapped roles would break this on non-square shapes
    rows = np.array([M - 1, 0], dtype=np.int64)
    Ysub, _ = oracle.gemm(qa, qw, rows=rows)
    assert (Ysub == Y[rows]).all()


def test_gemm_integer_special_case_and_scale_linearity(oracle):
    """All block scales 1 and s_g = 1: the result is an exact multiple of 0.25."""
    g = np.random.default_rng(4)
    mags = np.array(_gold_e2m1())

    def unit_tensor(rows, K):
        v = mags[g.integers(0, 8, size=(rows, K))] * g.choice([-1.0, 1.0], size=(rows, K))
        v[:, 0::16] = 6.0                    # block max 6 -> s_b = 1
        v[0, 1] = 2688.0                     # s_g = 1 ; its block gets s_b = 448
        return v

    a, w = unit_tensor(5, 32), unit_tensor(6, 32)
    qa, qw = oracle.quantize(bits(a)), oracle.quantize(bits(w))
    assert qa.global_scale == 1 and qw.global_scale == 1
    Y, _ = oracle.gemm(qa, qw)
    A, W = oracle.dequant_f64(qa), oracle.dequant_f64(qw)
    assert (Y == A @ W.T).all()              # integers/4: every summation order is exact
    assert (Y * 4 == np.round(Y * 4)).all()
    # linearity in the tensor scales
    q2 = oracle.Q(qa.codes, qa.scales, np.float32(0.5))
    Y2, _ = oracle.gemm(q2, qw)
    assert (Y2 == 0.5 * Y).all()


# --------------------------------------------------------------- activation

def test_gelu_tanh_against_torch_and_symmetry(oracle):
    L = oracle.lib()
    y = np.linspace(-8, 8, 2001)
    got = np.array([L.nvfp4o_gelu_tanh(float(v)) for v in y])
    want = torch.nn.functional.gelu(torch.from_numpy(y), approximate="tanh").numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-15)
    assert np.allclose(got - got[::-1], y, rtol=0, atol=1e-14)      # gelu(y) - gelu(-y) = y
    h = oracle.gelu_tanh_bf16(y)
    want_h = torch.nn.functional.gelu(torch.from_numpy(y.astype(np.float32)).double(),
                                      approximate="tanh").to(torch.bfloat16)
    ok = y >= -5.0        # below, 1 + tanh cancels and libm / torch differ in the last bits of a ~1e-7 result
    assert (h == want_h.view(torch.int16).numpy().view(np.uint16))[ok].all()


# ------------------------------------------------------------ four over six

def test_four_over_six_never_worse_and_brute(oracle):
    cfg = wl.config2(seed=1, M=32)
    xb = cfg["A"][:, :256].copy()
    q6 = oracle.quantize(xb)
    q46 = oracle.quantize(xb, four_over_six=True)
    assert q46.global_scale == q6.global_scale
    x = wl.bf16_bits_to_f32(xb).astype(np.float64)
    e6 = ((x - oracle.dequant_f64(q6)) ** 2).reshape(x.shape[0], -1, 16).sum(-1)
    e46 = ((x - oracle.dequant_f64(q46)) ** 2).reshape(x.shape[0], -1, 16).sum(-1)
    assert (e46 <= e6 * (1 + 1e-12)).all()
    changed = q46.scales != q6.scales
    assert 0 < changed.mean() < 1                      # some blocks switch, not all
    # where the choice changed, the new scale is the 4-target one: cast_E4M3(bmax / (4 s_g))
    L = oracle.lib()
    bmax = np.abs(x).reshape(x.shape[0], -1, 16).max(-1)
    sg = float(q6.global_scale)
    for r, b in zip(*np.nonzero(changed)):
        assert q46.scales[r, b] == L.nvfp4o_e4m3_cast_ratio(float(bmax[r, b]), 4.0 * sg)
    # unchanged blocks carry identical codes
    same = np.repeat(~changed, 8, axis=1)
    assert (q46.codes[same] == q6.codes[same]).all()


def _four_over_six_brute(xb, gs_in=None):
    """Appendix Eq. 12-13 in exact rationals, independent of the oracle: for every block BOTH
    candidates (block maximum mapped to 6 and to 4) are encoded in distance-argmin form, their
    squared errors sum_j (|x_j| - m_j s_b s_g)^2 are formed exactly, and the 4-based candidate is
    taken only when its error is strictly smaller.  Returns codes, scales, the tensor scale, and
    per block (err6, err4) as Fractions."""
    x = wl.bf16_bits_to_f32(xb).astype(np.float64)
    R, K = x.shape
    amax = Fraction(float(np.abs(x).max()))
    sg = np.float32(gs_in) if gs_in is not None else (np.float32(1.0) if amax == 0 else _fp32_nearest(amax / 2688))
    sgF = Fraction(float(sg))
    e4 = [Fraction(float(v)) for v in E4M3_VALUES[:127]]
    mags = [Fraction(v) for v in _gold_e2m1()]
    codes = np.zeros((R, K // 2), np.uint8)
    scales = np.zeros((R, K // 16), np.uint8)
    errs = {}
    for r in range(R):
        for b in range(K // 16):
            blk = x[r, b * 16:(b + 1) * 16]
            ax = [Fraction(float(abs(v))) for v in blk]
            bmax = max(ax)
            cand = []
            for target in (6, 4):
                sb = _nearest_brute(e4, bmax / (target * sgF))
                den = e4[sb] * sgF
                idx = [0 if den == 0 else _nearest_brute(mags, a / den) for a in ax]
                err = sum((a - mags[i] * den) ** 2 for a, i in zip(ax, idx))
                cand.append((sb, idx, err))
            pick = 1 if cand[1][2] < cand[0][2] else 0          # equal errors keep the 6-based encoding
            errs[(r, b)] = (cand[0][2], cand[1][2])
            scales[r, b] = cand[pick][0]
            for j, i in enumerate(cand[pick][1]):
                c = i | (8 if np.signbit(blk[j]) else 0)
                codes[r, b * 8 + j // 2] |= c << (4 * (j % 2))
    return codes, scales, sg, errs


def _four_over_six_cases():
    g = np.random.default_rng(46)
    act = wl.bf16_bits_to_f32(wl.config2(seed=1, M=12)["A"][:, :192])          # N(0,1), outlier channels x20
    kv = wl.bf16_bits_to_f32(wl.kv_tensor(2, 6, 128, 4, 0).reshape(12, 128))   # per-head scales
    grad = (g.standard_normal((6, 96)) * 1e-3).astype(np.float32)              # gradient-sized values
    # values on a coarse grid: many blocks where both candidates reconstruct exactly or equally badly
    grid = (g.integers(-12, 13, size=(8, 96)) * 0.25).astype(np.float32)
    grid[0, :16] = 0.0                                                         # a zero block
    grid[1, 16:32] = 0.0
    grid[1, 16] = 3.0                                                          # a lone maximum
    grid[2, 32:48] = np.float32(1.5)                                           # a constant block
    spread = (g.standard_normal((4, 64)) * np.exp2(g.integers(-12, 4, size=(4, 64)))).astype(np.float32)
    # exact ties between two DIFFERENT encodings: with the tensor maximum 2688 the tensor scale is 1, and a
    # block whose values are 6 v, 3 v, ... for an E4M3 value v is reconstructed without error on scale v
    # (target 6) and on scale 1.5 v (target 4) alike
    lone = np.zeros((4, 128), np.float32)
    lone[0, 0] = 2688.0
    for b, v in enumerate([1.0, 2.0, 0.5, 16.0, 0.25, 1.25, 40.0]):
        lone[1, 16 * b] = 6.0 * v                     # a lone maximum
        lone[2, 16 * b: 16 * b + 3] = [6.0 * v, -3.0 * v, 1.5 * v]
        lone[3, 16 * b: 16 * b + 16] = 6.0 * v        # a constant block
    return [("activations", act, None), ("kv", kv, None), ("gradients", grad, None), ("grid", grid, None),
            ("wide dynamic range", spread, None), ("exact ties", lone, None),
            # tensor scales given by the caller: block scales that saturate at 448, and that underflow
            ("given scale, saturating", act[:3, :64], np.float32(2.0 ** -14)),
            ("given scale, underflowing", grad[:3, :64], np.float32(8.0))]


def test_four_over_six_both_candidates_in_exact_rationals(oracle):
    """Every block of several seeded tensors: the oracle's scale byte and all sixteen codes equal
    those of the candidate that an exact evaluation of both encodings and both squared errors
    selects (Appendix Eq. 12-13).  A search that is biased towards 6, that compares with <= instead
    of <, or that mis-encodes the codes of the blocks it switches, fails here."""
    switched = ties = total = 0
    for name, x, gs in _four_over_six_cases():
        xb = wl.to_bf16_bits(np.ascontiguousarray(x, dtype=np.float32))
        q = oracle.quantize(xb, four_over_six=True, global_scale_in=gs)
        codes, scales, sg, errs = _four_over_six_brute(xb, gs)
        assert q.global_scale == sg, name
        bad = np.argwhere(q.scales != scales)
        assert bad.size == 0, f"{name}: scale byte of block {tuple(bad[0])}: oracle {q.scales[tuple(bad[0])]:#x}, " \
                              f"exact {scales[tuple(bad[0])]:#x}, errors (6, 4) = {[float(e) for e in errs[tuple(bad[0])]]}"
        assert (q.codes == codes).all(), name
        e6 = np.array([[float(errs[(r, b)][0]) for b in range(scales.shape[1])] for r in range(scales.shape[0])])
        e4 = np.array([[float(errs[(r, b)][1]) for b in range(scales.shape[1])] for r in range(scales.shape[0])])
        switched += int(sum(1 for v in errs.values() if v[1] < v[0]))
        ties += int(sum(1 for v in errs.values() if v[1] == v[0]))
        total += len(errs)
        assert np.isfinite(e6).all() and np.isfinite(e4).all()
    # the cases exercise all three outcomes many times over
    assert switched > 100 and ties > 20 and total - switched - ties > 100, (switched, ties, total)


def test_four_over_six_exact_ties_between_different_encodings(oracle):
    """Blocks that both targets reconstruct without error, on different scales: the 6-based encoding
    stays (a search that takes the 4-based candidate on equal error changes these bytes)."""
    name, x, gs = [c for c in _four_over_six_cases() if c[0] == "exact ties"][0]
    xb = wl.to_bf16_bits(x)
    q = oracle.quantize(xb, four_over_six=True)
    codes, scales, sg, errs = _four_over_six_brute(xb)
    differing_ties = 0
    for (r, b), (e6, e4) in errs.items():
        if e6 == e4 and r >= 1 and b < 7:
            differing_ties += 1
            assert e6 == 0
    assert differing_ties >= 15
    assert (q.scales == scales).all() and (q.codes == codes).all()
    assert (q.scales == oracle.quantize(xb).scales).all()          # i.e. exactly the plain max -> 6 rule here


def test_four_over_six_equal_error_keeps_six(oracle):
    """A block holding only its maximum is exact under both targets; the reading keeps 6."""
    x = np.zeros((1, 32), np.float32)
    x[0, 0] = 2688.0
    x[0, 16] = 6.0
    q = oracle.quantize(bits(x), four_over_six=True)
    assert q.scales[0, 1] == 0x38 and (q.codes[0, 8] & 7) == 7


# ------------------------------------------------------------ K-smoothing (KV)

def _bf16_of_exact(v):
    """RNE to bf16 of a value that float32 holds exactly, by torch's own cast."""
    t = torch.tensor([v], dtype=torch.float64)
    assert float(t.to(torch.float32)[0]) == v
    return int(t.to(torch.float32).to(torch.bfloat16).view(torch.int16)[0]) & 0xFFFF


def test_kv_smooth_closed_forms(oracle):
    """Sec. 3.2, Eq. 6: the row mean over the features is removed."""
    d = 32
    # (a) a constant row is its own mean: nothing is left to quantize, and it comes back exactly
    x = np.tile(np.array([[1.5], [-0.375], [96.0], [0.0]], np.float32), (1, d))
    mean, xbar = oracle.kv_smooth(bits(x))
    assert (mean == bits(x)[:, 0]).all() and (xbar & 0x7FFF == 0).all()
    q = oracle.quantize(xbar, four_over_six=True)
    assert (q.codes & 0x77 == 0).all()
    assert (oracle.dequant_bf16(q, mean) == bits(x)).all()
    # (b) antisymmetric rows have mean zero: smoothing changes nothing
    g = np.random.default_rng(5)
    h = wl.bf16_bits_to_f32(wl.to_bf16_bits(g.standard_normal((6, d // 2)).astype(np.float32)))
    y = np.concatenate([h, -h], axis=1)
    mean, ybar = oracle.kv_smooth(bits(y))
    assert (mean & 0x7FFF == 0).all() and (ybar == bits(y)).all()
    # (c) shifting a row by a constant moves the mean and leaves the smoothed row alone
    #     (small integers: every value, sum and difference is exact in bf16)
    z = g.integers(-20, 21, size=(5, d)).astype(np.float32)
    z[:, 0] -= z.sum(axis=1) % d                      # make every row sum a multiple of d: integer means
    m0, z0 = oracle.kv_smooth(bits(z))
    m1, z1 = oracle.kv_smooth(bits(z + 7.0))
    assert (z0 == z1).all()
    assert (wl.bf16_bits_to_f32(m1) - wl.bf16_bits_to_f32(m0) == 7.0).all()
    assert (wl.bf16_bits_to_f32(m0) == z.sum(axis=1) / d).all()
    assert (wl.bf16_bits_to_f32(z0) == z - (z.sum(axis=1) / d)[:, None]).all()


def test_kv_smooth_against_rational_arithmetic(oracle):
    """Mean and smoothed elements against exact rationals rounded by torch's bf16 cast."""
    g = np.random.default_rng(6)
    d = 16
    xb = wl.to_bf16_bits((g.standard_normal((40, d)) * 3).astype(np.float32))
    x = wl.bf16_bits_to_f32(xb)
    mean, xbar = oracle.kv_smooth(xb)
    for r in range(x.shape[0]):
        s = sum(Fraction(float(v)) for v in x[r]) / d
        sf = float(s)                                  # d = 16 and 8-bit values within 2^10: exact, and exact in fp32
        assert Fraction(sf) == s
        assert mean[r] == _bf16_of_exact(sf)
        mu = Fraction(float(wl.bf16_bits_to_f32(mean[r:r + 1])[0]))
        for j in range(d):
            df = float(Fraction(float(x[r, j])) - mu)
            assert xbar[r, j] == _bf16_of_exact(df)


def test_kv_smooth_reconstruction(oracle):
    """RN_bf16(x^ + mean): the nearest bf16 to the exact rational sum of the independently
    decoded value and the mean; smoothing shrinks the error on rows with a large common offset."""
    g = np.random.default_rng(7)
    rows, d = 48, 128
    x = g.standard_normal((rows, d)).astype(np.float32) + g.uniform(-8, 8, size=(rows, 1)).astype(np.float32)
    xb = wl.to_bf16_bits(x)
    mean, xbar = oracle.kv_smooth(xb)
    q = oracle.quantize(xbar, four_over_six=True)
    got = oracle.dequant_bf16(q, mean)
    deq = _py_dequant(q)
    mu = wl.bf16_bits_to_f32(mean).astype(np.float64)
    o = wl.bf16_bits_to_f32(got).astype(np.float64)
    nb = lambda b: Fraction(float(wl.bf16_bits_to_f32(np.array([b], np.uint16))[0]))
    for r in range(rows):
        for k in range(r % 5, d, 5):
            exact = Fraction(deq[r, k]) + Fraction(mu[r])       # exact rational sum of the two exact terms
            b = int(got[r, k])
            e = abs(exact - Fraction(o[r, k]))
            up = nb(b + 1)
            dn = nb(b - 1) if b & 0x7FFF else -up
            assert e <= abs(exact - up) and e <= abs(exact - dn)
            if e == abs(exact - up) or e == abs(exact - dn):
                assert b % 2 == 0                               # a tie went to the even significand
    xf = wl.bf16_bits_to_f32(xb).astype(np.float64)
    e_smooth = np.linalg.norm(xf - wl.bf16_bits_to_f32(got))
    plain = oracle.quantize(xb, four_over_six=True)
    e_plain = np.linalg.norm(xf - wl.bf16_bits_to_f32(oracle.dequant_bf16(plain)))
    assert e_smooth < 0.8 * e_plain


# ------------------------------------------------- 2-D block scaling (weights)

def test_quantize_2d_tiles_against_rational_brute_force(oracle):
    """Sec. 2.2 training recipe: one scale per 16x16 tile.  Exact rationals: the tile's scale is
    the E4M3 value nearest to tilemax / (6 s_g), every code the E2M1 value nearest to x / (s s_g)."""
    xb = wl.normal((32, 48), 0.02, 21, 0)
    xb[5, 7] = wl.to_bf16_bits(np.array([0.31], np.float32))[0]           # an outlier inside one tile
    x = wl.bf16_bits_to_f32(xb).astype(np.float64)
    q, qt = oracle.quantize_2d(xb)
    sg = _fp32_nearest(Fraction(float(np.abs(x).max())) / 2688)
    assert np.float32(q.global_scale) == sg and np.float32(qt.global_scale) == sg
    sgF = Fraction(float(sg))
    e4 = [Fraction(float(v)) for v in E4M3_VALUES[:127]]
    mags = [Fraction(v) for v in _gold_e2m1()]
    for I in range(2):
        for J in range(3):
            tile = x[16 * I:16 * I + 16, 16 * J:16 * J + 16]
            sb = _nearest_brute(e4, Fraction(float(np.abs(tile).max())) / (6 * sgF))
            assert (q.scales[16 * I:16 * I + 16, J] == sb).all()           # the same byte on all 16 rows of the tile
            assert (qt.scales[16 * J:16 * J + 16, I] == sb).all()          # and on all 16 columns
            den = e4[sb] * sgF
            for i in range(16):
                for j in range(16):
                    idx = _nearest_brute(mags, Fraction(float(abs(tile[i, j]))) / den) | (8 if np.signbit(tile[i, j]) else 0)
                    byte = q.codes[16 * I + i, (16 * J + j) // 2]
                    assert (byte >> (4 * (j % 2))) & 15 == idx
                    byte_t = qt.codes[16 * J + j, (16 * I + i) // 2]
                    assert (byte_t >> (4 * (i % 2))) & 15 == idx


def test_quantize_2d_serves_the_transposed_operand(oracle):
    """The point of 2-D scaling: W and W^T dequantize to the same matrix, and quantizing the
    transposed matrix gives the transposed pair."""
    xb = wl.normal((64, 96), 0.02, 22, 0)
    q, qt = oracle.quantize_2d(xb)
    assert (oracle.dequant_f64(qt) == oracle.dequant_f64(q).T).all()
    q2, q2t = oracle.quantize_2d(np.ascontiguousarray(xb.T))
    assert (q2.codes == qt.codes).all() and (q2.scales == qt.scales).all()
    assert (q2t.codes == q.codes).all() and (q2t.scales == q.scales).all()
    # a tile whose rows all share the tile maximum is quantized like sixteen 1-D blocks
    x = wl.bf16_bits_to_f32(xb).copy()
    x[:16, :16] = np.clip(x[:16, :16], -0.01, 0.01)
    x[:16, 0] = 0.05
    yb = wl.to_bf16_bits(x)
    a, _ = oracle.quantize_2d(yb)
    b = oracle.quantize(yb)
    assert (a.scales[:16, 0] == b.scales[:16, 0]).all() and (a.codes[:16, :8] == b.codes[:16, :8]).all()
    # 1-D scales can only be finer: the 2-D error is never smaller in total
    xf = wl.bf16_bits_to_f32(xb).astype(np.float64)
    assert np.linalg.norm(xf - oracle.dequant_f64(q)) >= np.linalg.norm(xf - oracle.dequant_f64(oracle.quantize(xb))) * 0.999


# ----------------------------------------------------- random Hadamard transform

def _h16():
    i = np.arange(16)
    return np.where(np.array([[bin(a & b).count("1") & 1 for b in i] for a in i]), -1.0, 1.0)


def test_rht_is_the_scaled_sylvester_matrix(oracle):
    """Sec. 2.2: the transform of unit vectors spells out (1/4) H16 diag(s); H16 is the Kronecker
    power of [[1, 1], [1, -1]] (scipy's construction), and the transform is orthogonal."""
    from scipy.linalg import hadamard
    assert (_h16() == hadamard(16)).all()
    mask = 0b1010_0011_0101_1100
    s = np.array([-1.0 if (mask >> j) & 1 else 1.0 for j in range(16)])
    eye = np.eye(16, dtype=np.float32) * 4.0                       # 4 e_j: the images are exact in bf16
    y = wl.bf16_bits_to_f32(oracle.rht_rows(bits(eye), mask))
    assert (y == hadamard(16) * s[None, :]).all()
    T = hadamard(16) * s[None, :] / 4.0
    assert (T @ T.T == np.eye(16)).all()


def test_rht_on_integers_is_exact_and_preserves_the_product(oracle):
    """Small-integer operands: every sum is exact in bf16 after the 1/4 only if divisible, so use
    multiples of 4; then (T a)^T (T b) = a^T b exactly, column by column, group by group."""
    g = np.random.default_rng(31)
    mask = int(g.integers(0, 1 << 16))
    a = (g.integers(-3, 4, size=(64, 5)) * 4).astype(np.float32)
    b = (g.integers(-3, 4, size=(64, 7)) * 4).astype(np.float32)
    ta = wl.bf16_bits_to_f32(oracle.rht_rows(bits(a), mask)).astype(np.float64)
    tb = wl.bf16_bits_to_f32(oracle.rht_rows(bits(b), mask)).astype(np.float64)
    s = np.array([-1.0 if (mask >> j) & 1 else 1.0 for j in range(16)])
    T = _h16() * s[None, :] / 4.0
    for grp in range(4):
        assert (ta[16 * grp:16 * grp + 16] == T @ a[16 * grp:16 * grp + 16].astype(np.float64)).all()
    assert (ta.T @ tb == a.astype(np.float64).T @ b.astype(np.float64)).all()


def test_rht_rounds_once_to_bf16(oracle):
    g = np.random.default_rng(32)
    mask = 0x9A3C
    xb = wl.to_bf16_bits(g.standard_normal((32, 6)).astype(np.float32))
    x = wl.bf16_bits_to_f32(xb)
    y = oracle.rht_rows(xb, mask)
    s = [(-1 if (mask >> j) & 1 else 1) for j in range(16)]
    H = _h16()
    for grp in range(2):
        for c in range(6):
            v = [Fraction(float(x[16 * grp + j, c])) * s[j] for j in range(16)]
            for i in range(16):
                exact = sum(v[j] * int(H[i, j]) for j in range(16)) / 4
                ef = float(exact)
                assert Fraction(ef) == exact                   # fits fp32 here: torch's cast is then the single rounding
                assert y[16 * grp + i, c] == _bf16_of_exact(ef)


# ----------------------------------------------------------- LoRA side branch

def test_lora_branch_against_numpy(oracle):
    """Sec. 2.2: W ~ Dequant(Q(W0)) + (alpha/r) B A.  The oracle's loops against numpy's matmul on
    independently decoded operands; zero adapters leave the GEMM alone; the update is linear in its scale."""
    M, N, K, r = 6, 7, 32, 16
    xb = wl.normal((M, K), 1.0, 41, 0)
    wb = wl.normal((N, K), 0.02, 41, 1)
    ab = wl.normal((r, K), 0.05, 41, 2)
    bb = wl.normal((N, r), 0.05, 41, 3)
    x, a, b = (wl.bf16_bits_to_f32(v).astype(np.float64) for v in (xb, ab, bb))
    t = oracle.lora_down(xb, ab)
    assert (t == oracle.bf16_rne(x @ a.T)).all()
    # the rounding of T is torch's bf16 cast where fp32 holds the sum exactly enough: compare values
    tt = torch.tensor(x @ a.T).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert (np.abs(wl.bf16_bits_to_f32(t) - tt) <= np.abs(tt) * 2.0 ** -8).all()
    qa, qw = oracle.quantize(xb), oracle.quantize(wb)
    Y0, S0 = oracle.gemm(qa, qw)
    tv = wl.bf16_bits_to_f32(t).astype(np.float64)
    Y, S = oracle.gemm_lora(qa, qw, t, bb, 0.5)
    assert np.allclose(Y, Y0 + 0.5 * (tv @ b.T), rtol=1e-13, atol=1e-300)
    assert np.allclose(S, S0 + 0.5 * (np.abs(tv) @ np.abs(b).T), rtol=1e-13)
    Yz, _ = oracle.gemm_lora(qa, qw, t, wl.to_bf16_bits(np.zeros((N, r), np.float32)), 0.5)
    assert (Yz == Y0).all()
    Y2, _ = oracle.gemm_lora(qa, qw, t, bb, 1.0)
    assert np.allclose(Y2 - Y0, 2 * (Y - Y0), rtol=1e-12, atol=1e-300)
    rows = np.array([4, 1], np.int64)
    Yr, Sr = oracle.gemm_lora(qa, qw, t, bb, 0.5, rows=rows)
    assert (Yr == Y[rows]).all() and (Sr == S[rows]).all()
