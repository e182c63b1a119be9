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


def _hadamard16(v):
    """Butterflies of the 16-point Walsh-Hadamard transform along axis 1, in the dtype of v (one rounding per add)."""
    v = v.copy()
    h = 1
    while h < 16:
        for i in range(16):
            if (i & h) == 0:
                a, b = v[:, i].copy(), v[:, i + h].copy()
                v[:, i], v[:, i + h] = a + b, a - b
        h <<= 1
    return v


def _fp32_test_passes(bits):
    """The kernels' test on the packed exponents of a group of 16 bf16 values (rows of `bits`): all non-zero
    magnitudes within 12 binades of the largest, the largest exponent field in [40, 240]."""
    a = (bits.astype(np.uint32) << 1) & 0xFFFF
    emax = (a.max(axis=1) >> 8).astype(np.int64)
    am1 = np.where(a == 0, 0xFFFF, a - 1)
    emin = np.maximum(((am1.min(axis=1) + 1) >> 8).astype(np.int64), 1)
    return (emax >= 40) & (emax <= 240) & (emax - emin <= 12)


def test_fp32_hadamard_of_bf16_groups_is_exact_when_the_exponent_test_passes():
    """The random Hadamard transform (Sec. 2.2) takes its sums in fp32 for groups that pass the exponent
    test and in fp64 otherwise (here: butterfly order; the next test: the order of the matrix pipes).  For groups that pass, the fp32 sums carry no rounding at all (equal to the fp64
    sums, which are exact there), so the one rounding to bf16 that follows is that of the exact value; the test
    is not vacuous (groups one binade wider do lose bits in fp32), and it lets most Gaussian groups through."""
    g = np.random.default_rng(12)
    n = 200_000
    mant = g.integers(0, 128, size=(n, 16), dtype=np.uint32)
    sign = g.integers(0, 2, size=(n, 16), dtype=np.uint32)
    top = g.integers(41, 240, size=(n, 1), dtype=np.uint32)
    spread = g.integers(0, 16, size=(n, 1))
    expo = (top - np.minimum(g.integers(0, 16, size=(n, 16)), spread).astype(np.uint32)).astype(np.uint32)
    bits = (sign << 15) | (expo << 7) | mant
    bits[g.random((n, 16)) < 0.05] = 0                          # some zeros, which the test ignores
    x32 = _bf16_to_f32(bits.ravel()).reshape(n, 16)
    ok = _fp32_test_passes(bits)
    f32 = _hadamard16(x32.astype(np.float32))
    f64 = _hadamard16(x32.astype(np.float64))
    same = (f32.astype(np.float64) == f64).all(axis=1)
    assert ok.sum() > n // 4 and (~ok).sum() > n // 20
    assert same[ok].all(), "an fp32 butterfly rounded inside a group that passed the test"
    assert not same[~ok].all(), "the test rejects nothing that fp32 would get wrong"
    gauss = g.standard_normal((50_000, 16)).astype(np.float32)
    gb = _rne_f32_to_bf16(gauss.ravel()).reshape(-1, 16)
    assert _fp32_test_passes(gb).mean() > 0.97


def _h16_signs():
    i = np.arange(16)
    return (1 - 2 * (np.array([[bin(a & b).count("1") & 1 for b in i] for a in i]))).astype(np.float64)


def test_fp32_hadamard_sums_are_exact_in_the_order_the_matrix_pipes_take_them():
    """The kernels take the sixteen-term sums of the transform on the matrix pipes: four chains per group, each adding
    four products at a time onto an fp32 accumulator (k-groups 0..3, 4..7, ...).  For groups that pass the exponent
    test every partial sum of +-x/4 terms, in ANY order and grouping, has at most 24 significant bits: checked here for
    that order with every partial sum rounded to fp32 (a stricter model than hardware that rounds once per four
    products), against the exact sums."""
    g = np.random.default_rng(21)
    n = 100_000
    mant = g.integers(0, 128, size=(n, 16), dtype=np.uint32)
    sign = g.integers(0, 2, size=(n, 16), dtype=np.uint32)
    top = g.integers(40, 241, size=(n, 1), dtype=np.uint32)
    expo = (top - g.integers(0, 13, size=(n, 16)).astype(np.uint32)).astype(np.uint32)
    bits = (sign << 15) | (expo << 7) | mant
    bits[g.random((n, 16)) < 0.05] = 0
    ok = _fp32_test_passes(bits)
    assert ok.mean() > 0.9
    x = _bf16_to_f32(bits[ok].ravel()).reshape(-1, 16).astype(np.float64)
    n = x.shape[0]
    H = _h16_signs()
    exact = 0.25 * (x @ H.T)                                      # fp64: exact here
    acc = np.zeros((n, 16), dtype=np.float32)
    for k in range(16):                                           # one product at a time, every partial sum rounded to fp32
        acc = (acc.astype(np.float64) + 0.25 * H[:, k][None, :] * x[:, k][:, None]).astype(np.float32)
    assert (acc.astype(np.float64) == exact).all()


def test_hadamard_of_a_wide_group_as_two_fp32_halves():
    """Groups that span 13..25 binades are transformed as two sets -- the elements within 12 binades of the largest,
    and the rest -- whose fp32 transforms L and S are exact, so that the exact result is L + S.  The kernels round
    fl32(L + S) to bf16 and fall back to fp64 only when fl32(L + S) has the low sixteen bits 0x8000 (a bf16 midpoint).
    Checked against the exact sum rounded once: wherever the low bits differ from 0x8000 the two roundings agree, and
    the rule is not vacuous (without it some results would differ)."""
    g = np.random.default_rng(22)
    n = 200_000
    mant = g.integers(0, 128, size=(n, 16), dtype=np.uint32)
    sign = g.integers(0, 2, size=(n, 16), dtype=np.uint32)
    top = g.integers(66, 241, size=(n, 1), dtype=np.uint32)
    # a few large elements, the rest 13..25 binades below: cancellation among the large ones leaves sums the small ones decide
    drop = np.where(g.random((n, 16)) < 0.3, g.integers(0, 2, size=(n, 16)), g.integers(13, 26, size=(n, 16)))
    expo = (top - drop.astype(np.uint32)).astype(np.uint32)
    mant[g.random((n, 16)) < 0.5] = 0                             # many powers of two: exact cancellations, sums on midpoints
    bits = (sign << 15) | (expo << 7) | mant
    x = _bf16_to_f32(bits.ravel()).reshape(n, 16).astype(np.float64)
    e = (bits >> 7) & 0xFF
    big = e >= (e.max(axis=1, keepdims=True) - 12)
    H = _h16_signs()
    L = (0.25 * ((x * big) @ H.T)).astype(np.float32)
    S = (0.25 * ((x * ~big) @ H.T)).astype(np.float32)
    assert (L.astype(np.float64) == 0.25 * ((x * big) @ H.T)).all() and (S.astype(np.float64) == 0.25 * ((x * ~big) @ H.T)).all()
    exact = L.astype(np.float64) + S.astype(np.float64)           # at most 25 + 8 + 4 bits: exact in fp64
    y = (L + S)                                                   # fp32, rounded to nearest
    want = _rne_f64_to_bf16(exact.ravel())
    got = _rne_f32_to_bf16(y.ravel())
    midpoint = (y.ravel().view(np.uint32) & 0xFFFF) == 0x8000
    assert (got[~midpoint] == want[~midpoint]).all()
    assert midpoint.any() and (got[midpoint] != want[midpoint]).any(), "the midpoint rule guards nothing in this sample"


def test_near_tie_difference_is_an_exact_fp32_number():
    """Near-ties of the E2M1 rounding are settled by the sign of fma(c, s_g, -|x|) in fp32, c = midpoint x block
    scale.  The claim behind it: when |x| lies within 2^-19 of c s_g, the exact difference c s_g - |x| is itself an
    fp32 number (c has at most 7 significant bits, s_g 24, |x| 8, and the leading bits cancel), so the one rounding of
    the fused multiply-add changes nothing and the sign it returns is the sign of the exact difference.  Checked in
    exact rationals for every midpoint and every E4M3 mantissa: near-ties are made by choosing the tensor scale as
    the fp32 number nearest to |x| / c, and up to 12 ulps to either side of it (2^-19 is 16 ulps)."""
    from fractions import Fraction
    g = np.random.default_rng(5)
    mids = [Fraction(1, 4), Fraction(3, 4), Fraction(5, 4), Fraction(7, 4), Fraction(5, 2), Fraction(7, 2), Fraction(5)]
    checked = zero = 0
    for _ in range(40):
        xbits = np.uint32((int(g.integers(60, 200)) << 7 | int(g.integers(0, 128))) << 16)
        x = Fraction(float(xbits.view(np.float32)))
        for m3 in range(8):
            sb = Fraction(8 + m3, 8) * Fraction(2) ** int(g.integers(-6, 9))
            for t in mids:
                c = t * sb
                assert np.float32(float(c)) == float(c)                      # c itself is exact in fp32
                centre = int(np.float32(float(x / c)).view(np.uint32))
                for off in (-12, -5, -1, 0, 1, 2, 7, 12):
                    sg = Fraction(float(np.uint32(centre + off).view(np.float32)))
                    d = c * sg - x
                    assert abs(d) <= Fraction(1, 2 ** 19) * x                  # a near-tie by construction
                    assert Fraction(float(np.float32(float(d)))) == d, (float(c), float(sg), float(x))
                    checked += 1
                    zero += d == 0
    assert checked > 10_000 and 0 < zero < checked // 4                        # exact ties occur, most cases are not
