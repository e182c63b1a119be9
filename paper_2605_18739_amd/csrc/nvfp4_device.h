// Device-side helpers shared by the gfx950 NVFP4 kernels: format conversions,
// exact rounding decisions, wavefront reductions.  (Sec. 2.2 "NVFP4
// Preliminaries"; Appendix "Scale Search NVFP4 Quantization", Eq. 12.)
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

namespace nvfp4 {

constexpr int kWave = 64;
constexpr float kFp4Max = 6.0f;      // M^FP4
constexpr float kFp8Max = 448.0f;    // M^FP8

__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// max of the absolute values of two packed bf16 pairs, on their bit patterns
// (|bf16| patterns order like unsigned integers).
__device__ __forceinline__ uint32_t pk_absmax_u16(uint32_t acc, uint32_t w)
{
    uint32_t a = w & 0x7FFF7FFFu;
    ushort2v x = __builtin_bit_cast(ushort2v, acc), y = __builtin_bit_cast(ushort2v, a);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(x, y));
}
__device__ __forceinline__ uint32_t pk_hmax_u16(uint32_t p) { return max(p & 0xFFFFu, p >> 16); }

// ---- wavefront max over 64 lanes with DPP (unsigned compare) -------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max_step(uint32_t v)
{
    uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
    return max(v, o);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = dpp_max_step<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_max_step<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_max_step<0x124>(v);   // row_ror:4
    v = dpp_max_step<0x128>(v);   // row_ror:8  -> every lane holds its 16-lane row max
    uint32_t a = __builtin_amdgcn_readlane((int)v, 0), b = __builtin_amdgcn_readlane((int)v, 16);
    uint32_t c = __builtin_amdgcn_readlane((int)v, 32), d = __builtin_amdgcn_readlane((int)v, 48);
    return max(max(a, b), max(c, d));
}

// ---- E4M3 (1-4-3, bias 7, max 448) ---------------------------------------
// byte 0x00..0x7E -> value, exact
__device__ __forceinline__ float e4m3_to_f32(uint32_t b)
{
    float normal = __uint_as_float((b << 20) + (120u << 23));
    float sub = (float)(b & 7u) * 0.001953125f;    // m * 2^-9
    return (b >> 3) ? normal : sub;
}
// value -> f16 bit pattern (every E4M3 value, subnormals included, is a normal f16)
__device__ __forceinline__ _Float16 e4m3_to_f16(uint32_t b)
{
    uint16_t nb = (uint16_t)((b << 7) + 0x2000u);
    _Float16 normal = __builtin_bit_cast(_Float16, nb);
    _Float16 sub = (_Float16)((float)(b & 7u) * 0.001953125f);
    return (b >> 3) ? normal : sub;
}
// q >= 0 finite -> nearest E4M3 byte, ties to even, gradual underflow, saturating at 448
__device__ __forceinline__ uint32_t e4m3_rne_from_f32(float q)
{
    q = fminf(q, kFp8Max);
    uint32_t u = __float_as_uint(q);
    uint32_t bn = ((u + 0x7FFFFu + ((u >> 20) & 1u)) >> 20) - 960u;
    uint32_t bs = (uint32_t)__builtin_rintf(q * 512.0f);
    return q < 0.015625f ? bs : bn;
}

// Relative half-width of the bracket put around every fp32 quotient before it
// is rounded to a format: the fp32 evaluation (one rounded product or scale,
// one reciprocal good to 1 ulp, one rounded multiply, one more for the bracket
// itself) is off by less than 3.5 * 2^-23, so the exact quotient always lies
// strictly inside [q(1-2^-20), q(1+2^-20)].  If both ends round to the same
// code, that code is the exact answer; otherwise the decision is redone in
// fp64 by cross-multiplication, which is exact.
constexpr float kBracketLo = 1.0f - 0x1p-20f;
constexpr float kBracketHi = 1.0f + 0x1p-20f;

// Block scale of Eq. 12 for target magnitude M (6, or 4 for the second candidate of the
// scale search): E4M3 nearest to bmax / (M sg), decided exactly.  inv_msg = 1 / (M sg) in fp32.
__device__ __forceinline__ uint32_t block_scale_exact(float bmax, float sg, float inv_msg, double target = 6.0)
{
    float q = bmax * inv_msg;
    uint32_t blo = e4m3_rne_from_f32(q * kBracketLo);
    uint32_t bhi = e4m3_rne_from_f32(q * kBracketHi);
    if (__builtin_expect(blo != bhi, 0)) {
        double mid = 0.5 * ((double)e4m3_to_f32(blo) + (double)e4m3_to_f32(bhi));
        double t = mid * target * (double)sg;  // <= 5 + 2 + 24 significant bits: exact
        double b = (double)bmax;
        blo = (b > t) ? bhi : ((b < t) ? blo : ((blo & 1u) ? bhi : blo));
    }
    return blo;
}

// midpoint between E2M1 magnitude index i and i+1
__device__ __forceinline__ double e2m1_midpoint(uint32_t i)
{
    // magnitudes 0 .5 1 1.5 2 3 4 6 -> midpoints .25 .75 1.25 1.75 2.5 3.5 5
    return i < 4u ? 0.25 + 0.5 * (double)i : (i == 4u ? 2.5 : (i == 5u ? 3.5 : 5.0));
}

// Exact E2M1 decision for one element whose bracket ends gave neighbouring
// indices lo < hi: compare |x| with midpoint * s_b * s_g (<= 3 + 4 + 24 bits).
__device__ __forceinline__ uint32_t e2m1_resolve(float ax, uint32_t lo, uint32_t hi, double den)
{
    double t = e2m1_midpoint(lo) * den;
    double a = (double)ax;
    return (a > t) ? hi : ((a < t) ? lo : ((lo & 1u) ? hi : lo));
}

// 16 consecutive bf16 (8 dwords) -> 16 E2M1 codes (2 dwords) on the scale
// den = s_b * s_g.  The hardware conversion (round to nearest even, saturating,
// sign preserved) is applied to both ends of the bracket; disagreeing nibbles
// are resolved exactly.
__device__ __forceinline__ void encode_block16(const uint32_t (&w)[8], float sb, float sg,
                                               uint32_t &c0, uint32_t &c1)
{
    float d = sb * sg;
    float inv = (sb == 0.0f) ? 0.0f : __builtin_amdgcn_rcpf(d);
    float il = inv * kBracketLo, ih = inv * kBracketHi;
    uint32_t l0 = 0, l1 = 0, h0 = 0, h1 = 0;
#define NVFP4_CVT(L, H, W, SEL)                                                                   \
    L = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(L, bf16lo_to_f32(W) * il, bf16hi_to_f32(W) * il, \
                                                 1.0f, SEL);                                       \
    H = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(H, bf16lo_to_f32(W) * ih, bf16hi_to_f32(W) * ih, \
                                                 1.0f, SEL);
    NVFP4_CVT(l0, h0, w[0], 0) NVFP4_CVT(l0, h0, w[1], 1) NVFP4_CVT(l0, h0, w[2], 2) NVFP4_CVT(l0, h0, w[3], 3)
    NVFP4_CVT(l1, h1, w[4], 0) NVFP4_CVT(l1, h1, w[5], 1) NVFP4_CVT(l1, h1, w[6], 2) NVFP4_CVT(l1, h1, w[7], 3)
#undef NVFP4_CVT
    if (__builtin_expect((l0 != h0) | (l1 != h1), 0)) {
        double den = (double)sb * (double)sg;      // exact
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            uint32_t &L = (j < 8) ? l0 : l1;
            uint32_t H = (j < 8) ? h0 : h1;
            int sh = 4 * (j & 7);
            uint32_t a = (L >> sh) & 7u, b = (H >> sh) & 7u;
            if (a != b) {
                uint32_t ww = w[j >> 1];
                float ax = fabsf((j & 1) ? bf16hi_to_f32(ww) : bf16lo_to_f32(ww));
                uint32_t r = e2m1_resolve(ax, a, b, den);
                L = (L & ~(7u << sh)) | (r << sh);
            }
        }
    }
    c0 = l0;
    c1 = l1;
}

// ---- Four-over-Six scale search (Appendix "Scale Search NVFP4 Quantization", Eq. 12-13) ----
// Squared reconstruction error of a 16-element block under one candidate encoding, in fp32.
// den = s_b * s_g rounded to fp32; the codes carry the sign of x, so the decoded values are
// subtracted as they are.
__device__ __forceinline__ float block_error_f32(const uint32_t (&w)[8], uint32_t c0, uint32_t c1, float den)
{
    typedef float float2v __attribute__((ext_vector_type(2)));
    float err = 0.0f;
#define NVFP4_ERR(W, C, SEL)                                                                  \
    {                                                                                         \
        float2v q = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(C, 1.0f, SEL);                   \
        float d0 = __builtin_fmaf(-q.x, den, bf16lo_to_f32(W)), d1 = __builtin_fmaf(-q.y, den, bf16hi_to_f32(W)); \
        err = __builtin_fmaf(d0, d0, err);                                                    \
        err = __builtin_fmaf(d1, d1, err);                                                    \
    }
    NVFP4_ERR(w[0], c0, 0) NVFP4_ERR(w[1], c0, 1) NVFP4_ERR(w[2], c0, 2) NVFP4_ERR(w[3], c0, 3)
    NVFP4_ERR(w[4], c1, 0) NVFP4_ERR(w[5], c1, 1) NVFP4_ERR(w[6], c1, 2) NVFP4_ERR(w[7], c1, 3)
#undef NVFP4_ERR
    return err;
}

// The same error as the fp64 definition evaluates it: every difference |x| - m s_b s_g taken
// once in fp64, squared, and summed in element order, each operation rounded on its own (no
// fused multiply-add), so that "is candidate 4 strictly better" has one answer everywhere.
__device__ __forceinline__ double block_error_f64(const uint32_t (&w)[8], uint32_t c0, uint32_t c1, float sb, float sg)
{
    const double den = (double)sb * (double)sg;     // exact
    double err = 0.0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const uint32_t ww = w[j >> 1];
        const double a = (double)fabsf((j & 1) ? bf16hi_to_f32(ww) : bf16lo_to_f32(ww));
        const uint32_t idx = (((j < 8) ? c0 : c1) >> (4 * (j & 7))) & 7u;
        const double m = idx < 4u ? 0.5 * (double)idx : (idx == 4u ? 2.0 : (idx == 5u ? 3.0 : (idx == 6u ? 4.0 : 6.0)));
        const double d = __dsub_rn(a, __dmul_rn(m, den));
        err = __dadd_rn(err, __dmul_rn(d, d));
    }
    return err;
}

// Scale search for one block: encode with the block maximum mapped to 6 and to 4, keep the
// encoding with the strictly smaller squared error (equal errors keep 6).  The fp32 errors
// decide whenever they differ by more than their own uncertainty; otherwise fp64 does.
__device__ __forceinline__ void encode_block16_4over6(const uint32_t (&w)[8], float bmax, float sg, float inv_6sg,
                                                      float inv_4sg, uint32_t &sbyte, uint32_t &c0, uint32_t &c1)
{
    const uint32_t s6 = block_scale_exact(bmax, sg, inv_6sg, 6.0);
    const uint32_t s4 = block_scale_exact(bmax, sg, inv_4sg, 4.0);
    const float sb6 = e4m3_to_f32(s6), sb4 = e4m3_to_f32(s4);
    uint32_t a0, a1;
    encode_block16(w, sb6, sg, a0, a1);
    sbyte = s6;
    c0 = a0;
    c1 = a1;
    if (s4 == s6) return;                          // same scale, same codes, same error (zero blocks, saturated scales)
    uint32_t b0, b1;
    encode_block16(w, sb4, sg, b0, b1);
    const float den6 = sb6 * sg, den4 = sb4 * sg;
    const float e6 = block_error_f32(w, a0, a1, den6), e4 = block_error_f32(w, b0, b1, den4);
    // |d~ - d| <= 2^-24 (|x| + |x^| + 6 den) < u; |d~^2 - d^2| <= u (2 |d~| + u), and the sixteen
    // |d~| add up to at most 4 sqrt(sum d~^2) (Cauchy-Schwarz; 4.01 covers the approximate square
    // root and the rounding of the sum); sixteen fused accumulations add at most 2^-19 of the sum
    const float u6 = 0x1p-22f * (bmax + 6.0f * den6), u4 = 0x1p-22f * (bmax + 6.0f * den4);
    const float r6 = u6 * (8.02f * __builtin_amdgcn_sqrtf(e6) + 16.0f * u6) + 0x1p-19f * e6;
    const float r4 = u4 * (8.02f * __builtin_amdgcn_sqrtf(e4) + 16.0f * u4) + 0x1p-19f * e4;
    // the relative bounds above need normal fp32 numbers: errors near the underflow range
    // (and exact zeros) go to fp64 as well
    const bool tiny = fminf(e4, e6) < 0x1p-100f;
    bool pick4;
    if (!tiny && e4 + r4 < e6 - r6) pick4 = true;
    else if (!tiny && e4 - r4 > e6 + r6) pick4 = false;
    else pick4 = block_error_f64(w, b0, b1, sb4, sg) < block_error_f64(w, a0, a1, sb6, sg);
    if (pick4) {
        sbyte = s4;
        c0 = b0;
        c1 = b1;
    }
}

// Round a non-negative exact product held in a double to bf16 once (nearest
// even): go through fp32 with round-to-odd so the second rounding is innocuous.
__device__ __forceinline__ uint32_t bf16_rne_from_f64(double p)
{
    float hi = (float)p;
    double rem = p - (double)hi;                  // exact
    uint32_t u = __float_as_uint(hi);
    if (rem < 0.0) u -= 1u;                       // truncate toward zero
    if (rem != 0.0) u |= 1u;                      // sticky
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// Signed variant: nearest-even bf16 of any finite double (sign kept, also for zero results).
__device__ __forceinline__ uint32_t bf16_rne_signed_from_f64(double v)
{
    const uint32_t sign = (uint32_t)(__double_as_longlong(v) >> 48) & 0x8000u;
    return sign | bf16_rne_from_f64(fabs(v));
}

// two fp32 -> packed bf16 (round to nearest even), one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float float2v __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
    float2v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2v));
}

// K-smoothing (Sec. 3.2, Eq. 6) of one 16-element block given its row mean (a bf16 value):
// x_j -> RN_bf16(x_j - mean), one rounding of the exact difference.  An fp32 subtraction
// followed by the rounding to bf16 gives exactly that for every pair of finite bf16 numbers:
// when the exponents are at most 15 apart the fp32 difference is exact (8 + 15 + 1 bits), and
// when they are further apart the smaller operand is below 2^-15 of the larger, which is a
// bf16 number at least 2^-10 of its magnitude away from the nearest rounding boundary, so both
// the exact difference and its fp32 rounding round to that operand.
__device__ __forceinline__ void smooth_block16(uint32_t (&w)[8], float mu)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = pack_bf16x2(bf16lo_to_f32(w[i]) - mu, bf16hi_to_f32(w[i]) - mu);
}

// Random Hadamard transform (Sec. 2.2, weight-gradient operands) of one group of 16 values
// held as eight packed bf16 pairs: y = (1/4) H16 diag(s) v, H16[i][j] = (-1)^popcount(i & j),
// s_j = -1 where bit j of sign_mask is set.  Fast Walsh-Hadamard butterflies in fp64 (exact
// while the 16 values span less than 2^40), one rounding to bf16.
__device__ __forceinline__ void rht_block16(uint32_t (&w)[8], uint32_t sign_mask)
{
    double v[16];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v[2 * i] = (double)bf16lo_to_f32(w[i]);
        v[2 * i + 1] = (double)bf16hi_to_f32(w[i]);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j)
        if ((sign_mask >> j) & 1u) v[j] = -v[j];
#pragma unroll
    for (int h = 1; h < 16; h <<= 1)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if ((i & h) == 0) {
                const double a = v[i], b = v[i + h];
                v[i] = a + b;
                v[i + h] = a - b;
            }
#pragma unroll
    for (int i = 0; i < 8; ++i)
        w[i] = bf16_rne_signed_from_f64(0.25 * v[2 * i]) | (bf16_rne_signed_from_f64(0.25 * v[2 * i + 1]) << 16);
}

// global scale from the tensor's largest |bf16| pattern: RN_fp32(amax / 2688), 1 if zero
__device__ __forceinline__ float global_scale_from_amax_bits(uint32_t amax_bits16)
{
    float amax = __uint_as_float(amax_bits16 << 16);
    // IEEE division; 2688 = 448 * 6
    return amax_bits16 == 0u ? 1.0f : __fdiv_rn(amax, kFp8Max * kFp4Max);
}

}  // namespace nvfp4
