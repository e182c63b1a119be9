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
typedef short short4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

namespace nvfp4 {

constexpr int kWave = 64;
constexpr float kFp4Max = 6.0f;      // M^FP4
constexpr float kFp8Max = 448.0f;    // M^FP8

__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// two fp32 -> packed bf16 (round to nearest even), one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float float2v __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
    float2v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2v));
}

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

// Settle the nibbles on which the two ends of the bracket disagree.  l holds the codes of the lower end, h of the
// upper end (neighbouring magnitudes, same sign).  Such an element lies within 2^-19 of the midpoint T between the
// two magnitudes times s_b s_g, and which side it lies on is the sign of  T s_b s_g - |x|:  c = T s_b is exact in
// fp32 (3 + 4 bits), the fused multiply-add rounds c s_g - |x| once, and because the two terms nearly cancel
// (the difference has at most 12 significant bits) that one rounding is exact.  Tensor scales so small that the
// difference could leave the normal range take the same comparison in fp64.  A tie goes to the even code.
// One nibble per pass of the loop; a wave runs as many passes as its busiest lane needs (rarely more than two).
__device__ __forceinline__ void resolve_codes(const uint32_t (&w)[8], float sb, float sg, uint32_t &l0, uint32_t &l1,
                                              uint32_t h0, uint32_t h1)
{
    typedef float float2v __attribute__((ext_vector_type(2)));
    uint32_t d0 = l0 ^ h0, d1 = l1 ^ h1;
    const bool wide = sg >= 0x1p-80f;                                      // (the same for every lane)
    while (__builtin_expect((d0 | d1) != 0u, 0)) {                         // (selects, no branches, inside)
        const bool first = d0 != 0u;
        const uint32_t d = first ? d0 : d1, lw = first ? l0 : l1;
        const uint32_t sh = (uint32_t)__builtin_ctz(d) & 28u;              // bit position of the nibble in its word
        const bool odd = (sh & 8u) != 0u, upper = (sh & 16u) != 0u;        // which of the word's four bf16 pairs
        const uint32_t w01 = odd ? w[1] : w[0], w23 = odd ? w[3] : w[2];
        const uint32_t w45 = odd ? w[5] : w[4], w67 = odd ? w[7] : w[6];
        const uint32_t wlo = upper ? w23 : w01, whi = upper ? w67 : w45;
        const uint32_t ww = first ? wlo : whi;
        const float ax = __uint_as_float((ww >> ((sh & 4u) << 2) << 16) & 0x7FFF0000u);
        const uint32_t lo = (lw >> sh) & 7u;
        const float2v m = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(lo | ((lo + 1u) << 4), 1.0f, 0);
        const float c = (0.5f * (m.x + m.y)) * sb;                         // midpoint times block scale, exact
        bool above, equal;
        if (wide) {
            const float t = __builtin_fmaf(c, sg, -ax);
            above = t < 0.0f;
            equal = t == 0.0f;
        } else {
            const double t = (double)c * (double)sg, a = (double)ax;
            above = a > t;
            equal = a == t;
        }
        const bool up = above | (equal & ((lo & 1u) != 0u));
        const uint32_t nib = d & (0xFu << sh);
        const uint32_t nw = lw ^ (up ? nib : 0u), nd = d ^ nib;
        l0 = first ? nw : l0;
        l1 = first ? l1 : nw;
        d0 = first ? nd : d0;
        d1 = first ? d1 : nd;
    }
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
    resolve_codes(w, sb, sg, l0, l1, h0, h1);
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
// (A rolled loop: the fallback is inlined wherever a block is encoded and taken rarely, so it is written for
// small code, not for speed.)
__device__ __forceinline__ double block_error_f64(const uint32_t (&w)[8], uint32_t c0, uint32_t c1, float sb, float sg)
{
    // (under the default contraction mode the compiler fuses these into multiply-adds: one rounding where the
    //  definition has two, and a different answer on blocks whose two errors are equal in exact arithmetic)
#pragma clang fp contract(off)
    typedef float float2v __attribute__((ext_vector_type(2)));
    const double den = (double)sb * (double)sg;     // exact
    double err = 0.0;
#pragma unroll 1
    for (uint32_t j = 0; j < 16; ++j) {
        const bool odd = (j & 2u) != 0u, upper = (j & 4u) != 0u, second = (j & 8u) != 0u;
        const uint32_t w01 = odd ? w[1] : w[0], w23 = odd ? w[3] : w[2], w45 = odd ? w[5] : w[4], w67 = odd ? w[7] : w[6];
        const uint32_t wlo = upper ? w23 : w01, whi = upper ? w67 : w45;
        const uint32_t ww = second ? whi : wlo;
        const double a = (double)__uint_as_float((ww >> ((j & 1u) << 4) << 16) & 0x7FFF0000u);
        const uint32_t idx = ((second ? c1 : c0) >> (4u * (j & 7u))) & 7u;
        const float2v m = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(idx, 1.0f, 0);       // the code's magnitude, exact
        const double prod = (double)m.x * den;            // (plain operators: contraction is switched off for this function;
        const double d = a - prod;                         //  the rounding intrinsics are inlined with the contraction mode
        const double sq = d * d;                           //  of their own header and would be fused all the same)
        err = err + sq;
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

// ---- tensor scales outside the range in which the fp32 quotients above are safe ----------------------
// Below s_g = 2^-100 or above 2^100 the reciprocal 1 / (M s_g) or the products s_b s_g leave the normal fp32
// range.  Every decision of the quantizer compares ratios, so it commutes with multiplying the tensor AND its
// scale by a power of two: such tensors are encoded as (x 2^k, s_g 2^k) with k = +96 or -96, which puts the scale
// back into range.  The scaled elements are exact (bf16 has the exponent range of fp32) except those that underflow
// when a huge tensor is scaled down: they are below 2^-30, more than a hundred binades under a quarter of the
// smallest block scale times s_g, so their code is zero either way, and so is the scale of a block made of them.
// The stored tensor scale is the unscaled one.  The test is the same for every lane: a scalar branch.
__device__ __forceinline__ bool scale_out_of_range(float sg) { return !(sg >= 0x1p-100f && sg <= 0x1p100f); }
__device__ __forceinline__ float range_shift(float sg) { return sg < 0x1p-100f ? 0x1p96f : (sg > 0x1p100f ? 0x1p-96f : 1.0f); }
__device__ __forceinline__ void rescale_block16(uint32_t (&w)[8], float f)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = pack_bf16x2(bf16lo_to_f32(w[i]) * f, bf16hi_to_f32(w[i]) * f);
}

// ---- straight-line forms for kernels that hold many blocks per lane -------------------------------
// The functions above take one block from start to end.  The forms below run two independent chains of
// work through one stretch of code -- two blocks for the plain rule, the two candidates of one block for
// the scale search -- so that the latency of one chain's dependent instructions (a conversion writes one
// byte of its destination, so the four that fill a code word wait on one another) hides behind the other.
// The results are the exact ones: the common case is decided by fp32 arithmetic alone, and the rare
// near-tie drops into the same exact resolution the functions above use.

// Block scale byte for quotient q = bmax * inv_msg in the normal E4M3 range, by integer arithmetic on
// the bits of q.  "unsure" is raised when q lies within 24 ulps of a rounding tie (the true quotient lies
// within 16 ulps of q), below the normal range (subnormal scales, zero blocks), or is not an ordinary
// number; the caller then calls block_scale_exact.
__device__ __forceinline__ uint32_t block_scale_fast(float q, bool &unsure)
{
    q = fminf(q, kFp8Max);
    const uint32_t u = __float_as_uint(q);
    const uint32_t b = ((u + 0x7FFFFu + ((u >> 20) & 1u)) >> 20) - 960u;
    unsure = ((u & 0xFFFFFu) - (0x80000u - 24u) <= 48u) | !(q >= 0.015625f * 1.0001f);
    return b;
}

// E4M3 byte (normal range, as block_scale_fast returns it) -> f32, one instruction
__device__ __forceinline__ float e4m3_normal_to_f32(uint32_t b) { return __uint_as_float((b << 20) + (120u << 23)); }

// largest magnitude of 16 bf16 values as a float (exact: a maximum of exact values)
__device__ __forceinline__ float block_absmax_f32(const uint32_t (&w)[8])
{
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) m = fmaxf(fmaxf(fabsf(bf16lo_to_f32(w[i])), fabsf(bf16hi_to_f32(w[i]))), m);
    return m;
}

// sixteen values -> their largest magnitude through a tree of three-operand maxima (depth 3 instead of 8)
__device__ __forceinline__ float absmax16_tree(const float (&f)[16])
{
    auto m3 = [](float a, float b, float c) { return fmaxf(fmaxf(fabsf(a), fabsf(b)), fabsf(c)); };
    const float t0 = m3(f[0], f[1], f[2]), t1 = m3(f[3], f[4], f[5]), t2 = m3(f[6], f[7], f[8]);
    const float t3 = m3(f[9], f[10], f[11]), t4 = m3(f[12], f[13], f[14]);
    return fmaxf(m3(t0, t1, t2), m3(t3, t4, f[15]));
}

__device__ __forceinline__ void unpack16(const uint32_t (&w)[8], float (&f)[16])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        f[2 * i] = bf16lo_to_f32(w[i]);
        f[2 * i + 1] = bf16hi_to_f32(w[i]);
    }
}

// Scale byte, its value and the reciprocal of s_b s_g for one block (target magnitude M = 6 or 4).
__device__ __forceinline__ void block_scale_inline(float bmax, float sg, float inv_msg, double target, uint32_t &sbyte,
                                                   float &sb, float &inv)
{
    bool unsure;
    sbyte = block_scale_fast(bmax * inv_msg, unsure);
    sb = e4m3_normal_to_f32(sbyte);
    inv = __builtin_amdgcn_rcpf(sb * sg);
    if (__builtin_expect(unsure, 0)) {
        sbyte = block_scale_exact(bmax, sg, inv_msg, target);
        sb = e4m3_to_f32(sbyte);
        inv = (sb == 0.0f) ? 0.0f : __builtin_amdgcn_rcpf(sb * sg);
    }
}

// one step of four conversions: pair K of the block(s) into byte K % 4 of code word K / 4, for four chains
#define NVFP4_CVT4(K, SEL, A, FA, MA, B, FB, MB, C, FC, MC, D, FD, MD)                                              \
    A[K >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(A[K >> 2], FA[2 * K] * MA, FA[2 * K + 1] * MA, 1.0f, SEL);  \
    B[K >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(B[K >> 2], FB[2 * K] * MB, FB[2 * K + 1] * MB, 1.0f, SEL);  \
    C[K >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(C[K >> 2], FC[2 * K] * MC, FC[2 * K + 1] * MC, 1.0f, SEL);  \
    D[K >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(D[K >> 2], FD[2 * K] * MD, FD[2 * K + 1] * MD, 1.0f, SEL);

// Plain rule (Eq. 1: block maximum -> 6) on two blocks side by side; the results of quantize_block16_exact
// for tensor scales inside the fp32-safe range.
__device__ __forceinline__ void quantize_pair16(const uint32_t (&wa)[8], const uint32_t (&wb)[8], float sg, float inv_6sg,
                                                uint32_t &sa, uint32_t &a0, uint32_t &a1,
                                                uint32_t &sb, uint32_t &b0, uint32_t &b1)
{
    float fa[16], fb[16];
    unpack16(wa, fa);
    unpack16(wb, fb);
    float sva, svb, inva, invb;
    block_scale_inline(absmax16_tree(fa), sg, inv_6sg, 6.0, sa, sva, inva);
    block_scale_inline(absmax16_tree(fb), sg, inv_6sg, 6.0, sb, svb, invb);
    const float ila = inva * kBracketLo, iha = inva * kBracketHi, ilb = invb * kBracketLo, ihb = invb * kBracketHi;
    uint32_t la[2] = {0, 0}, ha[2] = {0, 0}, lb[2] = {0, 0}, hb[2] = {0, 0};
#define NVFP4_STEP(K, SEL) NVFP4_CVT4(K, SEL, la, fa, ila, ha, fa, iha, lb, fb, ilb, hb, fb, ihb)
    NVFP4_STEP(0, 0) NVFP4_STEP(1, 1) NVFP4_STEP(2, 2) NVFP4_STEP(3, 3)
    NVFP4_STEP(4, 0) NVFP4_STEP(5, 1) NVFP4_STEP(6, 2) NVFP4_STEP(7, 3)
#undef NVFP4_STEP
    resolve_codes(wa, sva, sg, la[0], la[1], ha[0], ha[1]);
    resolve_codes(wb, svb, sg, lb[0], lb[1], hb[0], hb[1]);
    a0 = la[0]; a1 = la[1];
    b0 = lb[0]; b1 = lb[1];
}

// Scale search (Eq. 12-13) on one block, the two candidates side by side; the results of
// quantize_block16_4over6_exact for tensor scales inside the fp32-safe range.  The fp32 squared errors
// are summed in four partial sums (the bound r of encode_block16_4over6 holds for any order of summation).
__device__ __forceinline__ void quantize_block16_4over6_inline(const uint32_t (&w)[8], float sg, float inv_6sg, float inv_4sg,
                                                               uint32_t &sbyte, uint32_t &c0, uint32_t &c1)
{
    typedef float float2v __attribute__((ext_vector_type(2)));
    float f[16];
    unpack16(w, f);
    const float bmax = absmax16_tree(f);
    uint32_t s6, s4;
    float sb6, sb4, inv6, inv4;
    block_scale_inline(bmax, sg, inv_6sg, 6.0, s6, sb6, inv6);
    block_scale_inline(bmax, sg, inv_4sg, 4.0, s4, sb4, inv4);
    const float il6 = inv6 * kBracketLo, ih6 = inv6 * kBracketHi, il4 = inv4 * kBracketLo, ih4 = inv4 * kBracketHi;
    // The candidates are compared on the codes of the LOWER bracket end alone; the upper end is converted for the
    // winner only, whose near-ties are then settled.  A nibble on which the two ends would disagree lies within
    // 2^-19 of a midpoint T between magnitudes T -+ h, so its squared error changes by the factor
    // 1 +- 4 (T / h) 2^-19 at most when the nibble flips, and T / h <= 7: the settled codes' error lies within
    // 2^-14 (e + r) of the error e that is computed here, which the uncertainty r below takes in.
    uint32_t l6[2] = {0, 0}, l4[2] = {0, 0};
#define NVFP4_STEP(K, SEL)                                                                                              \
    l6[K >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(l6[K >> 2], f[2 * K] * il6, f[2 * K + 1] * il6, 1.0f, SEL);   \
    l4[K >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(l4[K >> 2], f[2 * K] * il4, f[2 * K + 1] * il4, 1.0f, SEL);
    NVFP4_STEP(0, 0) NVFP4_STEP(1, 1) NVFP4_STEP(2, 2) NVFP4_STEP(3, 3)
    NVFP4_STEP(4, 0) NVFP4_STEP(5, 1) NVFP4_STEP(6, 2) NVFP4_STEP(7, 3)
#undef NVFP4_STEP
    const float den6 = sb6 * sg, den4 = sb4 * sg;
    float e6a = 0.0f, e6b = 0.0f, e4a = 0.0f, e4b = 0.0f;
#define NVFP4_STEP(K, SEL)                                                                                        \
    {                                                                                                             \
        const float2v q6 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(l6[K >> 2], 1.0f, SEL);                       \
        const float2v q4 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(l4[K >> 2], 1.0f, SEL);                       \
        const float d60 = __builtin_fmaf(-q6.x, den6, f[2 * K]), d61 = __builtin_fmaf(-q6.y, den6, f[2 * K + 1]); \
        const float d40 = __builtin_fmaf(-q4.x, den4, f[2 * K]), d41 = __builtin_fmaf(-q4.y, den4, f[2 * K + 1]); \
        e6a = __builtin_fmaf(d60, d60, e6a);                                                                      \
        e6b = __builtin_fmaf(d61, d61, e6b);                                                                      \
        e4a = __builtin_fmaf(d40, d40, e4a);                                                                      \
        e4b = __builtin_fmaf(d41, d41, e4b);                                                                      \
    }
    NVFP4_STEP(0, 0) NVFP4_STEP(1, 1) NVFP4_STEP(2, 2) NVFP4_STEP(3, 3)
    NVFP4_STEP(4, 0) NVFP4_STEP(5, 1) NVFP4_STEP(6, 2) NVFP4_STEP(7, 3)
#undef NVFP4_STEP
    const float e6 = e6a + e6b, e4 = e4a + e4b;
    const float u6 = 0x1p-22f * (bmax + 6.0f * den6), u4 = 0x1p-22f * (bmax + 6.0f * den4);
    float r6 = u6 * (8.02f * __builtin_amdgcn_sqrtf(e6) + 16.0f * u6) + 0x1p-19f * e6;   // (eight fused steps and one
    float r4 = u4 * (8.02f * __builtin_amdgcn_sqrtf(e4) + 16.0f * u4) + 0x1p-19f * e4;   //  addition: below 2^-19 as well)
    r6 = __builtin_fmaf(0x1p-14f, e6, 1.0001f * r6);
    r4 = __builtin_fmaf(0x1p-14f, e4, 1.0001f * r4);
    const bool tiny = fminf(e4, e6) < 0x1p-100f;
    const bool same = s4 == s6;                    // (saturated scales, zero blocks: same codes, same error, 6 is kept)
    bool pick4 = e4 + r4 < e6 - r6;
    auto upper_end = [&](float ih, uint32_t (&h)[2]) {
        h[0] = h[1] = 0u;
#define NVFP4_STEP(K, SEL) h[K >> 2] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(h[K >> 2], f[2 * K] * ih, f[2 * K + 1] * ih, 1.0f, SEL);
        NVFP4_STEP(0, 0) NVFP4_STEP(4, 0) NVFP4_STEP(1, 1) NVFP4_STEP(5, 1)
        NVFP4_STEP(2, 2) NVFP4_STEP(6, 2) NVFP4_STEP(3, 3) NVFP4_STEP(7, 3)
#undef NVFP4_STEP
    };
    if (__builtin_expect(!same & (tiny | !(pick4 | (e4 - r4 > e6 + r6))), 0)) {     // too close in fp32: settle both, compare in fp64
        uint32_t h6[2], h4[2];
        upper_end(ih6, h6);
        upper_end(ih4, h4);
        resolve_codes(w, sb6, sg, l6[0], l6[1], h6[0], h6[1]);
        resolve_codes(w, sb4, sg, l4[0], l4[1], h4[0], h4[1]);
        pick4 = block_error_f64(w, l4[0], l4[1], sb4, sg) < block_error_f64(w, l6[0], l6[1], sb6, sg);
    }
    pick4 &= !same;
    sbyte = pick4 ? s4 : s6;
    c0 = pick4 ? l4[0] : l6[0];
    c1 = pick4 ? l4[1] : l6[1];
    uint32_t hw[2];
    upper_end(pick4 ? ih4 : ih6, hw);
    resolve_codes(w, pick4 ? sb4 : sb6, sg, c0, c1, hw[0], hw[1]);   // (settled codes pass through unchanged)
}
#undef NVFP4_CVT4

// the one-block-at-a-time counterparts, for any tensor scale (sgq, inv_6sgq, inv_4sgq: the scale after range_shift)
__device__ __forceinline__ void quantize_block16_exact(uint32_t (&w)[8], float shift, float sgq, float inv_6sgq, uint32_t &sbyte,
                                                       uint32_t &c0, uint32_t &c1)
{
    if (__builtin_expect(shift != 1.0f, 0)) rescale_block16(w, shift);
    sbyte = block_scale_exact(block_absmax_f32(w), sgq, inv_6sgq);
    encode_block16(w, e4m3_to_f32(sbyte), sgq, c0, c1);
}

__device__ __forceinline__ void quantize_block16_4over6_exact(uint32_t (&w)[8], float shift, float sgq, float inv_6sgq,
                                                              float inv_4sgq, uint32_t &sbyte, uint32_t &c0, uint32_t &c1)
{
    if (__builtin_expect(shift != 1.0f, 0)) rescale_block16(w, shift);
    encode_block16_4over6(w, block_absmax_f32(w), sgq, inv_6sgq, inv_4sgq, sbyte, c0, c1);
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
        // (+ 0.0: a sum that is zero is +0, as when the terms are added up from zero; only groups of negative zeros differ)
        w[i] = bf16_rne_signed_from_f64(0.25 * v[2 * i] + 0.0) | (bf16_rne_signed_from_f64(0.25 * v[2 * i + 1] + 0.0) << 16);
}

// The same transform in fp32 arithmetic, and the test that tells when it returns the same bits.  With all non-zero
// magnitudes of the group within 12 binades of the largest, every value is a multiple of 2^(e_min - 7) and every
// partial sum stays below 2^(e_max + 5): at most 24 significant bits, so fp32 sums of the sixteen terms are exact in
// any order and the one rounding to bf16 (v_cvt_pk_bf16_f32, nearest even) is the rounding of the exact value, as in
// the fp64 form.  Groups near the ends of the exponent range (sums that could overflow, results that could be
// subnormal) fail the test; a group of zeros passes it.  Gaussian data fails it in about 1 % of the groups.
// e_max and e_min are the largest and the smallest exponent field among the non-zero elements.
__device__ __forceinline__ void rht_exponent_range(const uint32_t (&w)[8], int &emax, int &emin, bool &all_zero)
{
    const ushort2v one = {1, 1};
    ushort2v mx = {0, 0}, mn = {0xFFFF, 0xFFFF};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const ushort2v a = __builtin_bit_cast(ushort2v, w[i]) << one;          // sign dropped: exponent in bits 15..8
        mx = __builtin_elementwise_max(mx, a);
        mn = __builtin_elementwise_min(mn, a - one);                            // zeros wrap to 0xFFFF and never win
    }
    const uint32_t hmax = max((uint32_t)mx.x, (uint32_t)mx.y), hmin = min((uint32_t)mn.x, (uint32_t)mn.y) + 1u;
    emax = (int)(hmax >> 8);
    emin = max((int)(hmin >> 8), 1);
    all_zero = hmax == 0u;
}
__device__ __forceinline__ bool rht_fp32_is_exact(const uint32_t (&w)[8])
{
    int emax, emin;
    bool all_zero;
    rht_exponent_range(w, emax, emin, all_zero);
    return all_zero | (emax >= 40 && emax <= 240 && emax - emin <= 12);
}

// The fp32 sums are taken on the matrix pipes.  v_mfma_f32_4x4x4_16B_bf16 multiplies, for each group of four
// lanes, a 4x4 matrix A (lane i of the group supplies row i) by a 4x4 matrix B (lane j supplies column j, four bf16
// in two registers) and adds a 4x4 fp32 matrix whose column j lane j holds: a lane's own four values go in, its own
// four sums come out, nothing crosses lanes but the constant A.  H16 = H4 (x) H4, so with the group's sixteen values
// x[4 g + k] and output index 4 a + b,   y[4 a + b] = sum_g sum_k ( (1/4) H4[a][g] H4[b][k] s[4 g + k] ) x[4 g + k]:
// sixteen instructions (four accumulating chains of four), A = +-(1/4) H4 diag(s) for k-group g.  The products
// (+-1/4 times a bf16 number) are exact and the sums are the ones the test above covers.  A sum of zero terms and a
// sum that cancels come out as +0, as in the fp64 form.
struct RhtRows {
    uint32_t pos[4][2], neg[4][2];      // row (lane % 4) of (1/4) H4 diag(s_4g .. s_4g+3), and of its negative, as bf16 pairs
};
__device__ __forceinline__ RhtRows rht_rows(uint32_t sign_mask, uint32_t lane)
{
    RhtRows h;
    const uint32_t b0 = lane & 1u, b1 = (lane >> 1) & 1u;                 // H4[b][k] = (-1)^popcount(b & k)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const uint32_t s = sign_mask >> (4 * g);
        const uint32_t n0 = s & 1u, n1 = (b0 ^ (s >> 1)) & 1u, n2 = (b1 ^ (s >> 2)) & 1u, n3 = (b0 ^ b1 ^ (s >> 3)) & 1u;
        h.pos[g][0] = 0x3E803E80u ^ (n0 << 15) ^ (n1 << 31);              // 0x3E80: 1/4 in bf16
        h.pos[g][1] = 0x3E803E80u ^ (n2 << 15) ^ (n3 << 31);
        h.neg[g][0] = h.pos[g][0] ^ 0x80008000u;
        h.neg[g][1] = h.pos[g][1] ^ 0x80008000u;
    }
    return h;
}
// (no branch around this function may diverge within a wave: matrix instructions are issued for the whole wave)
__device__ __forceinline__ void rht_block16_mfma(const uint32_t (&w)[8], const RhtRows &h, float (&y)[16])
{
    float4v acc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) acc[a] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const uint2v bw = {w[2 * g], w[2 * g + 1]};
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const bool minus = ((a & g) == 1) | ((a & g) == 2);            // H4[a][g] = -1
            const uint2v aw = {minus ? h.neg[g][0] : h.pos[g][0], minus ? h.neg[g][1] : h.pos[g][1]};
            acc[a] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(short4v, aw), __builtin_bit_cast(short4v, bw),
                                                            acc[a], 0, 0, 0);
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int i = 0; i < 4; ++i) y[4 * a + i] = acc[a][i];
}
__device__ __forceinline__ void pack16(const float (&y)[16], uint32_t (&w)[8])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = pack_bf16x2(y[2 * i], y[2 * i + 1]);
}

// Groups that span up to 25 binades: the elements within 12 binades of the largest and the smaller ones are
// transformed separately (each set passes the test above on its own), which gives the exact result as the sum of
// two fp32 numbers L + S.  fl(L + S) lies within half an fp32 ulp of it, and nearest-even rounding to bf16 is
// constant between consecutive bf16 midpoints, which are fp32 numbers: the two round alike unless fl(L + S) is
// itself such a midpoint (low sixteen bits 0x8000).  Returns false, and leaves w as it was, for a group it cannot
// settle this way (a wider span, the ends of the exponent range, a sum on a midpoint): those take the fp64 form.
__device__ __forceinline__ bool rht_block16_mfma_split(uint32_t (&w)[8], const RhtRows &h)
{
    int emax, emin;
    bool all_zero;
    rht_exponent_range(w, emax, emin, all_zero);
    const bool in_range = emax >= 40 && emax <= 240 && emax - emin <= 25;
    const uint32_t t = ((uint32_t)max(emax - 12, 1) << 8) - 1u;           // keep halves whose (bits << 1) exceed this
    const ushort2v thr = {(unsigned short)t, (unsigned short)t}, one = {1, 1}, ones = {0xFFFF, 0xFFFF};
    uint32_t big[8], small[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const ushort2v a = __builtin_bit_cast(ushort2v, w[i]) << one;
        const ushort2v keep = __builtin_elementwise_min(__builtin_elementwise_sub_sat(a, thr), one) * ones;   // 0xFFFF or 0
        big[i] = w[i] & __builtin_bit_cast(uint32_t, keep);
        small[i] = w[i] ^ big[i];
    }
    float L[16], S[16];
    rht_block16_mfma(big, h, L);
    rht_block16_mfma(small, h, S);
    uint32_t r[8], hit = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float y0 = L[2 * i] + S[2 * i], y1 = L[2 * i + 1] + S[2 * i + 1];
        const uint32_t low = __builtin_amdgcn_perm(__float_as_uint(y1), __float_as_uint(y0), 0x05040100u) ^ 0x80008000u;
        hit = __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(ushort2v, hit), __builtin_bit_cast(ushort2v, low)));
        r[i] = pack_bf16x2(y0, y1);
    }
    const bool ok = in_range & ((hit & 0xFFFFu) != 0u) & ((hit >> 16) != 0u);
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = ok ? r[i] : w[i];
    return ok;
}

// global scale from the tensor's largest |bf16| pattern: RN_fp32(amax / 2688), 1 if zero
__device__ __forceinline__ float global_scale_from_amax_bits(uint32_t amax_bits16)
{
    float amax = __uint_as_float(amax_bits16 << 16);
    // IEEE division; 2688 = 448 * 6
    return amax_bits16 == 0u ? 1.0f : __fdiv_rn(amax, kFp8Max * kFp4Max);
}

}  // namespace nvfp4
