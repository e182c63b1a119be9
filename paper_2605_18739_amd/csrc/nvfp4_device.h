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

// Block scale of Eq. 12 (target 6): E4M3 nearest to bmax / (6 sg), decided exactly.
__device__ __forceinline__ uint32_t block_scale_exact(float bmax, float sg, float inv_6sg)
{
    float q = bmax * inv_6sg;
    uint32_t blo = e4m3_rne_from_f32(q * kBracketLo);
    uint32_t bhi = e4m3_rne_from_f32(q * kBracketHi);
    if (__builtin_expect(blo != bhi, 0)) {
        double mid = 0.5 * ((double)e4m3_to_f32(blo) + (double)e4m3_to_f32(bhi));
        double t = mid * 6.0 * (double)sg;     // <= 5 + 2 + 24 significant bits: exact
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

// global scale from the tensor's largest |bf16| pattern: RN_fp32(amax / 2688), 1 if zero
__device__ __forceinline__ float global_scale_from_amax_bits(uint32_t amax_bits16)
{
    float amax = __uint_as_float(amax_bits16 << 16);
    // IEEE division; 2688 = 448 * 6
    return amax_bits16 == 0u ? 1.0f : __fdiv_rn(amax, kFp8Max * kFp4Max);
}

}  // namespace nvfp4
