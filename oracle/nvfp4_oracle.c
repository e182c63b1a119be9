/*
 * NVFP4 CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 implementation of what the NVFP4 hot path computes,
 * written from the paper's definition of the format (Sec. 2.2 "NVFP4
 * Preliminaries", Eq. 2; Appendix "Scale Search NVFP4 Quantization",
 * Eq. 12-13; Sec. 3.2 "Parallel KV Quantization", Eq. 5-6).  It shares no
 * code with the HIP library and is only ever called from tests, the smoke
 * check and the bench's cpu_baseline leg.
 *
 * Format (Eq. 2):  X^ = X^FP4 * alpha^FP8 * alpha^FP32
 *   X^FP4      E2M1 value, one of {0, .5, 1, 1.5, 2, 3, 4, 6} with a sign
 *   alpha^FP8  E4M3 scale shared by 16 consecutive elements along K
 *   alpha^FP32 one FP32 scale per tensor
 * with M^FP8 = 448 and M^FP4 = 6 (Sec. 2.2) and the rule that the block
 * maximum maps to FP4 magnitude 6 (Appendix, first paragraph):
 *   alpha^FP32 = max|X| / (448 * 6)                              rounded to FP32
 *   alpha^FP8_i = cast_E4M3( max_{j in B_i}|X_j| / (6 alpha^FP32) )   (Eq. 12)
 *   X^FP4_j   = cast_E2M1( X_j / (alpha^FP8_i alpha^FP32) )
 *
 * Reading used everywhere: the formulas are evaluated in exact real
 * arithmetic and rounded once at each stored format, round-to-nearest with
 * ties to the even mantissa, saturating at the format maximum.  "Exact" is
 * realised by never forming a quotient: "v is nearest to num/den" is decided
 * by comparing num with mid*den for the midpoints between neighbouring
 * format values.  Every such product has at most 31 significant bits here
 * (<= 5 for a midpoint, 2 for the factor 6, 24 for an FP32), so fp64
 * evaluates it without rounding.
 *
 * Every function with a pin in tests/ names it; none is "parity unpinned"
 * except where stated.
 */
#include "nvfp4_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- formats */

/* E2M1 magnitudes, index = low three code bits (Appendix: the FP4 value set). */
static const double E2M1_MAG[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

double nvfp4o_e2m1_decode(unsigned code)
{
    double m = E2M1_MAG[code & 7u];
    return (code & 8u) ? -m : m;
}

/* E4M3 (1-4-3, bias 7, no infinities, 0x7F/0xFF are NaN, largest 448). */
double nvfp4o_e4m3_decode(unsigned byte)
{
    unsigned e = (byte >> 3) & 15u, m = byte & 7u;
    double v;
    if (e == 15u && m == 7u) return NAN;
    if (e == 0u) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, (int)e - 7);
    return (byte & 0x80u) ? -v : v;
}

double nvfp4o_bf16_decode(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Round a double to the nearest bf16 (8-bit significand, FP32 exponent range,
 * gradual underflow), ties to even; one rounding.  v/ulp is exact because ulp
 * is a power of two, and nearbyint rounds to nearest-even in the default
 * rounding mode. */
uint16_t nvfp4o_bf16_rne(double v)
{
    double a = fabs(v), r;
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    int e;
    float f;
    uint32_t u;
    if (a == 0.0) return sign;
    if (isnan(v)) return 0x7FC0u;
    (void)frexp(a, &e);            /* a = m * 2^e, m in [0.5, 1) => floor(log2 a) = e - 1 */
    e -= 1;
    if (e < -126) e = -126;        /* subnormal bf16 share the exponent of 2^-126 */
    r = ldexp(nearbyint(ldexp(a, 7 - e)), e - 7);
    f = (float)r;                  /* exact: r has <= 8 significant bits (or overflows to inf) */
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(sign | (u >> 16));
}

/* Index of the value nearest to the real number num/den among the ascending
 * list v[0..n-1] (v[0] = 0), ties to the even index, saturating at v[n-1].
 * num >= 0, den >= 0.  den == 0 gives index 0 (nothing can be represented on
 * a zero scale; also covers the all-zero block). */
static int nearest_ratio(const double *v, int n, double num, double den)
{
    int i;
    if (den == 0.0) return 0;
    for (i = 0; i + 1 < n; ++i) {
        double mid = 0.5 * (v[i] + v[i + 1]);
        double t = mid * den;               /* exact, see header */
        if (num < t) return i;
        if (num == t) return (i & 1) ? i + 1 : i;
    }
    return n - 1;
}

static double E4M3_POS[127];   /* bytes 0x00..0x7E ascending */
static int tables_ready = 0;
static void init_tables(void)
{
    int b;
    if (tables_ready) return;
    for (b = 0; b < 127; ++b) E4M3_POS[b] = nvfp4o_e4m3_decode((unsigned)b);
#pragma omp atomic write
    tables_ready = 1;
}

/* cast_E4M3(num/den): byte of the nearest non-negative E4M3 value (Eq. 12's
 * cast), RNE on the 3-bit mantissa (byte parity = mantissa parity), gradual
 * underflow, saturating at 448 = 0x7E. */
int nvfp4o_e4m3_cast_ratio(double num, double den)
{
    init_tables();
    return nearest_ratio(E4M3_POS, 127, num, den);
}

/* cast_E2M1(|num|/den): magnitude index 0..7, RNE on the single mantissa bit
 * (index parity = mantissa bit), saturating at 6. */
int nvfp4o_e2m1_cast_ratio(double num, double den)
{
    return nearest_ratio(E2M1_MAG, 8, num, den);
}

/* ------------------------------------------------------------ quantizer */

/* element (row r of the OUTPUT, position k along its K) of the input matrix */
static inline uint16_t in_elem(const uint16_t *x, int64_t ld, int block_axis, int64_t r, int64_t k)
{
    return block_axis == 0 ? x[r * ld + k] : x[k * ld + r];
}

/* alpha^FP32 = amax / (M^FP8 * M^FP4), rounded to FP32; 1.0 for an all-zero
 * tensor.  amax/2688 is formed in fp64 and then rounded to fp32: 2688 = 2^7*21
 * and amax has 8 significant bits, so the quotient is either exact in a few
 * bits or has a periodic expansion of period 6 that cannot lie within 2^-53
 * of a 25-bit midpoint -- the double rounding is the single rounding. */
float nvfp4o_global_scale(const uint16_t *x, int64_t R, int64_t C, int64_t ld)
{
    double amax = 0.0;
    int64_t r, c;
    for (r = 0; r < R; ++r)
        for (c = 0; c < C; ++c) {
            double a = fabs(nvfp4o_bf16_decode(x[r * ld + c]));
            if (a > amax) amax = a;
        }
    if (amax == 0.0) return 1.0f;
    return (float)(amax / (448.0 * 6.0));
}

/* One block of 16: scale byte and 16 codes, given the tensor scale. */
static void quantize_block(const double *xb, double sg, uint8_t *scale_byte, uint8_t *code16)
{
    double bmax = 0.0, sb, den;
    int j, sbyte;
    for (j = 0; j < 16; ++j)
        if (fabs(xb[j]) > bmax) bmax = fabs(xb[j]);
    sbyte = nvfp4o_e4m3_cast_ratio(bmax, 6.0 * sg);       /* Eq. 12, target 6 */
    sb = nvfp4o_e4m3_decode((unsigned)sbyte);
    den = sb * sg;                                        /* exact: 4 + 24 bits */
    for (j = 0; j < 16; ++j) {
        int idx = nvfp4o_e2m1_cast_ratio(fabs(xb[j]), den);
        code16[j] = (uint8_t)((signbit(xb[j]) ? 8 : 0) | idx);   /* sign bit copies the input's */
    }
    *scale_byte = (uint8_t)sbyte;
}

void nvfp4o_quantize(const uint16_t *x, int64_t R, int64_t C, int64_t ld, int block_axis,
                     const float *global_scale_in, uint8_t *codes, uint8_t *scales,
                     float *global_scale_out)
{
    int64_t rows = block_axis == 0 ? R : C;
    int64_t K = block_axis == 0 ? C : R;
    int64_t nb = K / 16, r;
    float sgf = global_scale_in ? *global_scale_in : nvfp4o_global_scale(x, R, C, ld);
    double sg = (double)sgf;
    init_tables();
    *global_scale_out = sgf;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t b;
        for (b = 0; b < nb; ++b) {
            double xb[16];
            uint8_t c16[16], sbyte;
            int j;
            for (j = 0; j < 16; ++j)
                xb[j] = nvfp4o_bf16_decode(in_elem(x, ld, block_axis, r, b * 16 + j));
            quantize_block(xb, sg, &sbyte, c16);
            scales[r * nb + b] = sbyte;
            for (j = 0; j < 8; ++j)   /* even element in the low nibble */
                codes[r * (K / 2) + b * 8 + j] = (uint8_t)(c16[2 * j] | (c16[2 * j + 1] << 4));
        }
    }
}

/* 2-D block scaling for weights (Sec. 2.2, the training recipe): one E4M3 scale per 16x16
 * tile, from the tile's maximum, so that W and W^T carry the same quantized values.  The
 * tensor format does not change: the scale is written once per row of the tile in
 * scales[R, C/16] and once per column of the tile in scales_t[C, R/16]; codes_t is the
 * transpose of codes (the operand K-contiguous along R).  codes_t / scales_t may be NULL. */
void nvfp4o_quantize_2d(const uint16_t *x, int64_t R, int64_t C, int64_t ld,
                        const float *global_scale_in, uint8_t *codes, uint8_t *scales,
                        uint8_t *codes_t, uint8_t *scales_t, float *global_scale_out)
{
    int64_t tr = R / 16, tc = C / 16, I;
    float sgf = global_scale_in ? *global_scale_in : nvfp4o_global_scale(x, R, C, ld);
    double sg = (double)sgf;
    init_tables();
    *global_scale_out = sgf;
#pragma omp parallel for schedule(static)
    for (I = 0; I < tr; ++I) {
        int64_t J;
        for (J = 0; J < tc; ++J) {
            double bmax = 0.0, den;
            uint8_t c[16][16];
            int i, j, sbyte;
            for (i = 0; i < 16; ++i)
                for (j = 0; j < 16; ++j) {
                    double a = fabs(nvfp4o_bf16_decode(x[(16 * I + i) * ld + 16 * J + j]));
                    if (a > bmax) bmax = a;
                }
            sbyte = nvfp4o_e4m3_cast_ratio(bmax, 6.0 * sg);
            den = nvfp4o_e4m3_decode((unsigned)sbyte) * sg;
            for (i = 0; i < 16; ++i)
                for (j = 0; j < 16; ++j) {
                    double v = nvfp4o_bf16_decode(x[(16 * I + i) * ld + 16 * J + j]);
                    c[i][j] = (uint8_t)((signbit(v) ? 8 : 0) | nvfp4o_e2m1_cast_ratio(fabs(v), den));
                }
            for (i = 0; i < 16; ++i) {
                scales[(16 * I + i) * tc + J] = (uint8_t)sbyte;
                for (j = 0; j < 8; ++j)
                    codes[(16 * I + i) * (C / 2) + 8 * J + j] = (uint8_t)(c[i][2 * j] | (c[i][2 * j + 1] << 4));
            }
            if (codes_t)
                for (j = 0; j < 16; ++j) {
                    scales_t[(16 * J + j) * tr + I] = (uint8_t)sbyte;
                    for (i = 0; i < 8; ++i)
                        codes_t[(16 * J + j) * (R / 2) + 8 * I + i] = (uint8_t)(c[2 * i][j] | (c[2 * i + 1][j] << 4));
                }
        }
    }
}

/* Four-over-Six (Appendix, Eq. 12-13): per block also try the scale that maps
 * the block maximum to 4 and keep the candidate with the lower squared
 * reconstruction error; equal error keeps the 6-based encoding (the paper does
 * not say).  The errors are sums of 16 squares of exactly representable
 * differences; they are compared after fp64 summation in element order. */
void nvfp4o_quantize_4over6(const uint16_t *x, int64_t R, int64_t C, int64_t ld,
                            const float *global_scale_in, uint8_t *codes, uint8_t *scales,
                            float *global_scale_out)
{
    int64_t nb = C / 16, r;
    float sgf = global_scale_in ? *global_scale_in : nvfp4o_global_scale(x, R, C, ld);
    double sg = (double)sgf;
    init_tables();
    *global_scale_out = sgf;
#pragma omp parallel for schedule(static)
    for (r = 0; r < R; ++r) {
        int64_t b;
        for (b = 0; b < nb; ++b) {
            double xb[16], bmax = 0.0, err[2];
            uint8_t c16[2][16];
            int sbyte[2], j, t, pick;
            for (j = 0; j < 16; ++j) {
                xb[j] = nvfp4o_bf16_decode(x[r * ld + b * 16 + j]);
                if (fabs(xb[j]) > bmax) bmax = fabs(xb[j]);
            }
            for (t = 0; t < 2; ++t) {
                double target = t == 0 ? 6.0 : 4.0, sb, den;
                sbyte[t] = nvfp4o_e4m3_cast_ratio(bmax, target * sg);
                sb = nvfp4o_e4m3_decode((unsigned)sbyte[t]);
                den = sb * sg;
                err[t] = 0.0;
                for (j = 0; j < 16; ++j) {
                    int idx = nvfp4o_e2m1_cast_ratio(fabs(xb[j]), den);
                    double d = fabs(xb[j]) - E2M1_MAG[idx] * den;
                    c16[t][j] = (uint8_t)((signbit(xb[j]) ? 8 : 0) | idx);
                    err[t] += d * d;
                }
            }
            pick = err[1] < err[0] ? 1 : 0;
            scales[r * nb + b] = (uint8_t)sbyte[pick];
            for (j = 0; j < 8; ++j)
                codes[r * (C / 2) + b * 8 + j] =
                    (uint8_t)(c16[pick][2 * j] | (c16[pick][2 * j + 1] << 4));
        }
    }
}

/* ---------------------------------------------------------- dequantizer */

/* Eq. 2 evaluated exactly: <= 2 + 4 + 24 significant bits. */
static inline double dequant_elem(const uint8_t *codes, const uint8_t *scales, double sg,
                                  int64_t K, int64_t r, int64_t k)
{
    uint8_t byte = codes[r * (K / 2) + k / 2];
    unsigned code = (k & 1) ? (byte >> 4) : (byte & 15u);
    return nvfp4o_e2m1_decode(code) * nvfp4o_e4m3_decode(scales[r * (K / 16) + k / 16]) * sg;
}

void nvfp4o_dequant_f64(const uint8_t *codes, const uint8_t *scales, float global_scale,
                        int64_t rows, int64_t K, double *out)
{
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t k;
        for (k = 0; k < K; ++k)
            out[r * K + k] = dequant_elem(codes, scales, (double)global_scale, K, r, k);
    }
}

/* KV-cache reconstruction (Sec. 3.2): Eq. 2 exactly, then ONE rounding to bf16. */
void nvfp4o_dequant_bf16(const uint8_t *codes, const uint8_t *scales, float global_scale,
                         int64_t rows, int64_t K, uint16_t *out)
{
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t k;
        for (k = 0; k < K; ++k)
            out[r * K + k] =
                nvfp4o_bf16_rne(dequant_elem(codes, scales, (double)global_scale, K, r, k));
    }
}

/* ------------------------------------------- random Hadamard transform */

/* Random Hadamard transform of a weight-gradient operand (Sec. 2.2: "RHT before quantization
 * on the operands of the weight-gradient GEMM").  X [R, C] is contracted over R (tokens); every
 * group of 16 consecutive rows of a column, v = X[16g .. 16g+15, c], becomes
 *   y = (1/4) H16 diag(s) v,   H16[i][j] = (-1)^popcount(i & j),   s_j = -1 if bit j of
 * sign_mask is set, else +1
 * (the sign vector is the caller's random draw).  (1/4) H16 diag(s) is orthogonal, so applying
 * it to both operands of the GEMM leaves their product unchanged.  The paper gives no
 * arithmetic; the reading: the sums in fp64 (exact for columns whose 16 values span less than
 * 2^40), one rounding to bf16; the result is then quantized along R like any operand. */
void nvfp4o_rht_rows(const uint16_t *x, int64_t R, int64_t C, int64_t ld, unsigned sign_mask,
                     uint16_t *out)
{
    int64_t g;
#pragma omp parallel for schedule(static)
    for (g = 0; g < R / 16; ++g) {
        int64_t c;
        for (c = 0; c < C; ++c) {
            double v[16];
            int i, j;
            for (j = 0; j < 16; ++j) {
                v[j] = nvfp4o_bf16_decode(x[(16 * g + j) * ld + c]);
                if ((sign_mask >> j) & 1u) v[j] = -v[j];
            }
            for (i = 0; i < 16; ++i) {
                double y = 0.0;
                for (j = 0; j < 16; ++j) y += (__builtin_popcount((unsigned)(i & j)) & 1) ? -v[j] : v[j];
                out[(16 * g + i) * C + c] = nvfp4o_bf16_rne(0.25 * y);
            }
        }
    }
}

/* ------------------------------------------------------- K-smoothing (KV) */

/* K-smoothing (Sec. 3.2, Eq. 6): every cached key row (one token, one head) has its mean
 * over the d features removed before it is quantized.  The paper gives the real-number
 * formula only; the reading taken: the row sum is accumulated in fp64 in element order and
 * divided by d in fp64 (both exact for any realistic cache row: d a power of two, 8-bit
 * significands spread over less than 2^40), mean = RN_bf16(that); the smoothed element is
 * RN_bf16(x_j - mean) with the difference taken in fp64 (exact under the same proviso).
 * The means are part of the cache entry: reconstruction adds them back. */
void nvfp4o_kv_smooth(const uint16_t *x, int64_t rows, int64_t d, uint16_t *mean_out,
                      uint16_t *xbar_out)
{
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        double sum = 0.0, mu;
        int64_t j;
        for (j = 0; j < d; ++j) sum += nvfp4o_bf16_decode(x[r * d + j]);
        mean_out[r] = nvfp4o_bf16_rne(sum / (double)d);
        mu = nvfp4o_bf16_decode(mean_out[r]);
        for (j = 0; j < d; ++j)
            xbar_out[r * d + j] = nvfp4o_bf16_rne(nvfp4o_bf16_decode(x[r * d + j]) - mu);
    }
}

/* Reconstruction of a smoothed key cache: RN_bf16(x^_j + mean), x^_j the exact value of
 * Eq. 2 and the sum taken once in fp64. */
void nvfp4o_dequant_bf16_smooth(const uint8_t *codes, const uint8_t *scales, float global_scale,
                                const uint16_t *mean, int64_t rows, int64_t K, uint16_t *out)
{
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        double mu = nvfp4o_bf16_decode(mean[r]);
        int64_t k;
        for (k = 0; k < K; ++k)
            out[r * K + k] = nvfp4o_bf16_rne(
                dequant_elem(codes, scales, (double)global_scale, K, r, k) + mu);
    }
}

/* ----------------------------------------------------------------- GEMM */

/* Y[m,n] = sum_k A^[m,k] W^[n,k] over the dequantized operands, in fp64, and
 * S[m,n] = sum_k |A^[m,k] W^[n,k]| for the per-element error bound.  Only the
 * rows listed in `rows` (or all M when rows == NULL) are computed; output row
 * i corresponds to rows[i].  Plain triple loop, no blocking. */
void nvfp4o_gemm(const uint8_t *codesA, const uint8_t *scalesA, float gsA,
                 const uint8_t *codesW, const uint8_t *scalesW, float gsW,
                 int64_t M, int64_t N, int64_t K, const int64_t *rows, int64_t nrows,
                 double *Y, double *S)
{
    int64_t nr = rows ? nrows : M, i;
    double *Wd = (double *)malloc((size_t)N * (size_t)K * sizeof(double));
    if (!Wd) abort();
    nvfp4o_dequant_f64(codesW, scalesW, gsW, N, K, Wd);
#pragma omp parallel
    {
        double *a = (double *)malloc((size_t)K * sizeof(double));
        if (!a) abort();
#pragma omp for schedule(dynamic, 1)
        for (i = 0; i < nr; ++i) {
            int64_t m = rows ? rows[i] : i, n, k;
            for (k = 0; k < K; ++k) a[k] = dequant_elem(codesA, scalesA, (double)gsA, K, m, k);
            for (n = 0; n < N; ++n) {
                const double *w = Wd + n * K;
                double y = 0.0, s = 0.0;
                for (k = 0; k < K; ++k) {
                    double p = a[k] * w[k];
                    y += p;
                    s += fabs(p);
                }
                Y[i * N + n] = y;
                if (S) S[i * N + n] = s;
            }
        }
        free(a);
    }
    free(Wd);
}

/* ------------------------------------------------------------ activation */

/* ----------------------------------------------------- LoRA side branch */

/* Low-rank adapter beside the quantized weight (Sec. 2.2 "Few-step Distillation in NVFP4":
 * W ~ Dequant(Q(W0)) + (alpha_LoRA / r) B A, adapter weights in bf16; Sec. 3.1: deployed as a
 * separate branch or fused).  Down projection: T[m, j] = RN_bf16(sum_k X[m,k] A[j,k]), the sum
 * in fp64 over the UNQUANTIZED bf16 activations (the adapter branch runs in bf16). */
void nvfp4o_lora_down(const uint16_t *x, const uint16_t *a, int64_t M, int64_t K, int64_t r,
                      uint16_t *t_out)
{
    int64_t m;
#pragma omp parallel for schedule(static)
    for (m = 0; m < M; ++m) {
        int64_t j, k;
        for (j = 0; j < r; ++j) {
            double acc = 0.0;
            for (k = 0; k < K; ++k) acc += nvfp4o_bf16_decode(x[m * K + k]) * nvfp4o_bf16_decode(a[j * K + k]);
            t_out[m * r + j] = nvfp4o_bf16_rne(acc);
        }
    }
}

/* Low-rank update added to a GEMM result: Y[i, n] += scale * sum_j T[m_i, j] B[n, j] and
 * S[i, n] += |scale| * sum_j |T B| (T [M, r], B [N, r] bf16; rows as in nvfp4o_gemm). */
void nvfp4o_lora_up_add(const uint16_t *t, const uint16_t *b, int64_t N, int64_t r, double scale,
                        const int64_t *rows, int64_t nrows, double *Y, double *S)
{
    int64_t i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i, n, j;
        for (n = 0; n < N; ++n) {
            double y = 0.0, sabs = 0.0;
            for (j = 0; j < r; ++j) {
                double p = nvfp4o_bf16_decode(t[m * r + j]) * nvfp4o_bf16_decode(b[n * r + j]);
                y += p;
                sabs += fabs(p);
            }
            Y[i * N + n] += scale * y;
            if (S) S[i * N + n] += fabs(scale) * sabs;
        }
    }
}

/* GELU, tanh form: 0.5 y (1 + tanh( sqrt(2/pi) (y + 0.044715 y^3) )). */
double nvfp4o_gelu_tanh(double y)
{
    const double c = 0.79788456080286535588; /* sqrt(2/pi) */
    return 0.5 * y * (1.0 + tanh(c * (y + 0.044715 * y * y * y)));
}

/* H = RNE_bf16( gelu_tanh( RNE_fp32(y) ) ): the activation input is the FP32
 * value the GEMM hands to its epilogue. */
void nvfp4o_gelu_tanh_bf16(const double *y, int64_t n, uint16_t *h)
{
    int64_t i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < n; ++i) h[i] = nvfp4o_bf16_rne(nvfp4o_gelu_tanh((double)(float)y[i]));
}

int nvfp4o_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
