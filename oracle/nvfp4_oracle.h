/*
 * NVFP4 CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 * Interface of nvfp4_oracle.c; all pointers are HOST pointers owned by the
 * caller.  bf16 tensors travel as uint16_t bit patterns.  Only tests, the
 * smoke check and the bench's cpu_baseline leg may link or load this.
 */
#ifndef NVFP4_ORACLE_H
#define NVFP4_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* formats (Sec. 2.2; Appendix on scale search, first paragraph) */
double   nvfp4o_e2m1_decode(unsigned code);   /* 4-bit code, bit 3 = sign */
double   nvfp4o_e4m3_decode(unsigned byte);   /* 0x7F / 0xFF -> NaN */
double   nvfp4o_bf16_decode(uint16_t h);
uint16_t nvfp4o_bf16_rne(double v);

/* nearest format value to the real num/den (num, den >= 0), ties to even, saturating */
int nvfp4o_e4m3_cast_ratio(double num, double den);   /* -> byte 0x00..0x7E */
int nvfp4o_e2m1_cast_ratio(double num, double den);   /* -> magnitude index 0..7 */

/* alpha^FP32 = amax / (448*6) as FP32 (1.0 if the tensor is all zero) */
float nvfp4o_global_scale(const uint16_t *x, int64_t R, int64_t C, int64_t ld);

/* X bf16 [R, C] with row stride ld.  block_axis 0: blocks of 16 along C,
 * output rows = R, K = C.  block_axis 1: blocks along R, output rows = C,
 * K = R (the operand is quantized along the other axis and comes out
 * K-contiguous).  codes [rows, K/2] (even element in the low nibble), scales
 * [rows, K/16].  global_scale_in == NULL: derive from amax. */
void nvfp4o_quantize(const uint16_t *x, int64_t R, int64_t C, int64_t ld, int block_axis,
                     const float *global_scale_in, uint8_t *codes, uint8_t *scales,
                     float *global_scale_out);

/* 2-D block scaling for weights (Sec. 2.2 training recipe): one scale per 16x16 tile; the
 * [R, C] operand (blocks along C) and, if asked for, the [C, R] operand (blocks along R). */
void nvfp4o_quantize_2d(const uint16_t *x, int64_t R, int64_t C, int64_t ld,
                        const float *global_scale_in, uint8_t *codes, uint8_t *scales,
                        uint8_t *codes_t, uint8_t *scales_t, float *global_scale_out);

/* Four-over-Six scale search (Appendix, Eq. 12-13); blocks along C only. */
void nvfp4o_quantize_4over6(const uint16_t *x, int64_t R, int64_t C, int64_t ld,
                            const float *global_scale_in, uint8_t *codes, uint8_t *scales,
                            float *global_scale_out);

void nvfp4o_dequant_f64(const uint8_t *codes, const uint8_t *scales, float global_scale,
                        int64_t rows, int64_t K, double *out);
void nvfp4o_dequant_bf16(const uint8_t *codes, const uint8_t *scales, float global_scale,
                         int64_t rows, int64_t K, uint16_t *out);

/* Random Hadamard transform along the rows (groups of 16) of a weight-gradient operand
 * (Sec. 2.2): out [R, C] bf16 = RN_bf16((1/4) H16 diag(s) x) per group and column. */
void nvfp4o_rht_rows(const uint16_t *x, int64_t R, int64_t C, int64_t ld, unsigned sign_mask,
                     uint16_t *out);

/* LoRA side branch (Sec. 2.2 / 3.1): T = RN_bf16(X A^T) on bf16 activations, and the update
 * Y += scale * T B^T added to a GEMM result (S += the matching sum of absolute terms). */
void nvfp4o_lora_down(const uint16_t *x, const uint16_t *a, int64_t M, int64_t K, int64_t r,
                      uint16_t *t_out);
void nvfp4o_lora_up_add(const uint16_t *t, const uint16_t *b, int64_t N, int64_t r, double scale,
                        const int64_t *rows, int64_t nrows, double *Y, double *S);

/* K-smoothing of the key cache (Sec. 3.2, Eq. 6): x bf16 [rows, d] -> per-row mean (bf16) and
 * the smoothed rows RN_bf16(x - mean) (bf16), which are then quantized like any tensor;
 * reconstruction RN_bf16(x^ + mean). */
void nvfp4o_kv_smooth(const uint16_t *x, int64_t rows, int64_t d, uint16_t *mean_out,
                      uint16_t *xbar_out);
void nvfp4o_dequant_bf16_smooth(const uint8_t *codes, const uint8_t *scales, float global_scale,
                                const uint16_t *mean, int64_t rows, int64_t K, uint16_t *out);

/* Y[i,n] = sum_k A^[rows[i],k] W^[n,k]; S = same with absolute values (may be NULL).
 * rows == NULL: all M rows. */
void nvfp4o_gemm(const uint8_t *codesA, const uint8_t *scalesA, float gsA,
                 const uint8_t *codesW, const uint8_t *scalesW, float gsW,
                 int64_t M, int64_t N, int64_t K, const int64_t *rows, int64_t nrows,
                 double *Y, double *S);

double nvfp4o_gelu_tanh(double y);
void   nvfp4o_gelu_tanh_bf16(const double *y, int64_t n, uint16_t *h);

int nvfp4o_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
