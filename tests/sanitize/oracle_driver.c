/* Exercises every function of the CPU oracle on small exact-size heap buffers; built with
 * -fsanitize=address,undefined by tests/test_sanitizers.py, so any out-of-bounds access or
 * undefined operation inside the oracle aborts the run.  Inputs come from a fixed LCG and
 * include zeros, negative zero, huge and tiny magnitudes.  Prints "ok" on success. */
#include "../../oracle/nvfp4_oracle.h"

#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static uint32_t state = 12345u;
static uint32_t lcg(void) { state = state * 1664525u + 1013904223u; return state >> 8; }

/* a finite bf16 pattern: random sign and mantissa, exponent in a band around 1.0 (or anywhere) */
static uint16_t rand_bf16(int wide)
{
    uint32_t r = lcg();
    uint32_t e = wide ? 1u + r % 253u : 120u + r % 14u;
    if (r % 37u == 0) return (uint16_t)((r & 1u) << 15);          /* +0 / -0 */
    return (uint16_t)(((r >> 3 & 1u) << 15) | (e << 7) | (r >> 5 & 0x7Fu));
}

static void *xmalloc(size_t n) { void *p = malloc(n ? n : 1); if (!p) abort(); return p; }

static void run(int64_t R, int64_t C, int wide)
{
    int64_t ld = C, i;
    uint16_t *x = xmalloc((size_t)(R * ld) * 2);
    for (i = 0; i < R * ld; ++i) x[i] = rand_bf16(wide);
    for (int axis = 0; axis < 2; ++axis) {
        int64_t rows = axis == 0 ? R : C, K = axis == 0 ? C : R;
        uint8_t *codes = xmalloc((size_t)(rows * K / 2)), *scales = xmalloc((size_t)(rows * K / 16));
        double *d64 = xmalloc((size_t)(rows * K) * 8);
        uint16_t *d16 = xmalloc((size_t)(rows * K) * 2);
        float gs = 0.0f, gs_given = 0.0123f;
        nvfp4o_quantize(x, R, C, ld, axis, NULL, codes, scales, &gs);
        nvfp4o_dequant_f64(codes, scales, gs, rows, K, d64);
        nvfp4o_dequant_bf16(codes, scales, gs, rows, K, d16);
        nvfp4o_quantize(x, R, C, ld, axis, &gs_given, codes, scales, &gs);
        if (gs != gs_given) abort();
        free(codes); free(scales); free(d64); free(d16);
    }
    {   /* scale search, 2-D tiles, Hadamard transform, K-smoothing */
        uint8_t *codes = xmalloc((size_t)(R * C / 2)), *scales = xmalloc((size_t)(R * C / 16));
        uint8_t *codes_t = xmalloc((size_t)(R * C / 2)), *scales_t = xmalloc((size_t)(R * C / 16));
        uint16_t *y = xmalloc((size_t)(R * C) * 2), *mean = xmalloc((size_t)R * 2), *back = xmalloc((size_t)(R * C) * 2);
        float gs;
        nvfp4o_quantize_4over6(x, R, C, ld, NULL, codes, scales, &gs);
        nvfp4o_quantize_2d(x, R, C, ld, NULL, codes, scales, codes_t, scales_t, &gs);
        nvfp4o_quantize_2d(x, R, C, ld, NULL, codes, scales, NULL, NULL, &gs);
        nvfp4o_rht_rows(x, R, C, ld, 0xA53Cu, y);
        nvfp4o_kv_smooth(x, R, C, mean, y);
        nvfp4o_quantize_4over6(y, R, C, C, NULL, codes, scales, &gs);
        nvfp4o_dequant_bf16_smooth(codes, scales, gs, mean, R, C, back);
        free(codes); free(scales); free(codes_t); free(scales_t); free(y); free(mean); free(back);
    }
    free(x);
}

static void run_gemm(int64_t M, int64_t N, int64_t K)
{
    uint16_t *a = xmalloc((size_t)(M * K) * 2), *w = xmalloc((size_t)(N * K) * 2);
    uint8_t *ca = xmalloc((size_t)(M * K / 2)), *sa = xmalloc((size_t)(M * K / 16));
    uint8_t *cw = xmalloc((size_t)(N * K / 2)), *sw = xmalloc((size_t)(N * K / 16));
    double *Y = xmalloc((size_t)(M * N) * 8), *S = xmalloc((size_t)(M * N) * 8);
    int64_t rows[3] = {M - 1, 0, M / 2}, i;
    float ga, gw;
    for (i = 0; i < M * K; ++i) a[i] = rand_bf16(0);
    for (i = 0; i < N * K; ++i) w[i] = rand_bf16(0);
    nvfp4o_quantize(a, M, K, K, 0, NULL, ca, sa, &ga);
    nvfp4o_quantize(w, N, K, K, 0, NULL, cw, sw, &gw);
    nvfp4o_gemm(ca, sa, ga, cw, sw, gw, M, N, K, NULL, 0, Y, S);
    nvfp4o_gemm(ca, sa, ga, cw, sw, gw, M, N, K, rows, 3, Y, NULL);
    {   /* activation + LoRA branch (rank r = 16 here) */
        int64_t r = 16;
        uint16_t *h = xmalloc((size_t)(M * N) * 2), *la = xmalloc((size_t)(r * K) * 2), *t = xmalloc((size_t)(M * r) * 2);
        uint16_t *lb = xmalloc((size_t)(N * r) * 2);
        for (i = 0; i < r * K; ++i) la[i] = rand_bf16(0);
        for (i = 0; i < N * r; ++i) lb[i] = rand_bf16(0);
        nvfp4o_gelu_tanh_bf16(Y, 3 * N, h);
        nvfp4o_lora_down(a, la, M, K, r, t);
        nvfp4o_gemm(ca, sa, ga, cw, sw, gw, M, N, K, NULL, 0, Y, S);
        nvfp4o_lora_up_add(t, lb, N, r, 0.5, NULL, M, Y, S);
        nvfp4o_lora_up_add(t, lb, N, r, 0.5, rows, 3, Y, S);
        free(h); free(la); free(t); free(lb);
    }
    free(a); free(w); free(ca); free(sa); free(cw); free(sw); free(Y); free(S);
}

int main(void)
{
    unsigned c;
    for (c = 0; c < 256; ++c) (void)nvfp4o_e4m3_decode(c);
    for (c = 0; c < 16; ++c) (void)nvfp4o_e2m1_decode(c);
    for (c = 0; c < 0x7F80u; c += 61u)
        if (nvfp4o_bf16_rne(nvfp4o_bf16_decode((uint16_t)c)) != c) abort();
    (void)nvfp4o_bf16_rne(1e300); (void)nvfp4o_bf16_rne(-1e-300); (void)nvfp4o_bf16_rne(0.0);
    (void)nvfp4o_gelu_tanh(-40.0); (void)nvfp4o_gelu_tanh(40.0);
    run(16, 16, 0);
    run(48, 32, 0);
    run(32, 80, 1);          /* the whole exponent range: saturating and underflowing scales */
    run(16, 128, 1);
    run_gemm(5, 7, 16);
    run_gemm(33, 9, 48);
    printf("ok %d threads\n", nvfp4o_num_threads());
    return 0;
}
