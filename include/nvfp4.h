/*
 * nvfp4.h -- C ABI of the MI355X (gfx950) NVFP4 hot-path library.
 *
 * The library implements the W4A4 NVFP4 linear-layer path of the paper:
 * the quantizer of Sec. 2.2 ("NVFP4 Preliminaries", Eq. 2 and the scale
 * definitions that follow it; Appendix "Scale Search NVFP4 Quantization",
 * Eq. 12), the block-scaled FP4 GEMM used for forward, input-gradient and
 * weight-gradient products (Sec. 2.2 "Multi-Shot AR NVFP4 Training",
 * Sec. 3.1, Appendix "Implementation Details"), the NVFP4 KV cache of
 * Sec. 3.2 (Eq. 5), and a fused activation + re-quantize GEMM epilogue.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or reads results back; scratch memory comes in
 *     through the workspace argument (size from nvfp4_workspace_bytes()).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Every call only enqueues work on that stream and returns.
 *   - An nvfp4_tensor is a HOST struct holding device pointers.
 *   - Return value: NVFP4_OK or a negative nvfp4_status.  Arguments are
 *     validated on the host before anything is launched; a call that returns
 *     an error has launched nothing.  Non-finite inputs are outside the
 *     contract.
 *   - Stream capture: an entry point only enqueues kernels (no memset or copy
 *     nodes, no synchronisation), so it may be called while `stream` is being
 *     captured into a HIP graph, provided the same entry point has run once
 *     before on this device with arguments of the same kind (the first launch
 *     of a kernel variant raises its dynamic LDS limit, which is not a stream
 *     operation), and launch timing is off.
 *
 * NVFP4 tensor format (Eq. 2):  x^ = code * block_scale * global_scale
 *   codes   [rows, K/2]  two E2M1 codes per byte; element 2j in bits 3:0 and
 *                        element 2j+1 in bits 7:4; a code is s|e1 e0|m with the
 *                        magnitudes {0, .5, 1, 1.5, 2, 3, 4, 6} at indices 0..7
 *   scales  [rows, K/16] one E4M3 byte (1-4-3, bias 7, max 448) per 16
 *                        consecutive elements along K, plain row-major
 *   global_scale [1]     FP32, one per tensor
 * Rounding: global_scale = RN_fp32(amax / (448*6)) (1.0 for an all-zero
 * tensor); block scale = E4M3 nearest to blockmax / (6*global_scale); code =
 * E2M1 nearest to x / (block_scale*global_scale); all three decided in exact
 * arithmetic, ties to the even mantissa, saturating at the format maximum.
 * The sign bit of a code copies the sign bit of the input.
 */
#ifndef NVFP4_H
#define NVFP4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum nvfp4_status {
    NVFP4_OK = 0,
    NVFP4_ERR_NULL = -1,       /* a required pointer is NULL */
    NVFP4_ERR_SHAPE = -2,      /* non-positive size, K not a multiple of 16, K mismatch, bad enum */
    NVFP4_ERR_ALIGN = -3,      /* pointer not 16-byte aligned, or a row stride that does not keep rows 16-byte aligned */
    NVFP4_ERR_WORKSPACE = -4,  /* workspace NULL or smaller than nvfp4_workspace_bytes() */
    NVFP4_ERR_LAUNCH = -5      /* the HIP runtime refused a launch */
} nvfp4_status;

typedef struct nvfp4_tensor {
    uint8_t *codes;        /* device, [rows, K/2], 16-byte aligned */
    uint8_t *scales;       /* device, [rows, K/16], 16-byte aligned */
    float   *global_scale; /* device, [1] */
    int64_t  rows;
    int64_t  K;            /* multiple of 16 */
} nvfp4_tensor;

enum { NVFP4_OUT_F32 = 0, NVFP4_OUT_BF16 = 1 };
enum { NVFP4_ACT_NONE = 0, NVFP4_ACT_GELU_TANH = 1 };
enum { NVFP4_OP_QUANTIZE = 0, NVFP4_OP_KV_QUANT = 1, NVFP4_OP_GEMM_ACT_QUANT = 2, NVFP4_OP_GEMM = 3,
       NVFP4_OP_KV_DEQUANT = 4,
       NVFP4_OP_GEMM_ACT_QUANT_GEMM = 5 /* timing only: the GEMM kernel inside nvfp4_gemm_act_quant */,
       NVFP4_OP_QUANTIZE_4OVER6 = 6, NVFP4_OP_KV_QUANT_4OVER6 = 7, NVFP4_OP_KV_QUANT_K = 8,
       NVFP4_OP_KV_DEQUANT_GATHER = 9, NVFP4_OP_QUANTIZE_2D = 10,
       NVFP4_OP_QUANTIZE_RHT = 11, NVFP4_OP_QUANTIZE_A2A = 12,
       NVFP4_OP_LORA_DOWN = 13, NVFP4_OP_GEMM_LORA = 14,
       NVFP4_OP_PROBE = 15 /* timing only: nvfp4_probe */, NVFP4_OP_GEMM_SCALE_OUT = 16 };

/*
 * Quantizer (Sec. 2.2, Eq. 2; Eq. 12 with target magnitude 6).
 * x_bf16: device, bf16 [R, C], row stride ld elements (ld >= C, ld % 8 == 0).
 * block_axis 0: blocks of 16 run along C; out has rows = R, K = C.
 * block_axis 1: blocks run along R; out has rows = C, K = R (the operand
 *               re-quantized along its other axis, emitted K-contiguous, as
 *               the backward GEMMs need it).
 * global_scale_in: device pointer to one float, or NULL.  NULL: the scale is
 *               derived from the tensor's amax: contiguous row-block tensors of up
 *               to ~120 MB are held on the chip between the two steps (one launch,
 *               one pass over x; the launch occupies every compute unit while it
 *               runs), larger or strided ones take one extra pass over x.  A
 *               tensor that is needed along both axes (every training operand
 *               is) has one amax: pass the first call's out->global_scale to
 *               the second call and its extra pass is saved.
 * out: rows/K must already describe the result; codes/scales/global_scale are
 *      written (global_scale receives the scale that was used).
 * workspace: nvfp4_workspace_bytes(NVFP4_OP_QUANTIZE, R, C, 0) bytes; contents
 *      need no initialisation and are garbage afterwards.
 */
int nvfp4_quantize(const void *x_bf16, int64_t R, int64_t C, int64_t ld, int block_axis,
                   const float *global_scale_in, nvfp4_tensor *out,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Quantizer with the Four-over-Six scale search (Sec. 2.2 "Multi-Shot AR NVFP4
 * Training"; Appendix "Scale Search NVFP4 Quantization", Eq. 12-13): every
 * block is encoded twice, with its maximum mapped to 6 and to 4 (block scale =
 * E4M3 nearest to blockmax / (M * global_scale) for M = 6 and M = 4), and the
 * encoding with the smaller squared reconstruction error sum_j (x_j - x^_j)^2
 * is kept; equal errors keep M = 6.  The errors are those of the fp64
 * evaluation "difference, square, sum in element order, each step rounded".
 * Arguments, layout, workspace and global scale as nvfp4_quantize with
 * block_axis 0 (workspace size: NVFP4_OP_QUANTIZE_4OVER6).
 */
int nvfp4_quantize_4over6(const void *x_bf16, int64_t R, int64_t C, int64_t ld,
                          const float *global_scale_in, nvfp4_tensor *out,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Quantizer for the two operands of dW = dY^T X with a random Hadamard transform
 * applied first (the outlier-spreading step of the training recipe in Sec. 2.2
 * "Multi-Shot AR NVFP4 Training").  x_bf16
 * [R, C] is contracted over R (tokens).  Every group of 16 consecutive rows of a
 * column, v = x[16g .. 16g+15, c], is replaced by
 *   y = RN_bf16( (1/4) H16 diag(s) v ),  H16[i][j] = (-1)^popcount(i & j),
 *   s_j = -1 where bit j of sign_mask is set, +1 otherwise
 * (exact sums: on the matrix pipes in fp32 where the group's magnitudes lie close
 * enough together for that to be exact, in fp64 otherwise, which is exact for
 * groups whose values span less than 2^40), and y is
 * quantized along R exactly as nvfp4_quantize(block_axis = 1) would: out has
 * rows = C, K = R, the tensor scale comes from the amax of y.  The transform
 * is orthogonal: applied with the SAME sign_mask to both operands (dY and X) it
 * leaves the product dY^T X unchanged while spreading outliers over 16 tokens.
 * sign_mask: the caller's random draw, low 16 bits.  R % 16 == 0, C % 8 == 0.
 * workspace: nvfp4_workspace_bytes(NVFP4_OP_QUANTIZE_RHT, R, C, 0); the part beyond
 * nvfp4_workspace_bytes(NVFP4_OP_QUANTIZE, R, C, 0) carries, from the amax pass to
 * the encoding pass, which groups need the slower forms -- a workspace of only
 * that smaller size is accepted, and the encoding pass then finds them again.
 */
int nvfp4_quantize_rht(const void *x_bf16, int64_t R, int64_t C, int64_t ld, uint32_t sign_mask,
                       const float *global_scale_in, nvfp4_tensor *out,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Weight quantizer with square scaling tiles (the weight half of the training
 * recipe in Sec. 2.2 "Multi-Shot AR NVFP4 Training"; activations and gradients
 * keep the 16-element row blocks of nvfp4_quantize):
 * one E4M3 scale per 16 x 16 tile, from the tile's maximum, so that the forward
 * operand W [R, C] (blocks along C) and the backward operand W^T [C, R] (blocks
 * along R) contain the same quantized values.  The tensor format is unchanged:
 * the tile's scale byte is repeated on its 16 rows in out->scales and on its 16
 * columns in out_t->scales; out_t->codes is the transpose of out->codes.
 * R % 16 == 0, C % 16 == 0.  out: rows = R, K = C.  out_t: NULL, or rows = C,
 * K = R; both receive the same global scale.  global_scale_in and workspace as
 * nvfp4_quantize (workspace size: NVFP4_OP_QUANTIZE_2D).
 */
int nvfp4_quantize_2d(const void *w_bf16, int64_t R, int64_t C, int64_t ld,
                      const float *global_scale_in, nvfp4_tensor *out, nvfp4_tensor *out_t,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Block-scaled FP4 GEMM, FP32 accumulation (Sec. 2.2 / 3.1; Appendix
 * "Implementation Details": forward, backward and weight-gradient GEMM
 * operands are all NVFP4):
 *   Y[m,n] = gsA*gsW * sum_b sA[m,b] sW[n,b] * sum_{j in b} cA[m,j] cW[n,j]
 * A: [M, K], W: [N, K], both K-contiguous ("NT").  Y: device [M, N], row
 * stride ldy elements (ldy >= N and a multiple of 4; a multiple of 8 for bf16
 * output on the tiled kernels, so that every row starts on a 16-byte boundary:
 * NVFP4_ERR_ALIGN otherwise), fp32 (NVFP4_OUT_F32) or bf16
 * (NVFP4_OUT_BF16, the fp32 result rounded to nearest even).  dgrad and wgrad are this same call on
 * operands produced by nvfp4_quantize with the matching block_axis.
 * K % 64 == 0 and N % 8 == 0 run on the tiled MFMA kernels at any M and N
 * (operands of 2 GiB and more are cut into row chunks, one set of launches per
 * chunk); other shapes (K % 16 == 0) run on a plain, much slower kernel.
 */
int nvfp4_gemm(const nvfp4_tensor *A, const nvfp4_tensor *W, void *Y, int64_t ldy,
               int out_dtype, void *stream);

/*
 * LoRA side branch next to the quantized weight (Sec. 2.2 "Few-step Distillation
 * in NVFP4": W ~ Dequant(Q(W0)) + (alpha_LoRA / r) B A with bf16 adapters of rank
 * r = 128; Sec. 3.1: run as a separate branch or with fused low-rank kernels).
 *
 * nvfp4_lora_down: T = RN_bf16(X A^T), fp32 accumulation.  x_bf16 [M, K] bf16 (row
 *   stride ldx, the UNQUANTIZED activations), a_bf16 [NVFP4_LORA_RANK, K] bf16,
 *   t_bf16 [M, NVFP4_LORA_RANK] bf16 out.  K % 16 == 0, ldx % 8 == 0.  The K
 *   range is cut across workgroups; workspace (16-byte aligned,
 *   nvfp4_workspace_bytes(NVFP4_OP_LORA_DOWN, M, K, 0) bytes) holds their fp32
 *   partial sums, which are added in a fixed order: results are deterministic.
 * nvfp4_gemm_lora: Y = nvfp4_gemm(A, W) + lora_scale * T B^T in one kernel: the
 *   low-rank product (b_bf16 [N, NVFP4_LORA_RANK] bf16) is accumulated on the
 *   matrix cores into the accumulators of the FP4 product, in fp32.  Y, ldy,
 *   out_dtype as nvfp4_gemm; lora_scale = alpha_LoRA / r.  Needs K % 64 == 0
 *   and N % 8 == 0 (NVFP4_ERR_SHAPE otherwise).
 */
#define NVFP4_LORA_RANK 128
int nvfp4_lora_down(const void *x_bf16, int64_t M, int64_t K, int64_t ldx, const void *a_bf16,
                    void *t_bf16, void *workspace, size_t workspace_bytes, void *stream);
int nvfp4_gemm_lora(const nvfp4_tensor *A, const nvfp4_tensor *W, const void *t_bf16,
                    const void *b_bf16, float lora_scale, void *Y, int64_t ldy, int out_dtype,
                    void *stream);

/*
 * nvfp4_gemm with bf16 output that also returns the NVFP4 tensor scale of its output,
 * y_global_scale_out = RN_fp32(max|Y| / 2688) (Sec. 2.2, Eq. 2; 1.0 for an all-zero Y), one float in
 * device memory.  The quantizer needs a tensor's largest magnitude before it can write the first
 * code; for tensors too large to stay on the chip that is a pass over the tensor of its own.  A
 * tensor produced by a GEMM (an activation, a gradient) gets the maximum from the GEMM's epilogue
 * instead -- one maximum per workgroup, reduced by a small second launch -- so that the calls that
 * quantize Y afterwards (either axis, with the scale search or the Hadamard transform) take the
 * scale as given and read Y once each.
 * Y: [M, ldy] bf16, 16-byte aligned, ldy >= N a multiple of 8.
 * workspace: nvfp4_workspace_bytes(NVFP4_OP_GEMM_SCALE_OUT, M, N, 0) bytes, 16-byte aligned.
 */
int nvfp4_gemm_scale_out(const nvfp4_tensor *A, const nvfp4_tensor *W, void *Y_bf16, int64_t ldy,
                         float *y_global_scale_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * GEMM with fused activation and re-quantization of the result along N
 * (the "fused" W4A4 kernels of Sec. 3.1): H = bf16(act(A W^T)), out =
 * quantize(H).  The result is byte-identical to nvfp4_gemm(BF16) followed by
 * the activation in fp32, rounding to bf16, and nvfp4_quantize.
 * global_scale_in != NULL: single pass, H is never written unless h_bf16_opt
 *   is given.  NULL: H's amax is only known when the GEMM ends, so H is staged
 *   in the workspace (or h_bf16_opt) and packed by a second light kernel.
 * out: rows = M, K = N (N % 16 == 0).  h_bf16_opt: NULL or device bf16 [M, N].
 * workspace: nvfp4_workspace_bytes(NVFP4_OP_GEMM_ACT_QUANT, M, N, flags) with flags
 *   bit 0 set when h_bf16_opt is given and bit 1 set when global_scale_in is
 *   given (bit 1 assumes K % 64 == 0; other K fall back to staging H, leave it
 *   clear for them).
 */
int nvfp4_gemm_act_quant(const nvfp4_tensor *A, const nvfp4_tensor *W, int act,
                         const float *global_scale_in, nvfp4_tensor *out, void *h_bf16_opt,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * KV-cache quantization (Sec. 3.2, Eq. 5): a chunk [T, H, d] (contiguous bf16)
 * is viewed as [(T*H), d] and quantized with 16-element blocks along d and one
 * global scale per call.  out: rows = T*H, K = d.
 * workspace: nvfp4_workspace_bytes(NVFP4_OP_KV_QUANT, T, H, d).
 */
int nvfp4_kv_quant(const void *kv_bf16, int64_t T, int64_t H, int64_t d, nvfp4_tensor *out,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * nvfp4_kv_quant for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments and the same bytes as nvfp4_kv_quant, minus the workspace: the
 * partial maxima live in a fixed array inside the library's device image (4 KB on every GPU
 * the library runs on, held until the process ends; its address is looked up on the first
 * call on a device).  Windows for which the one-launch kernel is taken (see nvfp4_set_one_launch) need
 * no partial maxima and leave the array alone; the others take the two passes that use it.  The call allocates nothing, frees nothing and calls no allocating
 * routine; launch timing does not record it.
 * Limit: T * H * d <= NVFP4_NOALLOC_MAX_ELEMENTS, NVFP4_ERR_SHAPE beyond it.
 * All calls on one GPU share that array, and it keeps the last call's contents (every slot a
 * call reads it has written before, so nothing needs clearing): calls that overlap on one GPU
 * (different streams, or several host threads' work in flight together) race on it and
 * must be ordered by the caller.
 */
#define NVFP4_NOALLOC_MAX_ELEMENTS ((int64_t)1 << 32)
int nvfp4_kv_quant_noalloc(const void *kv_bf16, int64_t T, int64_t H, int64_t d, nvfp4_tensor *out,
                           void *stream);

/*
 * KV-cache quantization with the Four-over-Six scale search, the variant the
 * paper applies to the cache (Sec. 3.2; Appendix, Eq. 12-13).  Arguments as
 * nvfp4_kv_quant (workspace size: NVFP4_OP_KV_QUANT_4OVER6); the result is read
 * back by nvfp4_kv_dequant like any other NVFP4 tensor.
 */
int nvfp4_kv_quant_4over6(const void *kv_bf16, int64_t T, int64_t H, int64_t d, nvfp4_tensor *out,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Key-cache quantization as the paper applies it to keys (Sec. 3.2, Eq. 6, then
 * the scale search of Appendix Eq. 12-13): every row [t, h, :] first has its
 * mean over the d features removed,
 *   mean[t,h] = RN_bf16( (sum_u K[t,h,u]) / d ),  Kbar[t,h,u] = RN_bf16( K[t,h,u] - mean[t,h] )
 * (sum, quotient and difference in fp64: exact for rows whose values span less
 * than 2^40), and Kbar is quantized like nvfp4_kv_quant_4over6, its tensor scale
 * taken from the amax of Kbar.  The means belong to the cache entry.
 * row_mean_bf16_out: device, bf16 [T*H].  d / 16 must be a power of two <= 64.
 * workspace: nvfp4_workspace_bytes(NVFP4_OP_KV_QUANT_K, T, H, d).
 */
int nvfp4_kv_quant_k(const void *k_bf16, int64_t T, int64_t H, int64_t d, nvfp4_tensor *out,
                     void *row_mean_bf16_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Gathered KV-cache reconstruction (Sec. 3.2: with sink tokens and a sliding
 * window an attention step reads several cached chunks).  `chunks` is a HOST
 * array of n_chunks (1..NVFP4_KV_MAX_CHUNKS) descriptors of device data; chunk c
 * holds T tokens (q.rows == T*H, q.K == d) and, for keys stored with
 * nvfp4_kv_quant_k, its row means (NULL otherwise).  kv_bf16_out [sum_c T_c, H, d]
 * receives the chunks back to back from one launch:
 *   out = RN_bf16(code * block_scale * global_scale [+ row mean]), rounded once.
 */
#define NVFP4_KV_MAX_CHUNKS 64
typedef struct nvfp4_kv_chunk {
    nvfp4_tensor q;
    const void *row_mean_bf16;   /* device bf16 [T*H], or NULL */
    int64_t T;
} nvfp4_kv_chunk;
int nvfp4_kv_dequant_gather(const nvfp4_kv_chunk *chunks, int n_chunks, void *kv_bf16_out,
                            int64_t H, int64_t d, void *stream);

/*
 * Packer for the NVFP4 pre-attention all-to-all of sequence-parallel inference
 * (Appendix "Sequence Parallelism Inference", Eq. 11): the local Q (or K, V)
 * [T = L/P, H, d] is cast to NVFP4 along d and laid out as P slabs, one per
 * destination device, slab p holding heads p*H/P .. (p+1)*H/P - 1 of every
 * local token:
 *   out row (p * T + t) * (H/P) + h'  <-  x[t, p*H/P + h', :]
 * so that each slab (T*(H/P) rows of codes, of scales) is one contiguous
 * send buffer at ~4.5 bit per element; all slabs share the call's global
 * scale.  The exchange itself is not part of this library.  H % P == 0;
 * out: rows = T*H, K = d.  global_scale_in and workspace as nvfp4_quantize
 * (workspace size: NVFP4_OP_QUANTIZE_A2A).
 */
int nvfp4_quantize_for_all_to_all(const void *x_bf16, int64_t T, int64_t H, int64_t d, int64_t P,
                                  const float *global_scale_in, nvfp4_tensor *out,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * KV-cache reconstruction (Sec. 3.2): kv_bf16_out[t,h,:] = RN_bf16(code *
 * block_scale * global_scale), the product taken exactly and rounded once.
 */
int nvfp4_kv_dequant(const nvfp4_tensor *in, void *kv_bf16_out, int64_t T, int64_t H, int64_t d,
                     void *stream);

/* Workspace size in bytes for `op` (NVFP4_OP_*) at the given sizes; 0 on a bad op. */
size_t nvfp4_workspace_bytes(int op, int64_t a, int64_t b, int64_t c);

/* The kernel launches nvfp4_gemm (and the GEMM inside nvfp4_gemm_act_quant) issues
 * for an [M, K] x [N, K] problem, as text: one "BMxBN:workgroups" item per launch in
 * launch order, separated by spaces (tile shape and number of workgroups; "generic"
 * for shapes only the fallback kernel for odd shapes takes: about a third of the tiled rate).  The plan is this library's own
 * (a small cost model over its tile shapes and the 256 compute units): whole waves, or
 * whole tile rows, of large tiles, then the leftover rectangles on tiles that suit them.
 * Host pointers; nothing is launched.
 * Returns the number of launches, NVFP4_ERR_WORKSPACE if text_bytes is too small. */
int nvfp4_gemm_plan(int64_t M, int64_t N, int64_t K, char *text, size_t text_bytes);

/* Static, human-readable text for a status code. */
const char *nvfp4_status_string(int status);

/* Launch durations, for benchmarks.  While timing is enabled every entry point
 * records a pair of HIP events around its kernels on the caller's stream
 * (enabling also discards earlier records; at most 8192 calls are recorded).
 * nvfp4_timing_read() waits for the recorded events of entry point `op`
 * (NVFP4_OP_*) and returns how many calls were recorded and the sum of their
 * durations in milliseconds.  Host pointers.  An event pair costs a few
 * microseconds of idle stream per call; nvfp4_set_timing_ops() restricts the
 * recording to the entry points whose bit (1u << NVFP4_OP_*) is set in op_mask
 * (nvfp4_set_timing(1) = all, 0 = none). */
void nvfp4_set_timing(int enabled);
void nvfp4_set_timing_ops(uint32_t op_mask);
int  nvfp4_timing_read(int op, int *calls, float *total_ms);

/* The one-launch quantizers (tensors that fit on the chip) make the tensor maximum known to all
 * workgroups through a grid-wide wait that is bounded: a workgroup that has waited longer than this
 * many 10 ns ticks stops waiting and derives the maximum from the tensor itself (slow, same result).
 * Default 200000 (2 ms); 0 makes every workgroup give up at once, which is how the tests exercise
 * that path; 0xFFFFFFFF restores the default.  Applies to calls made afterwards.
 * The exchange runs through 64 slots of library-owned device memory taken in turn, and tells one
 * launch from the next by an epoch counted on the device, so a call captured into a HIP graph can
 * be replayed; more than 64 such launches in flight at once on one GPU, or one graph replayed
 * concurrently with itself, would race. */
void nvfp4_set_sync_spin_limit(uint32_t ticks_10ns);

/* Which form the row quantizers (nvfp4_quantize with block_axis 0, the scale search, nvfp4_kv_quant*,
 * nvfp4_quantize_for_all_to_all; no scale given) take for a tensor that fits on the chip.  The one-launch form
 * fetches the tensor from HBM once, the two-pass form twice; in time they are within a few per cent of each
 * other for the plain rule on large tensors, and the two passes are faster for middle sizes and for the scale
 * search and the smoothed keys.  AUTO (the default) goes by what was measured: one launch for the plain rule below
 * 0.4 M blocks of 16 and from 2.5 M blocks on, two passes otherwise; ALWAYS takes the one-launch form whenever
 * the tensor fits (least HBM traffic); NEVER always streams.
 * The bytes are the same either way.  Applies to calls made afterwards; NVFP4_ERR_SHAPE for another value. */
enum { NVFP4_ONE_LAUNCH_AUTO = 0, NVFP4_ONE_LAUNCH_ALWAYS = 1, NVFP4_ONE_LAUNCH_NEVER = 2 };
int nvfp4_set_one_launch(int mode);

/* Every recorded duration of entry point `op`, in call order: up to max_records values in ms_out
 * (host pointer); returns how many were written, or a negative status.  Waits for the events. */
int  nvfp4_timing_read_all(int op, float *ms_out, int max_records);

/* Ceiling probes for benchmarks (no part of the NVFP4 path): what the GPU sustains on plain
 * streaming kernels and on back-to-back matrix instructions, to set the library's kernels against.
 *   kind 0: read `bytes` of a once (b: a sink of >= 16 KB, practically never written)
 *   kind 1: write `bytes` to b          kind 2: copy `bytes` from a to b
 *   kind 3: 256 workgroups x 4 waves, each `iters` x 64 v_mfma_f32_32x32x16_f16 on register-resident
 *           pseudo-random operands (b: a sink of >= 256 KB, practically never written);
 *           flops of one call = 256 * 4 * iters * 64 * 32768
 * a, b: device, 16-byte aligned; bytes a multiple of 16.  Recorded by the launch timing as NVFP4_OP_PROBE. */
int nvfp4_probe(int kind, const void *a, void *b, size_t bytes, int iters, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NVFP4_H */
