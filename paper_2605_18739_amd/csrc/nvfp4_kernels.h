// Host-side launchers of the gfx950 NVFP4 kernels (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nvfp4 {

constexpr int kMaxPartials = 1024;   // workgroups of the amax pass = partial maxima in the workspace

hipError_t launch_amax(const uint16_t *x, int64_t R, int64_t C, int64_t ld, uint32_t *partial,
                       int *n_partial, hipStream_t s);
// scale_search: the Four-over-Six candidate search per block (Appendix, Eq. 12-13)
hipError_t launch_quantize_rows(const uint16_t *x, int64_t R, int64_t C, int64_t ld, const float *gs_in,
                                const uint32_t *partial, int n_partial, uint8_t *codes, uint8_t *scales,
                                float *gs_out, hipStream_t s, bool scale_search = false);
hipError_t launch_quantize_cols(const uint16_t *x, int64_t R, int64_t C, int64_t ld, const float *gs_in,
                                const uint32_t *partial, int n_partial, uint8_t *codes, uint8_t *scales,
                                float *gs_out, hipStream_t s);
// gs_out = RN_fp32(max of the partial maxima / 2688) (1 if they are all zero): one small launch
hipError_t launch_scale_from_partials(const uint32_t *partial, int n_partial, float *gs_out, hipStream_t s);
hipError_t launch_dequant_bf16(const uint8_t *codes, const uint8_t *scales, const float *gs, int64_t rows,
                               int64_t K, uint16_t *out, hipStream_t s);

// One-launch variant for contiguous tensors that fit on the chip (registers + LDS of 256 compute units): every
// workgroup loads its slice once, the tensor maximum crosses the grid through library-owned words and a bounded wait, the
// codes are produced from the on-chip copy.  mean_out != nullptr: the smoothed-key path (row means removed, scale search).
bool quantize_rows_resident_fits(int64_t rows, int64_t C, int64_t ld, bool smooth);
hipError_t launch_quantize_rows_resident(const uint16_t *x, int64_t rows, int64_t C, uint8_t *codes,
                                         uint8_t *scales, float *gs_out, bool scale_search, uint16_t *mean_out,
                                         hipStream_t s, int heads = 0, int slab_heads = 0);   // slab_heads > 0: all-to-all slab order
bool quantize_rows_resident_pays(int64_t nblk, bool search_or_smooth);   // the dispatch rule on top of ..._fits
void set_one_launch_mode(int mode);               // 0: by that rule, 1: whenever the tensor fits, 2: never
void set_resident_spin_limit(uint32_t ticks);      // bound of the grid-wide wait, 10 ns ticks (0: give up at once)
uint32_t resident_spin_limit();

// [T, H, d] quantized along d with the rows regrouped into H / slab_heads per-destination slabs
hipError_t launch_quantize_rows_slabs(const uint16_t *x, int64_t T, int64_t H, int64_t d, int slab_heads,
                                      const float *gs_in, const uint32_t *partial, int n_partial,
                                      uint8_t *codes, uint8_t *scales, float *gs_out, hipStream_t s);

// Weight-gradient operands with the random Hadamard transform along the contraction axis (rows of x,
// groups of 16) before the transposed quantizer; sign_mask bit j = 1: s_j = -1.
// inexact (may be null): rht_inexact_bytes(R, C) bytes in which pass 1 leaves, per tile and lane, which groups the fp32
// transform is not exact for, and pass 2 finds them
size_t rht_inexact_bytes(int64_t R, int64_t C);
hipError_t launch_amax_rht(const uint16_t *x, int64_t R, int64_t C, int64_t ld, uint32_t sign_mask,
                           uint32_t *partial, int *n_partial, uint8_t *inexact, hipStream_t s);
hipError_t launch_quantize_cols_rht(const uint16_t *x, int64_t R, int64_t C, int64_t ld, uint32_t sign_mask,
                                    const float *gs_in, const uint32_t *partial, int n_partial,
                                    uint8_t *codes, uint8_t *scales, float *gs_out, const uint8_t *inexact, hipStream_t s);

// 2-D block scaling (one scale per 16x16 tile); codes_t / scales_t: the transposed operand, or nullptr
hipError_t launch_quantize_tiles(const uint16_t *x, int64_t R, int64_t C, int64_t ld, const float *gs_in,
                                 const uint32_t *partial, int n_partial, uint8_t *codes, uint8_t *scales,
                                 uint8_t *codes_t, uint8_t *scales_t, float *gs_out, float *gs_out_t,
                                 hipStream_t s);

// Smoothed key cache (Sec. 3.2, Eq. 6): pass 1 writes the row means and the partial maxima of the
// smoothed values; pass 2 removes the means again and runs the scale search.  d / 16 must be a
// power of two, at most 64.
hipError_t launch_amax_smooth(const uint16_t *x, int64_t rows, int d, uint16_t *mean_out, uint32_t *partial,
                              int *n_partial, hipStream_t s);
hipError_t launch_quantize_rows_smooth(const uint16_t *x, int64_t rows, int d, const uint16_t *row_mean,
                                       const uint32_t *partial, int n_partial, uint8_t *codes,
                                       uint8_t *scales, float *gs_out, hipStream_t s);

// Gathered KV reconstruction: several chunks, one launch.
constexpr int kMaxKvChunks = 64;
struct KvChunkDesc { const uint8_t *codes, *scales; const float *global_scale; const uint16_t *row_mean; int64_t T; };
hipError_t launch_dequant_gather(const KvChunkDesc *chunks, int n_chunks, int64_t H, int64_t d, uint16_t *out,
                                 hipStream_t s);

// Ceiling probes (benchmark utilities): kind 0 read `bytes` of a (b: a sink of at least 8 KB), 1 write `bytes` to b,
// 2 copy a -> b, 3 `iters` x 64 register-resident MFMAs per wave on 256 x 4 waves (b: a sink of at least 256 KB)
hipError_t launch_probe(int kind, const void *a, void *b, int64_t bytes, int iters, hipStream_t s);

// Epilogue of the GEMM
struct GemmEpilogue {
    int out_dtype;            // 0 fp32, 1 bf16, 2 none (quantized output only)
    int act;                  // 0 none, 1 gelu-tanh
    void *Y;                  // [M, N] fp32 or bf16, or nullptr
    int64_t ldy;
    int stream_out;           // 1: Y is written with streaming stores (outputs too large for anything to find them cached)
    uint32_t *amax_partial;   // per-workgroup |bf16(H)| maxima, or nullptr
    const float *q_scale;     // global scale for the fused quantizer, or nullptr (no fused quantize)
    float *q_scale_out;       // receives the scale that was used
    uint8_t *q_codes;         // [M, N/2]
    uint8_t *q_scales;        // [M, N/16]
};

// LoRA side branch fused into the GEMM: Y += scale * T B^T with T [M, kLoraRank], B [N, kLoraRank] bf16
// (t == nullptr: none).  Only for shapes the tiled kernels take, plain fp32 / bf16 output.
constexpr int kLoraRank = 128;
struct LoraBranch { const uint16_t *t = nullptr, *b = nullptr; float scale = 0.0f; };

hipError_t launch_gemm(const uint8_t *codesA, const uint8_t *scalesA, const float *gsA,
                       const uint8_t *codesW, const uint8_t *scalesW, const float *gsW, int64_t M,
                       int64_t N, int64_t K, const GemmEpilogue &ep, int *n_wg, hipStream_t s,
                       const LoraBranch &lora = LoraBranch());
// T = bf16(X A^T): X [M, K] bf16 (row stride ldx), A [kLoraRank, K] bf16, K % 16 == 0; the workspace
// (lora_down_workspace_bytes, 16-byte aligned) holds the fp32 partial tiles of the K ranges
size_t lora_down_workspace_bytes(int64_t M, int64_t K);
hipError_t launch_lora_down(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const uint16_t *a,
                            uint16_t *t, float *workspace, hipStream_t s);
int gemm_workgroups(int64_t M, int64_t N, int64_t K);
// the launches of a GEMM of this shape as text ("256x256:768 64x64:192"); returns their number, -1 if the text does not fit
int gemm_plan_text(int64_t M, int64_t N, int64_t K, char *text, size_t text_bytes);
bool gemm_is_tiled(int64_t M, int64_t N, int64_t K);   // false: the untiled fallback kernel (no fused epilogues)

}  // namespace nvfp4
