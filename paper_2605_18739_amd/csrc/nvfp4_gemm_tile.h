// Block-scaled FP4 GEMM for gfx950 (Sec. 2.2 / 3.1; Appendix "Implementation
// Details"):  Y[m,n] = gsA gsW * sum_k (cA[m,k] sA[m,k/16]) (cW[n,k] sW[n,k/16]).
//
// Route: every code*block_scale product (<= 6 significant bits, magnitude in
// [2^-10, 2688]) is an exact f16 number, and f16*f16 products are exact in the
// FP32 accumulator of v_mfma_f32_32x32x16_f16, so the only rounding left is the
// FP32 accumulation.  Codes become f16 with v_cvt_scalef32_pk_f16_fp4 (two codes
// per instruction) and one packed f16 multiply by the block scale
// (v_cvt_scalef32_pk_f16_fp8 turns the E4M3 byte into f16).
//
// One tiled kernel, gemm_regdq_kernel, in four tile shapes (256x256 and 256x192 for the
// bulk of a problem, 128x128 and 64x64 for small problems and the leftover rectangle of
// a launch plan): the operands stay 4-bit through LDS (filled by buffer loads that write
// LDS directly) and are expanded in registers in the shadow of the MFMAs that precede
// their use.  gemm_edge_kernel (nvfp4_gemm.hip) takes the shapes the tiles cannot (K or N not a
// multiple of 64 / 8).  plan_gemm picks tile shapes and splits a problem into whole waves
// of large tiles plus the leftover on small ones.
//
// Orientation: the MFMA's row operand is the W fragment and its column operand
// the A fragment, so a lane ends up with ONE output row m and runs of four
// consecutive n.  The epilogue transposes 32-row slabs through LDS so that
// global stores are 16 bytes per lane and whole rows of the tile are contiguous.
//
// This header holds the tiled kernel and its launcher; every tile shape is instantiated in a
// translation unit of its own (nvfp4_gemm_tile_*.hip) so that they compile side by side.
#ifndef NVFP4_GEMM_TILE_H
#define NVFP4_GEMM_TILE_H
#include "nvfp4_device.h"
#include "nvfp4_kernels.h"

#include <cstdio>
#include <type_traits>

// Empty inline-asm statements that tie values (or memory) to a point of the
// instruction stream; register constraints only exist in the device pass.
#if defined(__HIP_DEVICE_COMPILE__)
#define NVFP4_PIN1(a) asm volatile("" : "+v"(a))
#define NVFP4_PIN2(a, b) asm volatile("" : "+v"(a), "+v"(b))
#else
#define NVFP4_PIN1(a) ((void)(a))
#define NVFP4_PIN2(a, b) ((void)(a), (void)(b))
#endif
#define NVFP4_COMPILER_FENCE() asm volatile("" ::: "memory")

namespace nvfp4 {

constexpr int BK = 64;                 // K elements per pipeline step
constexpr int ROW_BYTES = BK * 2;      // one staged f16 row

// Epilogue variants (kernel template parameter): the kind of output, plus kEpiGelu when the
// tanh-form GELU is applied (a compile-time choice: as a run-time one the compiler evaluates
// the activation for every output and selects afterwards).
// kEpiLora: before the quantized operands are multiplied, the accumulators receive the low-rank
// update of a LoRA adapter (a kernel variant of its own, so that the plain kernels stay as they are).
enum { kEpiF32 = 0, kEpiBF16 = 1, kEpiQuant = 2, kEpiGelu = 4, kEpiLora = 8 };   // fp32 out, bf16 out, bf16 + fused re-quantization

struct GemmArgs {
    const uint8_t *codesA, *scalesA;
    const uint8_t *codesW, *scalesW;
    const float *gsA, *gsW;
    int64_t M, N, K;           // this launch's (sub-)problem
    GemmEpilogue ep;
    int n_tiles_n;             // tiles along N: workgroup t works on tile (t / n_tiles_n, t % n_tiles_n)
    int64_t q_pitch;           // row pitch in ELEMENTS of the fused quantizer's output (N of the whole problem)
    int partial_base;          // first slot of this launch in ep.amax_partial
    // LoRA side branch (kEpiLora kernels): Y += lora_scale * T B^T, T [M, 128], B [N, 128] bf16
    const uint16_t *lora_t, *lora_b;
    float lora_scale;
};

// tanh-form GELU in fp32: 0.5 y (1 + tanh(u)), u = sqrt(2/pi) (y + 0.044715 y^3).  With
// e = exp(2u), 0.5 (1 + tanh(u)) = e / (e + 1), so gelu = y e / (e + 1): no subtraction, hence no
// cancellation for negative y.  exp and the reciprocal are the hardware approximations (1 ulp);
// the exponent is clamped so that e stays finite (for large y, e / (e + 1) is 1 to fp32 anyway).
__device__ __forceinline__ float gelu_tanh_f32(float y)
{
    const float c2 = 2.0f * 0.7978845608028654f * 1.4426950408889634f;   // 2 sqrt(2/pi) log2(e)
    const float y2 = y * y;
    const float t = fminf(y * (c2 + (c2 * 0.044715f) * y2), 64.0f);      // 2u log2(e)
    const float e = __builtin_amdgcn_exp2f(t);
    return (y * e) * __builtin_amdgcn_rcpf(e + 1.0f);
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// 3-bit swizzle key of a row: distinct over every 8 consecutive rows and,
// combined with the row parity, over every 16.  LDS reads are served 16 lanes at
// a time out of 64 banks (256 B), writes 8 lanes at a time out of 128 B; with
// rows of 128 B (or a multiple) XOR-ing the 16-byte chunk index with this key
// makes "many rows, same chunk" accesses conflict free in both directions.
__device__ __forceinline__ int swz_key(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// byte offset of 16-byte chunk `c` (0..7) of staged row `row`
__device__ __forceinline__ int lds_chunk_off(int row, int c) { return row * ROW_BYTES + ((c ^ swz_key(row)) << 4); }

// Epilogue shared by the tiled kernels.  Each wave transposes its accumulators
// through a private 16 KB slab of LDS, 32 output rows at a time: a lane owns (row
// m, four consecutive n) after the MFMA, and (row m, 16 consecutive bytes) when
// it stores, so whole rows of the wave tile leave as contiguous runs.
template <int TM, int TN, int EPI_ACT, int NW = 4>
__device__ __forceinline__ void gemm_epilogue(float16v (&acc)[TN][TM], const GemmArgs &g, uint8_t *lds,
                                              int64_t wave_m0, int64_t wave_n0)
{
    constexpr int EPI = EPI_ACT & 3;
    constexpr bool GELU = (EPI_ACT & kEpiGelu) != 0;
    constexpr int WN = TN * 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lhalf = lane >> 5;
    __syncthreads();                              // all fragment reads of the main loop are done
    const float alpha = (*g.gsA) * (*g.gsW);
    const GemmEpilogue &ep = g.ep;
    uint8_t *slab = lds + wave * 16384;
    uint32_t hmax = 0;                            // largest |bf16(H)| pattern seen by this lane
    // fused quantizer: the tensor scale comes from the caller
    float q_sg = 1.0f, q_inv_6sg = 1.0f, q_shift = 1.0f;
    if constexpr (EPI == kEpiQuant) {
        const float sg_given = *ep.q_scale;
        if (blockIdx.x == 0 && tid == 0) *ep.q_scale_out = sg_given;
        q_shift = range_shift(sg_given);                  // 1 unless the scale is outside the fp32-safe range
        q_sg = sg_given * q_shift;
        q_inv_6sg = 1.0f / (6.0f * q_sg);
    }
    // granule swizzle: XOR with as many key bits as keep the index inside a row
    constexpr int KEYMASK = (WN % 64 == 0) ? 7 : 3;
    const int key = swz_key(lrow) & KEYMASK;
    auto epilogue_slab = [&](auto j_c) {
        constexpr int j = decltype(j_c)::value;
        if constexpr (EPI == kEpiF32) {
            // fp32: slab row = WN * 4 bytes, granule = 4 floats
            constexpr int ROWB = WN * 4, GPR = WN / 4;       // granules per row
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    float4v o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float y = acc[i][j][rg * 4 + e] * alpha;
                        if constexpr (GELU) y = gelu_tanh_f32(y);
                        o[e] = y;
                    }
                    const int gi = 8 * i + 2 * rg + lhalf;
                    *(float4v *)(slab + lrow * ROWB + ((gi ^ key) << 4)) = o;
                }
            // read back: lanes sweep granules of a row, then the next row
#pragma unroll
            for (int p = 0; p < 32 * GPR / 64; ++p) {
                const int idx = p * 64 + lane, r = idx / GPR, gi = idx % GPR;
                float4v o = *(const float4v *)(slab + r * ROWB + ((gi ^ (swz_key(r) & KEYMASK)) << 4));
                const int64_t m = wave_m0 + j * 32 + r, n = wave_n0 + gi * 4;
                if (m < g.M && n < g.N) {
                    float4v *dst = (float4v *)((float *)ep.Y + m * ep.ldy + n);
                    if (ep.stream_out) __builtin_nontemporal_store(o, dst);
                    else *dst = o;
                }
            }
        } else {
            // bf16: slab row = WN * 2 bytes, granule = 8 bf16; lane halves trade their
            // four-element runs so that every lane holds eight consecutive n
            constexpr int ROWB = WN * 2, GPR = WN / 8;
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int rp = 0; rp < 2; ++rp) {
                    uint32_t pk[2][2];
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        float y[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            y[e] = acc[i][j][(2 * rp + s) * 4 + e] * alpha;
                            if constexpr (GELU) y[e] = gelu_tanh_f32(y[e]);
                        }
                        pk[s][0] = pack_bf16x2(y[0], y[1]);
                        pk[s][1] = pack_bf16x2(y[2], y[3]);
                    }
                    // lower half keeps run s=0 and receives the upper half's s=0; upper half
                    // keeps s=1 and receives the lower half's s=1
                    auto x0 = __builtin_amdgcn_permlane32_swap(pk[0][0], pk[1][0], false, false);
                    auto x1 = __builtin_amdgcn_permlane32_swap(pk[0][1], pk[1][1], false, false);
                    uint4v o = {x0[0], x1[0], x0[1], x1[1]};
                    const int gi = 4 * i + 2 * rp + lhalf;
                    *(uint4v *)(slab + lrow * ROWB + ((gi ^ key) << 4)) = o;
                }
            if (EPI == kEpiBF16 || ep.Y != nullptr) {
#pragma unroll
                for (int p = 0; p < 32 * GPR / 64; ++p) {
                    const int idx = p * 64 + lane, r = idx / GPR, gi = idx % GPR;
                    uint4v o = *(const uint4v *)(slab + r * ROWB + ((gi ^ (swz_key(r) & KEYMASK)) << 4));
                    const int64_t m = wave_m0 + j * 32 + r, n = wave_n0 + gi * 8;
                    if (m < g.M && n < g.N) {
                        if (ep.amax_partial) {
                            hmax = pk_absmax_u16(hmax, o.x);
                            hmax = pk_absmax_u16(hmax, o.y);
                            hmax = pk_absmax_u16(hmax, o.z);
                            hmax = pk_absmax_u16(hmax, o.w);
                        }
                        uint4v *dst = (uint4v *)((uint16_t *)ep.Y + m * ep.ldy + n);
                        if (ep.stream_out) __builtin_nontemporal_store(o, dst);
                        else *dst = o;
                    }
                }
            }
            if constexpr (EPI == kEpiQuant) {
                // fused re-quantization along n: a lane takes one 16-element block (two
                // granules) of the bf16 slab and runs the exact block quantizer on it
                constexpr int BPR = WN / 16;                  // blocks per slab row
#pragma unroll
                for (int p = 0; p < 32 * BPR / 64; ++p) {
                    const int idx = p * 64 + lane, r = idx / BPR, b = idx % BPR;
                    const int kr = swz_key(r) & KEYMASK;
                    uint4v lo = *(const uint4v *)(slab + r * ROWB + (((2 * b) ^ kr) << 4));
                    uint4v hi = *(const uint4v *)(slab + r * ROWB + (((2 * b + 1) ^ kr) << 4));
                    const int64_t m = wave_m0 + j * 32 + r, n = wave_n0 + b * 16;
                    if (m < g.M && n < g.N) {                 // N % 16 == 0: a block is all in or all out
                        uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                        if (__builtin_expect(q_shift != 1.0f, 0)) rescale_block16(w, q_shift);
                        uint32_t am = 0;
#pragma unroll
                        for (int q = 0; q < 8; ++q) am = pk_absmax_u16(am, w[q]);
                        const float bmax = __uint_as_float(pk_hmax_u16(am) << 16);
                        const uint32_t sbyte = block_scale_exact(bmax, q_sg, q_inv_6sg);
                        uint32_t c0, c1;
                        encode_block16(w, e4m3_to_f32(sbyte), q_sg, c0, c1);
                        uint2v cc = {c0, c1};
                        *(uint2v *)(ep.q_codes + m * (g.q_pitch >> 1) + (n >> 1)) = cc;
                        ep.q_scales[m * (g.q_pitch >> 4) + (n >> 4)] = (uint8_t)sbyte;
                    }
                }
            }
        }
    };
    epilogue_slab(std::integral_constant<int, 0>{});
    if constexpr (TM > 1) epilogue_slab(std::integral_constant<int, 1>{});
    if constexpr (TM > 2) epilogue_slab(std::integral_constant<int, 2>{});
    if constexpr (TM > 3) epilogue_slab(std::integral_constant<int, 3>{});
    if (ep.amax_partial) {
        uint32_t mx = wave_max_u32(pk_hmax_u16(hmax));
        __syncthreads();                          // slabs are no longer needed
        uint32_t *wmax = (uint32_t *)lds;
        if (lane == 0) wmax[wave] = mx;
        __syncthreads();
        if (tid == 0) {
            uint32_t all = wmax[0];
#pragma unroll
            for (int w = 1; w < NW; ++w) all = max(all, wmax[w]);
            ep.amax_partial[g.partial_base + blockIdx.x] = all;
        }
    }
}

// f(integral_constant<int, I>) for I = First .. Last - 1: a loop whose index is a compile-time
// constant in the body (array indices stay constants, guards can be `if constexpr`)
template <int First, int Last, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (First < Last) {
        f(std::integral_constant<int, First>{});
        static_for<First + 1, Last>(f);
    }
}

// ============================================================================
// Register-dequantizing tiled kernel.
//
// The operands stay 4-bit all the way into LDS.  Every 128 k the packed codes of
// the tile (64 B per row) are copied HBM -> LDS by buffer loads that write LDS
// directly (no registers, no VALU, no LDS-write instructions); four lanes fetch
// the four 16-byte chunks of one row, so a copy instruction touches 16 rows, not
// 64.  The E4M3 scales follow every 256 k (16 B per row).  A wave reads its own
// rows' codes back with one 128-bit LDS read per 32-row tile and 64 k, and
// expands them in registers right before the MFMAs that consume them: one
// v_cvt_scalef32_pk_f16_fp4 and one v_pk_mul_f16 per pair of elements.  On this
// machine VALU instructions issue in the shadow of a running MFMA while LDS and
// memory instructions largely do not, so trading LDS traffic (4x fewer bytes
// and instructions than staging f16) for VALU work (each operand element is
// expanded by the two waves that use it) is what keeps the matrix pipe busy.
//
// K order: a "register step" is 64 k = four MFMA sub-steps.  In register step
// (g, half) -- g counts 128-k copy steps -- lane half h (lanes 32h .. 32h+31) of
// an MFMA operand owns chunk 2 h + half of its row, i.e. k = 128 g + 32 (2 h +
// half) + 0..31, and MFMA sub-step j multiplies the eight codes of dword j of that
// chunk, which share block scale 4 h + 2 half + j/2 of the copy step: the four
// scale bytes a lane needs for one copy step are one aligned dword, read once.
// This is a permutation of k applied to both operands alike.
//
// LDS: chunk c of staged row r sits in 16-byte slot 4 r + (c ^ ((r >> 2) & 3)) of
// its stage; the copy instructions fill slots in lane order (lane l of unit u
// fetches row 16 u + l/4, chunk (l & 3) ^ key), and sixteen consecutive rows of
// one chunk -- what a fragment read touches per LDS cycle -- fall on distinct
// banks.
// ============================================================================
constexpr int kRegdqWaves = 4;         // waves per workgroup: 2 x 2, one per SIMD (two per SIMD measured no faster)
constexpr int kCodeStages = 4;         // LDS ring of 128-k code stages: copies run three copy steps ahead, one barrier per two
constexpr int kScaleSteps = 2;         // copy steps covered by one 16-byte run of scales

// s_waitcnt vmcnt(N) alone: vmcnt sits in bits 3:0 and 15:14, expcnt (6:4) and
// lgkmcnt (11:8) are left at "do not wait".
template <int N>
__device__ __forceinline__ void wait_vmcnt_le()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

// MFMA of a sub-step behind which fragment f is read (and, two sub-steps later, its scales converted): one
// fragment per MFMA where a sub-step has at least as many MFMAs as fragments (the large tiles), otherwise
// the fragments are dealt over the MFMAs there are
template <int NMF, int NF>
constexpr int frag_slot(int f) { return NMF >= NF ? f : f * NMF / NF; }

template <int BM, int BN, int EPI, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_regdq_kernel(GemmArgs g)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub
    // wave grid: 2 x 2 (one wave per SIMD), or eight waves (two per SIMD) as 2 x 4 / 4 x 2
    constexpr int WGN = NW == 4 ? 2 : (BN % 128 == 0 ? 4 : 2), WGM = NW / WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN;    // per-wave tile
    constexpr int TM = WM / 32, TN = WN / 32;      // 32x32 MFMA tiles per wave
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
    constexpr int NF = TM + TN;                    // operand fragments per MFMA sub-step
    constexpr int NMF = TM * TN;                   // MFMAs per sub-step
    constexpr int ROWS = BM + BN;                  // staged rows: A rows first, then W rows
    constexpr int CODE_STAGE = ROWS * 64;          // 128 k of codes per row
    constexpr int SCALE_STAGE = ROWS * 16;         // 256 k of scales per row
    constexpr int SCALE_BASE = kCodeStages * CODE_STAGE;
    constexpr int UNITS = ROWS / 16, UPW = (UNITS + NW - 1) / NW;     // 1 KB code copies per stage / per wave (at most)
    constexpr int SUNITS = ROWS / 64, SUPW = (SUNITS + NW - 1) / NW;  // 1 KB scale copies
    static_assert(BM % 64 == 0 && BN % 64 == 0, "tile shape");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    typedef __attribute__((address_space(3))) void *lds_ptr_t;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: it selects LDS targets of the copies
    const int wm = wave / WGN, wn = wave % WGN;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int64_t m0 = (int64_t)(blockIdx.x / g.n_tiles_n) * BM, n0 = (int64_t)(blockIdx.x % g.n_tiles_n) * BN;
    const int kbytes = (int)(g.K >> 1), kblocks = (int)(g.K >> 4);
    const int GT = (int)((g.K + 2 * BK - 1) / (2 * BK));   // copy steps
    const int KT = 2 * GT;                         // register steps (K = 64 mod 128: the upper half of the last copy step is zeros)
    const bool k_tail = (g.K & (2 * BK - 1)) != 0;

    // Copies are range checked against the operand size: a row past the end of the
    // operand, and the part of the last copy step past the end of the last row, read
    // as zeros (all per-lane offsets live in the checked vector offset).
    const __amdgpu_buffer_rsrc_t rcA = __builtin_amdgcn_make_buffer_rsrc((void *)g.codesA, 0, (int)(g.M * kbytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc((void *)g.scalesA, 0, (int)(g.M * kblocks), 0x00020000);
    const __amdgpu_buffer_rsrc_t rcW = __builtin_amdgcn_make_buffer_rsrc((void *)g.codesW, 0, (int)(g.N * kbytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsW = __builtin_amdgcn_make_buffer_rsrc((void *)g.scalesW, 0, (int)(g.N * kblocks), 0x00020000);

    // ---- copy units.  Code unit u (0 .. UNITS-1) is 16 consecutive staged rows, 64 B
    // each; wave w issues units w, w + NW, w + 2 NW, ...  Scale unit: 64 rows, 16 B each.
    // Every wave issues the same number of copies per step (the prologue's wait counts them):
    // where the units do not divide evenly a wave repeats the last unit, which writes the
    // same bytes to the same place.
    auto code_unit = [&](int x) { return min(wave + NW * x, UNITS - 1); };
    auto scale_unit = [&](int x) { return min(wave + NW * x, SUNITS - 1); };
    int cvoff[UPW], svoff[SUPW];
#pragma unroll
    for (int x = 0; x < UPW; ++x) {
        const int srow = code_unit(x) * 16 + (lane >> 2);
        const int chunk = (lane & 3) ^ ((srow >> 2) & 3);
        const bool isA = srow < BM;
        const int64_t gr = isA ? m0 + srow : n0 + (srow - BM);
        cvoff[x] = gr < (isA ? g.M : g.N) ? (int)(gr * kbytes) + chunk * 16 : 0x7FF00000;
    }
#pragma unroll
    for (int x = 0; x < SUPW; ++x) {
        const int srow = scale_unit(x) * 64 + lane;
        const bool isA = srow < BM;
        const int64_t gr = isA ? m0 + srow : n0 + (srow - BM);
        svoff[x] = gr < (isA ? g.M : g.N) ? (int)(gr * kblocks) : 0x7FF00000;
    }
    // A lane fetches chunk (lane & 3) ^ ((lane >> 4) & 3) of its row in every unit.  When K ends in
    // the middle of the last copy step, chunks 2 and 3 of that step lie past the end of the row:
    // their lanes get an offset past the end of the operand, which reads as zeros.
    const bool hi_chunk = (((lane & 3) ^ ((lane >> 4) & 3)) & 2) != 0;
    auto copy_code_unit = [&](int gs, int x) {      // this wave's x-th unit of copy step gs -> code stage gs % kCodeStages
        const int past = (k_tail && gs == GT - 1 && hi_chunk) ? 0x7FF00000 : 0;
        const int u = code_unit(x);
        uint8_t *dst = lds + (gs & (kCodeStages - 1)) * CODE_STAGE + u * 1024;
        if (u * 16 < BM) __builtin_amdgcn_raw_ptr_buffer_load_lds(rcA, (lds_ptr_t)dst, 16, (cvoff[x] + gs * 64) | past, 0, 0, 0);
        else __builtin_amdgcn_raw_ptr_buffer_load_lds(rcW, (lds_ptr_t)dst, 16, (cvoff[x] + gs * 64) | past, 0, 0, 0);
    };
    auto copy_codes = [&](int gs) {
#pragma unroll
        for (int x = 0; x < UPW; ++x) copy_code_unit(gs, x);
    };
    auto copy_scales = [&](int grp) {               // scale group grp (copy steps 2 grp, 2 grp + 1) -> scale stage grp & 1
#pragma unroll
        for (int x = 0; x < SUPW; ++x) {
            const int u = scale_unit(x);
            uint8_t *dst = lds + SCALE_BASE + (grp & 1) * SCALE_STAGE + u * 1024;
            if (u * 64 < BM) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (lds_ptr_t)dst, 16, svoff[x] + grp * 16, 0, 0, 0);
            else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsW, (lds_ptr_t)dst, 16, svoff[x] + grp * 16, 0, 0, 0);
        }
    };

    // ---- what this lane reads back.  Fragment f (0..TM-1: A tiles, TM..NF-1: W tiles)
    // is staged row frag_row(f); all of a lane's rows share the swizzle key.
    const int key = (lrow >> 2) & 3;
    int code_lane[2];                               // byte offset inside a stage for half 0 / 1, tile 0 of A
#pragma unroll
    for (int half = 0; half < 2; ++half) code_lane[half] = lrow * 64 + (((2 * lhalf + half) ^ key) << 4);
    const int scale_lane = lrow * 16 + 4 * lhalf;
    auto frag_row0 = [&](int f) { return f < TM ? wm * WM + f * 32 : BM + wn * WN + (f - TM) * 32; };
    uint4v codes[2][NF];          // packed codes of the register step being multiplied / the next one
    uint32_t scl[NF];             // the four block scales (E4M3 bytes) of a lane's two register steps of one copy step ...
    uint32_t scf[2][NF];          // ... and those of one register step as a pair of f16
    // register step rs = 2 gs + half; with_scales: rs is even, the copy step's scales are read too
    auto read_frag = [&](int rs, int set, int f, bool with_scales) {
        const int gs = rs >> 1, half = rs & 1;
        const uint8_t *cbase = lds + (gs & (kCodeStages - 1)) * CODE_STAGE + code_lane[half];
        const uint8_t *sbase = lds + SCALE_BASE + ((gs >> 1) & 1) * SCALE_STAGE + (gs & 1) * 8 + scale_lane;
        codes[set][f] = *(const uint4v *)(cbase + frag_row0(f) * 64);
        if (with_scales) scl[f] = *(const uint32_t *)(sbase + frag_row0(f) * 16);
    };
    auto read_step = [&](int rs, int set, bool with_scales) {
#pragma unroll
        for (int f = 0; f < NF; ++f) read_frag(rs, set, f, with_scales);
    };

    float16v acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    if constexpr ((EPI & kEpiLora) != 0) {
        // ---- LoRA phase (Sec. 2.2 / 3.1: low-rank adapter beside the quantized weight).  The
        // tile's 256 + BN rows of T and B (128 bf16 = 256 B each) are copied into LDS, multiplied
        // with v_mfma_f32_32x32x16_bf16 in eight 16-wide sub-steps, and the accumulators are
        // rescaled by lora_scale / (gsA gsW) so that the quantized product can be added on top
        // and the epilogue's single multiplication by gsA gsW leaves lora_scale * T B^T.
        // LDS: row r at 256 r, its sixteen 16-byte chunks XOR-swizzled with r & 15 (sixteen rows
        // of one chunk, what a fragment read touches per LDS cycle, fall on distinct banks).
        typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
        const __amdgpu_buffer_rsrc_t rT = __builtin_amdgcn_make_buffer_rsrc((void *)g.lora_t, 0, (int)(g.M * 256), 0x00020000);
        const __amdgpu_buffer_rsrc_t rB = __builtin_amdgcn_make_buffer_rsrc((void *)g.lora_b, 0, (int)(g.N * 256), 0x00020000);
        constexpr int LUNITS = ROWS / 4;               // 1 KB copies: four rows each
#pragma unroll
        for (int x = 0; x < LUNITS / NW; ++x) {
            const int u = wave + NW * x;
            const int srow = 4 * u + (lane >> 4);
            const int chunk = (lane & 15) ^ (srow & 15);
            uint8_t *dst = lds + u * 1024;
            if (4 * u < BM) {
                const int64_t gr = m0 + srow;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rT, (lds_ptr_t)dst, 16, gr < g.M ? (int)(gr * 256) + chunk * 16 : 0x7FF00000, 0, 0, 0);
            } else {
                const int64_t gr = n0 + (srow - BM);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rB, (lds_ptr_t)dst, 16, gr < g.N ? (int)(gr * 256) + chunk * 16 : 0x7FF00000, 0, 0, 0);
            }
        }
        wait_vmcnt_le<0>();
        NVFP4_COMPILER_FENCE();
        __builtin_amdgcn_s_barrier();
        NVFP4_COMPILER_FENCE();
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            uint4v lf[NF];
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                const int row = frag_row0(f) + lrow;
                lf[f] = *(const uint4v *)(lds + row * 256 + (((2 * kk + lhalf) ^ (row & 15)) << 4));
            }
#pragma unroll
            for (int t = 0; t < NMF; ++t) {
                const int i = t / TM, jj = t % TM;
                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8v, lf[TM + i]),
                                                                      __builtin_bit_cast(bf16x8v, lf[jj]), acc[i][jj], 0, 0, 0);
            }
        }
        const float rescale = g.lora_scale / ((*g.gsA) * (*g.gsW));
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] *= rescale;
        NVFP4_COMPILER_FENCE();
        __builtin_amdgcn_s_barrier();                   // every wave has read its rows: the stages may be filled
        NVFP4_COMPILER_FENCE();
    }

    // fragments of MFMA sub-step j live in frag[j & 1]; order: A tiles then W tiles
    uint4v frag[2][NF];
    // piece pc (0 .. 2 NF - 1) of sub-step j of register set `set`: half a fragment
    auto expand_piece = [&](int set, int j, int pc) {
        const int f = pc >> 1, hp = pc & 1;
        // the block scale of this sub-step sits in the LOW half of scf (see shift_scale below): a packed multiply
        // that broadcasts the low half of its first operand is the one form the compiler follows with an MFMA
        // without a wait state in between
        (void)j;
        const half2v sc = __builtin_bit_cast(half2v, scf[set][f]);
        const half2v p = half2v{sc.x, sc.x};
        const uint32_t w = codes[set][f][j];
        const int d0 = 2 * hp, d1 = 2 * hp + 1;
        half2v e0 = hp ? __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 2) : __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 0);
        half2v e1 = hp ? __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 3) : __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 1);
        uint32_t x0 = __builtin_bit_cast(uint32_t, e0 * p), x1 = __builtin_bit_cast(uint32_t, e1 * p);
        // keep the expansion where it is written: without this the optimizer sinks it
        // towards its use, out of the shadow of the MFMAs it is meant to hide behind
        NVFP4_PIN2(x0, x1);
        frag[j & 1][f][d0] = x0;
        frag[j & 1][f][d1] = x1;
    };
    // E4M3 pair of register step parity `odd` (low / high half of the dword) -> f16 pair, pinned where it is written
    auto convert_scales = [&](int set, int f, bool odd) {
        uint32_t raw = scl[f];
        NVFP4_PIN1(raw);                            // do not touch it before this point (the LDS read may still be in flight)
        uint32_t x = odd ? __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(raw, 1.0f, true))
                         : __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(raw, 1.0f, false));
        NVFP4_PIN1(x);
        scl[f] = raw;
        scf[set][f] = x;
    };

    // ---- prologue: copy steps 0, 1, 2 started, 0 and 1 awaited (step 1 is first read in an
    // iteration without a barrier), register step 0 read and expanded
    copy_scales(0);
    copy_codes(0);
    copy_codes(min(1, GT - 1));
    copy_scales(min(2, GT - 1) >> 1);
    copy_codes(min(2, GT - 1));
    wait_vmcnt_le<UPW + SUPW>();                    // everything but copy step 2 and its scales has landed
    NVFP4_COMPILER_FENCE();
    __builtin_amdgcn_s_barrier();
    NVFP4_COMPILER_FENCE();
    read_step(0, 0, true);
#pragma unroll
    for (int f = 0; f < NF; ++f) convert_scales(0, f, false);
#pragma unroll
    for (int pc = 0; pc < 2 * NF; ++pc) expand_piece(0, 0, pc);

    // ---- main loop over register steps.  Iteration rs reads register step rs+1 into
    // the other register set and multiplies step rs.  Copy step g lives in stage g mod 4
    // and is started three copy steps ahead: every odd iteration rs starts copy step
    // rs/2 + 3 into the stage of copy step rs/2 - 1.  Only every second odd iteration
    // (rs = 3 mod 4) waits for this wave's copies and joins a barrier: that makes copy
    // steps rs/2 + 1 and rs/2 + 2 visible (the second one is first read two iterations
    // later, without a barrier), and no wave can be more than one barrier ahead of
    // another, which is what keeps a stage from being refilled while it is still read.
    auto iteration = [&](int rs, auto quarter_c) {
        constexpr int quarter = decltype(quarter_c)::value;    // rs & 3
        constexpr int half = quarter & 1;                      // also the register set of step rs
        constexpr int set = half;
        if constexpr (quarter == 3) {
            wait_vmcnt_le<0>();
            NVFP4_COMPILER_FENCE();
            __builtin_amdgcn_s_barrier();
            NVFP4_COMPILER_FENCE();
        }
        // The LDS reads of the next register step and (odd iterations) the copies of copy step
        // rs/2 + 3 are dealt out behind the MFMAs of sub-steps 0 and 1, one per MFMA, so that
        // their issue overlaps a running MFMA instead of leaving the matrix pipe idle.
        const int ng = min((rs >> 1) + 3, GT - 1);          // copy step to start (clamped at the end of K)
        static_for<0, 4>([&](auto j_c) {
            constexpr int j = decltype(j_c)::value;
            static_for<0, NMF>([&](auto t_c) {
                constexpr int t = decltype(t_c)::value;
                constexpr int i = t / TM, jj = t % TM;
                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8v, frag[j & 1][TM + i]),
                                                                     __builtin_bit_cast(half8v, frag[j & 1][jj]),
                                                                     acc[i][jj], 0, 0, 0);
                // the MFMA stays first in its slot: left to itself the scheduler moves it behind the slot's copy
                // instruction, and two MFMAs then issue back to back with nothing in the first one's shadow
                __builtin_amdgcn_sched_barrier(0);
                // next sub-step's fragments: 2 NF pieces dealt over the NMF MFMAs
                static_for<0, 2 * NF>([&](auto pc_c) {
                    constexpr int pc = decltype(pc_c)::value;
                    if constexpr (pc * NMF / (2 * NF) == t) {
                        if constexpr (j < 3) expand_piece(set, j + 1, pc);
                        else expand_piece(set ^ 1, 0, pc);
                    }
                });
                // scf[set][f] holds (scale of sub-steps 0, 1 | scale of sub-steps 2, 3); once the fragment's pieces for
                // sub-step 1 are out (they are dealt during sub-step 0) the pair moves down by 16 bits, in place
                static_for<0, NF>([&](auto f_c) {
                    constexpr int f = decltype(f_c)::value;
                    if constexpr (j == 0 && (2 * f + 1) * NMF / (2 * NF) == t) {
                        uint32_t x = scf[set][f] >> 16;
                        NVFP4_PIN1(x);
                        scf[set][f] = x;
                    }
                });
                // fragment f of the next register step is read behind MFMA frag_slot(f) of sub-step 0
                static_for<0, NF>([&](auto f_c) {
                    constexpr int f = decltype(f_c)::value;
                    if constexpr (j == 0 && frag_slot<NMF, NF>(f) == t) read_frag(rs + 1, set ^ 1, f, half == 1);
                    // the next step's scales (read during sub-step 0) become f16 during sub-step 2
                    if constexpr (j == 2 && frag_slot<NMF, NF>(f) == t) convert_scales(set ^ 1, f, half == 0);
                });
                if constexpr (half == 1 && j == 1) {
                    static_for<0, UPW>([&](auto x_c) {
                        constexpr int x = decltype(x_c)::value;
                        if constexpr (x * NMF / UPW == t) copy_code_unit(ng, x);
                    });
                    if constexpr (quarter == 3 && t == NMF - 1) copy_scales(ng >> 1);   // ng is even here: a new scale group
                }
                __builtin_amdgcn_sched_barrier(0);      // keeps the hand-placed order: nothing moves across an MFMA
            });
        });
    };
    {
        using Q0 = std::integral_constant<int, 0>;
        using Q1 = std::integral_constant<int, 1>;
        using Q2 = std::integral_constant<int, 2>;
        using Q3 = std::integral_constant<int, 3>;
        int rs = 0;
        for (; rs + 3 < KT; rs += 4) {
            iteration(rs, Q0{});
            iteration(rs + 1, Q1{});
            iteration(rs + 2, Q2{});
            iteration(rs + 3, Q3{});
        }
        if (rs < KT) {                              // KT is even: two steps are left, or none
            iteration(rs, Q0{});
            iteration(rs + 1, Q1{});
        }
    }
    wait_vmcnt_le<0>();                            // no copy may still be writing LDS when the epilogue reuses it
    __syncthreads();
    gemm_epilogue<TM, TN, EPI, NW>(acc, g, lds, m0 + wm * WM, n0 + wn * WN);
#else
    (void)g;
#endif
}

template <int BM, int BN, int EPI>
static hipError_t launch_regdq(const GemmArgs &g, int64_t tiles, hipStream_t s)
{
    constexpr int NW = BM >= 256 ? kRegdqWaves : 4;   // the small tiles always run four waves
    constexpr int smem_main = kCodeStages * (BM + BN) * 64 + 2 * (BM + BN) * 16, smem_epi = NW * 16384;
    constexpr int smem = smem_main > smem_epi ? smem_main : smem_epi;
    // the dynamic LDS limit is raised once per kernel variant and device
    static uint64_t attr_set = 0;
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (((attr_set >> (dev & 63)) & 1u) == 0) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_regdq_kernel<BM, BN, EPI, NW>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set |= 1ull << (dev & 63);
    }
    GemmArgs a = g;
    a.n_tiles_n = (int)((g.N + BN - 1) / BN);
    const unsigned grid = (unsigned)tiles;          // a prefix of the row-major tile grid
    gemm_regdq_kernel<BM, BN, EPI, NW><<<grid, NW * 64, smem, s>>>(a);
    return hipGetLastError();
}

// One tile shape with the epilogue variant chosen at run time (epi: kEpi* bits).  The LoRA phase
// exists for the 256-row tiles only.
template <int BM, int BN>
static hipError_t launch_tile(int epi, const GemmArgs &g, int64_t tiles, hipStream_t s)
{
    switch (epi) {
    case kEpiF32: return launch_regdq<BM, BN, kEpiF32>(g, tiles, s);
    case kEpiBF16: return launch_regdq<BM, BN, kEpiBF16>(g, tiles, s);
    case kEpiBF16 | kEpiGelu: return launch_regdq<BM, BN, kEpiBF16 | kEpiGelu>(g, tiles, s);
    case kEpiQuant: return launch_regdq<BM, BN, kEpiQuant>(g, tiles, s);
    case kEpiQuant | kEpiGelu: return launch_regdq<BM, BN, kEpiQuant | kEpiGelu>(g, tiles, s);
    case kEpiF32 | kEpiLora:
        if constexpr (BM >= 256) return launch_regdq<BM, BN, kEpiF32 | kEpiLora>(g, tiles, s);
        else return hipErrorInvalidValue;
    case kEpiBF16 | kEpiLora:
        if constexpr (BM >= 256) return launch_regdq<BM, BN, kEpiBF16 | kEpiLora>(g, tiles, s);
        else return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
    }
}

// defined in nvfp4_gemm_tile_*.hip
hipError_t launch_tile_256x256(int epi, const GemmArgs &g, int64_t tiles, hipStream_t s);
hipError_t launch_tile_256x192(int epi, const GemmArgs &g, int64_t tiles, hipStream_t s);
hipError_t launch_tile_128x128(int epi, const GemmArgs &g, int64_t tiles, hipStream_t s);
hipError_t launch_tile_64x64(int epi, const GemmArgs &g, int64_t tiles, hipStream_t s);

}  // namespace nvfp4
#endif  // NVFP4_GEMM_TILE_H
