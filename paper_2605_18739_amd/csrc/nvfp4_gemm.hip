// Block-scaled FP4 GEMM for gfx950 (Sec. 2.2 / 3.1; Appendix "Implementation
// Details"):  Y[m,n] = gsA gsW * sum_k (cA[m,k] sA[m,k/16]) (cW[n,k] sW[n,k/16]).
//
// Route: every code*block_scale product (<= 6 significant bits, magnitude in
// [2^-10, 2688]) is an exact f16 number, and f16*f16 products are exact in the
// FP32 accumulator of v_mfma_f32_32x32x16_f16, so the only rounding left is the
// FP32 accumulation.  Packed codes travel HBM -> registers (128-bit loads),
// are expanded once per workgroup with v_cvt_scalef32_pk_f16_fp4 (two codes per
// instruction) and one packed f16 multiply by the block scale, and are staged
// in LDS as f16 in an XOR-swizzled layout that both the 128-bit writes and the
// 128-bit MFMA fragment reads hit without bank conflicts.
//
// Orientation: the MFMA's row operand is the W fragment and its column operand
// the A fragment, so a lane ends up with ONE output row m and runs of four
// consecutive n -- 16-byte stores, and the fused quantizer of the epilogue finds
// half of every 16-element block inside a lane.
#include "nvfp4_device.h"
#include "nvfp4_kernels.h"

namespace nvfp4 {

constexpr int BK = 64;                 // K elements per pipeline step
constexpr int ROW_BYTES = BK * 2;      // one staged f16 row

struct GemmArgs {
    const uint8_t *codesA, *scalesA;
    const uint8_t *codesW, *scalesW;
    const float *gsA, *gsW;
    int64_t M, N, K;
    GemmEpilogue ep;
};

// tanh-form GELU in fp32
__device__ __forceinline__ float gelu_tanh_f32(float y)
{
    const float c = 0.7978845608028654f;
    float u = c * (y + 0.044715f * y * y * y);
    // tanh(u) = 1 - 2 / (exp(2u) + 1)
    float e = __expf(2.0f * u);
    float t = 1.0f - 2.0f / (e + 1.0f);
    return 0.5f * y * (1.0f + t);
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// One 16-byte chunk of codes (32 elements = 2 blocks) -> four 16-byte f16 chunks.
__device__ __forceinline__ void expand_chunk(const uint4v &c, uint32_t scale2, half8v (&out)[4])
{
    _Float16 s0 = e4m3_to_f16(scale2 & 0x7Fu), s1 = e4m3_to_f16((scale2 >> 8) & 0x7Fu);
    half2v p0 = {s0, s0}, p1 = {s1, s1};
#define NVFP4_EXPAND(I, W, P)                                                        \
    {                                                                                \
        half2v a = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(W, 1.0f, 0) * P;         \
        half2v b = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(W, 1.0f, 1) * P;         \
        half2v cc = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(W, 1.0f, 2) * P;        \
        half2v d = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(W, 1.0f, 3) * P;         \
        out[I] = half8v{a.x, a.y, b.x, b.y, cc.x, cc.y, d.x, d.y};                   \
    }
    NVFP4_EXPAND(0, c.x, p0) NVFP4_EXPAND(1, c.y, p0) NVFP4_EXPAND(2, c.z, p1) NVFP4_EXPAND(3, c.w, p1)
#undef NVFP4_EXPAND
}

// byte offset of 16-byte chunk `c` (0..7) of staged row `row`
__device__ __forceinline__ int lds_chunk_off(int row, int c) { return row * ROW_BYTES + ((c ^ (row & 7)) << 4); }

template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_f16mfma_kernel(GemmArgs g)
{
    constexpr int WM = BM / 2, WN = BN / 2;        // per-wave tile (2 x 2 waves)
    constexpr int TM = WM / 32, TN = WN / 32;      // 32x32 MFMA tiles per wave
    constexpr int CA = BM * 2 / 256, CW = BN * 2 / 256;   // 16-byte code chunks per thread and step
    constexpr int STAGE = (BM + BN) * ROW_BYTES;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.y * BM, n0 = (int64_t)blockIdx.x * BN;
    const int64_t kbytes = g.K >> 1, kblocks = g.K >> 4;
    const int KT = (int)(g.K / BK);

    // staging assignment: chunk q of this thread covers row (tid + 256 q) / 2, half (tid & 1)
    const uint8_t *pa[CA], *psa[CA], *pw[CW], *psw[CW];
    int la[CA], lw[CW];
#pragma unroll
    for (int q = 0; q < CA; ++q) {
        int row = (tid + 256 * q) >> 1, h = tid & 1;
        int64_t gr = min(m0 + row, g.M - 1);
        pa[q] = g.codesA + gr * kbytes + h * 16;
        psa[q] = g.scalesA + gr * kblocks + h * 2;
        la[q] = row;
    }
#pragma unroll
    for (int q = 0; q < CW; ++q) {
        int row = (tid + 256 * q) >> 1, h = tid & 1;
        int64_t gr = min(n0 + row, g.N - 1);
        pw[q] = g.codesW + gr * kbytes + h * 16;
        psw[q] = g.scalesW + gr * kblocks + h * 2;
        lw[q] = row;
    }
    const int hsel = tid & 1;

    uint4v ra[CA], rw[CW];
    uint32_t sa[CA], sw[CW];
    auto load_step = [&](int kt) {
#pragma unroll
        for (int q = 0; q < CA; ++q) {
            ra[q] = *(const uint4v *)(pa[q] + (int64_t)kt * 32);
            sa[q] = *(const uint16_t *)(psa[q] + (int64_t)kt * 4);
        }
#pragma unroll
        for (int q = 0; q < CW; ++q) {
            rw[q] = *(const uint4v *)(pw[q] + (int64_t)kt * 32);
            sw[q] = *(const uint16_t *)(psw[q] + (int64_t)kt * 4);
        }
    };
    auto stage_step = [&](int buf) {
        uint8_t *base = lds + buf * STAGE;
#pragma unroll
        for (int q = 0; q < CA; ++q) {
            half8v e[4];
            expand_chunk(ra[q], sa[q], e);
#pragma unroll
            for (int i = 0; i < 4; ++i) *(half8v *)(base + lds_chunk_off(la[q], 4 * hsel + i)) = e[i];
        }
#pragma unroll
        for (int q = 0; q < CW; ++q) {
            half8v e[4];
            expand_chunk(rw[q], sw[q], e);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *(half8v *)(base + BM * ROW_BYTES + lds_chunk_off(lw[q], 4 * hsel + i)) = e[i];
        }
    };

    float16v acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    load_step(0);
    stage_step(0);
    __syncthreads();

    const int lrow = lane & 31, lhalf = lane >> 5;
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_step(kt + 1);
        const uint8_t *a_base = lds + buf * STAGE;
        const uint8_t *w_base = a_base + BM * ROW_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int c = 2 * kk + lhalf;
            half8v fa[TM], fw[TN];
#pragma unroll
            for (int j = 0; j < TM; ++j) fa[j] = *(const half8v *)(a_base + lds_chunk_off(wm * WM + j * 32 + lrow, c));
#pragma unroll
            for (int i = 0; i < TN; ++i) fw[i] = *(const half8v *)(w_base + lds_chunk_off(wn * WN + i * 32 + lrow, c));
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[i], fa[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) stage_step(buf ^ 1);
        __syncthreads();
    }

    // ---------------------------------------------------------------- epilogue
    const float alpha = (*g.gsA) * (*g.gsW);
    const GemmEpilogue &ep = g.ep;
    uint32_t hmax = 0;      // largest |bf16(H)| pattern seen by this lane
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int64_t m = m0 + wm * WM + j * 32 + lrow;
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int64_t n = n0 + wn * WN + i * 32 + rg * 8 + lhalf * 4;
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    y[e] = acc[i][j][rg * 4 + e] * alpha;
                    if (ep.act == 1) y[e] = gelu_tanh_f32(y[e]);
                }
                if (m < g.M && n < g.N) {      // N % 4 == 0: a run of four is all in or all out
                    if (ep.out_dtype == 0) {
                        float4v o = {y[0], y[1], y[2], y[3]};
                        *(float4v *)((float *)ep.Y + m * ep.ldy + n) = o;
                    } else {
                        uint32_t b0 = f32_to_bf16_rne(y[0]), b1 = f32_to_bf16_rne(y[1]);
                        uint32_t b2 = f32_to_bf16_rne(y[2]), b3 = f32_to_bf16_rne(y[3]);
                        uint2v o = {b0 | (b1 << 16), b2 | (b3 << 16)};
                        if (ep.amax_partial) {
                            hmax = pk_absmax_u16(hmax, o.x);
                            hmax = pk_absmax_u16(hmax, o.y);
                        }
                        *(uint2v *)((uint16_t *)ep.Y + m * ep.ldy + n) = o;
                    }
                }
            }
        }
    }
    if (ep.amax_partial) {
        __shared__ uint32_t wmax[4];
        uint32_t mx = wave_max_u32(pk_hmax_u16(hmax));
        if (lane == 0) wmax[wave] = mx;
        __syncthreads();
        if (tid == 0)
            ep.amax_partial[blockIdx.y * gridDim.x + blockIdx.x] = max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3]));
    }
}

// Any K % 16 == 0 (K not a multiple of 64), any M, N: one output per thread, plain loop.
// Only used for shapes the tiled kernel does not take; not a performance path.
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmArgs g)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= g.M * g.N) return;
    const int64_t m = idx / g.N, n = idx - m * g.N;
    const uint8_t *ca = g.codesA + m * (g.K >> 1), *cw = g.codesW + n * (g.K >> 1);
    const uint8_t *sa = g.scalesA + m * (g.K >> 4), *sw = g.scalesW + n * (g.K >> 4);
    float acc = 0.0f;
    for (int64_t b = 0; b < (g.K >> 4); ++b) {
        float part = 0.0f;
        for (int j = 0; j < 8; ++j) {
            typedef float float2v __attribute__((ext_vector_type(2)));
            float2v x = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4((uint32_t)ca[b * 8 + j], 1.0f, 0);
            float2v y = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4((uint32_t)cw[b * 8 + j], 1.0f, 0);
            part += x.x * y.x + x.y * y.y;     // multiples of 1/4, |sum| <= 576: exact
        }
        acc += part * (e4m3_to_f32(sa[b] & 0x7Fu) * e4m3_to_f32(sw[b] & 0x7Fu));   // scale product: 8 bits, exact
    }
    float y = acc * ((*g.gsA) * (*g.gsW));
    if (g.ep.act == 1) y = gelu_tanh_f32(y);
    if (g.ep.out_dtype == 0) ((float *)g.ep.Y)[m * g.ep.ldy + n] = y;
    else ((uint16_t *)g.ep.Y)[m * g.ep.ldy + n] = (uint16_t)f32_to_bf16_rne(y);
}

template <int BM, int BN>
static hipError_t launch_tiled(const GemmArgs &g, hipStream_t s)
{
    constexpr int smem = 2 * (BM + BN) * ROW_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_f16mfma_kernel<BM, BN>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)((g.N + BN - 1) / BN), (unsigned)((g.M + BM - 1) / BM));
    gemm_f16mfma_kernel<BM, BN><<<grid, 256, smem, s>>>(g);
    return hipGetLastError();
}

static bool use_big_tile(int64_t M, int64_t N)
{
    // 256x256 tiles once they fill the 256 CUs at least ~2 times over; else 128x128
    int64_t big = ((M + 255) / 256) * ((N + 255) / 256);
    return big >= 512;
}

int gemm_workgroups(int64_t M, int64_t N)
{
    if (use_big_tile(M, N)) return (int)(((M + 255) / 256) * ((N + 255) / 256));
    return (int)(((M + 127) / 128) * ((N + 127) / 128));
}

hipError_t launch_gemm(const uint8_t *codesA, const uint8_t *scalesA, const float *gsA,
                       const uint8_t *codesW, const uint8_t *scalesW, const float *gsW, int64_t M,
                       int64_t N, int64_t K, const GemmEpilogue &ep, int *n_wg, hipStream_t s)
{
    GemmArgs g{codesA, scalesA, codesW, scalesW, gsA, gsW, M, N, K, ep};
    if (K % BK != 0 || N % 4 != 0) {
        if (n_wg) *n_wg = 0;
        int64_t total = M * N;
        gemm_generic_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(g);
        return hipGetLastError();
    }
    if (n_wg) *n_wg = gemm_workgroups(M, N);
    if (use_big_tile(M, N)) return launch_tiled<256, 256>(g, s);
    return launch_tiled<128, 128>(g, s);
}

}  // namespace nvfp4
