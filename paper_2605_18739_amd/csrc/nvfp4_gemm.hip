// Block-scaled FP4 GEMM for gfx950 (Sec. 2.2 / 3.1; Appendix "Implementation Details"): the host
// side (launch plan, chunking, dispatch to the tile shapes of nvfp4_gemm_tile.h), the fallback
// kernel for odd shapes, and the down projection of the LoRA side branch.
#include "nvfp4_gemm_tile.h"
#include "nvfp4_gemm_plan.h"

namespace nvfp4 {

// ============================================================================
// Down projection of the LoRA side branch: T [M, 128] = bf16(X A^T), X [M, K] and A [128, K]
// bf16, fp32 accumulation on v_mfma_f32_32x32x16_bf16.  A skinny GEMM: with whole-K tiles
// either few workgroups run or every one of them pulls all of A through its compute unit, and
// a compute unit pulls only ~30-60 GB/s at the latency of one step in flight.  So K is cut:
// workgroup (i, s) multiplies rows 128 i .. 128 i + 127 with K range s of `splits` (64-k steps
// staged in LDS with full-line coalesced loads, one step ahead; 2 x 2 waves of 64 x 64), writes
// an fp32 partial tile to the workspace, and a second small kernel adds the partial tiles in
// split order and rounds to bf16.
// ============================================================================
constexpr int kLdRows = 128;                                      // rows of X per workgroup
__global__ __launch_bounds__(256) void lora_down_partial_kernel(const uint16_t *__restrict__ x, int64_t M,
                                                                int64_t K, int64_t ldx,
                                                                const uint16_t *__restrict__ a, int steps_per_split,
                                                                float *__restrict__ partial, int64_t m_pad)
{
    typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
    constexpr int ROWS = kLdRows + kLoraRank;                     // staged rows: X rows first, then A rows
    constexpr int STAGE = ROWS * ROW_BYTES;                       // 32 KB
    constexpr int CHUNKS = ROWS * 8 / 256;                        // 16-byte chunks per thread and step
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.x * kLdRows;
    const int step0 = blockIdx.y * steps_per_split;
    const int ksteps_all = (int)((K + 63) >> 6);                  // the last step may be partly past K (K % 16 == 0)
    const int nsteps = min(steps_per_split, ksteps_all - step0);
    // this thread's chunks: q = tid + 256 i -> staged row q / 8, chunk q % 8
    const uint16_t *src[CHUNKS];
    int dst[CHUNKS], kc[CHUNKS];
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
        const int q = tid + 256 * i, row = q >> 3, c = q & 7;
        src[i] = row < kLdRows ? x + min(m0 + row, M - 1) * ldx + 8 * c     // rows past the end repeat the last one (never used)
                               : a + (int64_t)(row - kLdRows) * K + 8 * c;
        dst[i] = lds_chunk_off(row, c);
        kc[i] = 8 * c;
    }
    uint4v regs[CHUNKS];
    auto fetch = [&](int step) {
#pragma unroll
        for (int i = 0; i < CHUNKS; ++i) {
            const int64_t k = (int64_t)step * 64 + kc[i];
            regs[i] = k < K ? *(const uint4v *)(src[i] + (int64_t)step * 64) : uint4v{0u, 0u, 0u, 0u};
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CHUNKS; ++i) *(uint4v *)(lds + buf * STAGE + dst[i]) = regs[i];
    };
    float16v acc[2][2];                                           // [column tile][row tile] of this wave's 64 x 64
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][j][r] = 0.0f;
    if (nsteps > 0) {
        fetch(step0);
        stage(0);
    }
    __syncthreads();
    for (int st = 0; st < nsteps; ++st) {
        const int buf = st & 1;
        if (st + 1 < nsteps) fetch(step0 + st + 1);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            uint4v fx[2], fa[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fx[j] = *(const uint4v *)(lds + buf * STAGE + lds_chunk_off(64 * wm + 32 * j + lrow, 2 * kk + lhalf));
#pragma unroll
            for (int c = 0; c < 2; ++c)
                fa[c] = *(const uint4v *)(lds + buf * STAGE + lds_chunk_off(kLdRows + 64 * wn + 32 * c + lrow, 2 * kk + lhalf));
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[c][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8v, fa[c]),
                                                                        __builtin_bit_cast(bf16x8v, fx[j]), acc[c][j], 0, 0, 0);
        }
        if (st + 1 < nsteps) stage(buf ^ 1);         // the other stage was last read before the previous barrier
        __syncthreads();
    }
    // lane = output row, register r = column 8 (r / 4) + 4 lhalf + r % 4 of the 32-column tile
    float *pp = partial + ((int64_t)blockIdx.y * m_pad + m0) * kLoraRank;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row = 64 * wm + 32 * j + lrow;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(float4v *)(pp + (int64_t)row * kLoraRank + 64 * wn + 32 * c + 8 * q + 4 * lhalf) =
                    float4v{acc[c][j][4 * q], acc[c][j][4 * q + 1], acc[c][j][4 * q + 2], acc[c][j][4 * q + 3]};
    }
}

// T = bf16(sum over the splits, in split order)
__global__ __launch_bounds__(256) void lora_down_reduce_kernel(const float *__restrict__ partial, int splits,
                                                               int64_t m_pad, int64_t M, uint16_t *__restrict__ t)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;           // four consecutive columns of one row
    if (i >= M * kLoraRank) return;
    float4v sum = *(const float4v *)(partial + i);
    for (int s = 1; s < splits; ++s) sum += *(const float4v *)(partial + (int64_t)s * m_pad * kLoraRank + i);
    *(uint2v *)(t + i) = uint2v{pack_bf16x2(sum.x, sum.y), pack_bf16x2(sum.z, sum.w)};
}

// ============================================================================
// Shapes the register-dequantizing kernels do not take (K not a multiple of 64, N not a multiple
// of 8): any M, N and any K % 16 == 0.  128 x 128 tiles, 2 x 2 waves of 64 x 64, 64-k steps.  Operands
// are staged through registers: a thread fetches four (row, 16-element block) items per step -- eight
// bytes of codes and one scale byte each -- expands them to f16 (code x block scale is exact in f16)
// and writes 32 bytes to LDS (same swizzle as the kernels above), one step ahead of the MFMAs; rows
// past the end of an operand and blocks past the end of K are staged as zeros.  Outputs are stored
// straight from the accumulator layout with a guard per element.  A fallback for odd shapes, bound by
// its LDS traffic (about a quarter of the main kernels' rate), not the performance path.
// ============================================================================
constexpr int kEdgeTile = 128;
__global__ __launch_bounds__(256) void gemm_edge_kernel(GemmArgs g)
{
    constexpr int ROWS = 2 * kEdgeTile;                           // staged rows: A rows first, then W rows
    constexpr int STAGE = ROWS * ROW_BYTES;                       // 32 KB
    constexpr int ITEMS = ROWS * 4 / 256;                         // (row, block) items per thread and step
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * STAGE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int64_t tiles_n = (g.N + kEdgeTile - 1) / kEdgeTile;
    const int64_t m0 = (int64_t)(blockIdx.x / tiles_n) * kEdgeTile, n0 = (int64_t)(blockIdx.x % tiles_n) * kEdgeTile;
    const int64_t kbytes = g.K >> 1, kblocks = g.K >> 4;
    const int nsteps = (int)((g.K + 63) >> 6);
    // this thread's items: q = tid + 256 i -> staged row q / 4, block q % 4 of the step
    const uint8_t *csrc[ITEMS], *ssrc[ITEMS];
    bool live[ITEMS];
    int dst[ITEMS][2], blk[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int q = tid + 256 * i, row = q >> 2, b = q & 3;
        const bool isA = row < kEdgeTile;
        const int64_t gr = isA ? m0 + row : n0 + (row - kEdgeTile);
        live[i] = gr < (isA ? g.M : g.N);
        const int64_t r = live[i] ? gr : 0;                      // (dead rows point at row 0 and are never read)
        csrc[i] = (isA ? g.codesA : g.codesW) + r * kbytes + 8 * b;
        ssrc[i] = (isA ? g.scalesA : g.scalesW) + r * kblocks + b;
        dst[i][0] = lds_chunk_off(row, 2 * b);
        dst[i][1] = lds_chunk_off(row, 2 * b + 1);
        blk[i] = b;
    }
    uint2v codes[ITEMS];
    uint32_t scale[ITEMS];
    auto fetch = [&](int step) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const bool in = live[i] && (int64_t)step * 4 + blk[i] < kblocks;
            codes[i] = in ? *(const uint2v *)(csrc[i] + (int64_t)step * 32) : uint2v{0u, 0u};
            scale[i] = in ? (uint32_t)ssrc[i][(int64_t)step * 4] & 0x7Fu : 0u;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const _Float16 sc = e4m3_to_f16(scale[i]);
            const half2v p = {sc, sc};
            uint32_t x[8];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t w = h ? codes[i].y : codes[i].x;
                x[4 * h + 0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 0) * p);
                x[4 * h + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 1) * p);
                x[4 * h + 2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 2) * p);
                x[4 * h + 3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 1.0f, 3) * p);
            }
            *(uint4v *)(lds + buf * STAGE + dst[i][0]) = uint4v{x[0], x[1], x[2], x[3]};
            *(uint4v *)(lds + buf * STAGE + dst[i][1]) = uint4v{x[4], x[5], x[6], x[7]};
        }
    };
    float16v acc[2][2];                                           // [column tile][row tile] of this wave's 64 x 64
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][j][r] = 0.0f;
    fetch(0);
    stage(0);
    __syncthreads();
    for (int st = 0; st < nsteps; ++st) {
        const int buf = st & 1;
        if (st + 1 < nsteps) fetch(st + 1);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            uint4v fa[2], fw[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fa[j] = *(const uint4v *)(lds + buf * STAGE + lds_chunk_off(64 * wm + 32 * j + lrow, 2 * kk + lhalf));
#pragma unroll
            for (int c = 0; c < 2; ++c)
                fw[c] = *(const uint4v *)(lds + buf * STAGE + lds_chunk_off(kEdgeTile + 64 * wn + 32 * c + lrow, 2 * kk + lhalf));
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[c][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8v, fw[c]),
                                                                       __builtin_bit_cast(half8v, fa[j]), acc[c][j], 0, 0, 0);
        }
        if (st + 1 < nsteps) stage(buf ^ 1);         // the other stage was last read before the previous barrier
        __syncthreads();
    }
    // lane = output row, register r = column 8 (r / 4) + 4 lhalf + r % 4 of the 32-column tile
    const float alpha = (*g.gsA) * (*g.gsW);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int64_t m = m0 + 64 * wm + 32 * j + lrow;
        if (m >= g.M) continue;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t n = n0 + 64 * wn + 32 * c + 8 * q + 4 * lhalf;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (n + e >= g.N) continue;
                    float y = acc[c][j][4 * q + e] * alpha;
                    if (g.ep.act == 1) y = gelu_tanh_f32(y);
                    if (g.ep.out_dtype == 0) ((float *)g.ep.Y)[m * g.ep.ldy + n + e] = y;
                    else ((uint16_t *)g.ep.Y)[m * g.ep.ldy + n + e] = (uint16_t)f32_to_bf16_rne(y);
                }
            }
    }
}


bool gemm_is_tiled(int64_t M, int64_t N, int64_t K) { return tiled_ok(M, N, K); }

// "BMxBN:workgroups" per launch, separated by spaces ("generic" for the untiled fallback)
int gemm_plan_text(int64_t M, int64_t N, int64_t K, char *text, size_t text_bytes)
{
    if (!tiled_ok(M, N, K)) {
        snprintf(text, text_bytes, "generic");
        return 1;
    }
    size_t used = 0;
    int launches = 0;
    bool fits = true;
    for_each_chunk(M, N, K, false, [&](int64_t, int64_t, int64_t, int64_t, const LaunchPlan &p) {
        for (int i = 0; i < p.n && fits; ++i) {
            const TileShape &t = kShapes[p.part[i].kind];
            const int w = snprintf(text + used, used < text_bytes ? text_bytes - used : 0, "%s%dx%d:%lld",
                                   launches ? " " : "", t.bm, t.bn, (long long)p.part[i].tiles);
            if (w < 0 || used + (size_t)w >= text_bytes) fits = false;
            else {
                used += (size_t)w;
                ++launches;
            }
        }
    });
    return fits ? launches : -1;
}

int gemm_workgroups(int64_t M, int64_t N, int64_t K)
{
    int64_t n = 0;
    for_each_chunk(M, N, K, false, [&](int64_t, int64_t, int64_t, int64_t, const LaunchPlan &p) {
        for (int i = 0; i < p.n; ++i) n += p.part[i].tiles;
    });
    return (int)n;
}

static hipError_t launch_kind(TileKind kind, int epi, const GemmArgs &g, int64_t tiles, hipStream_t s)
{
    switch (kind) {
    case kTile256x256: return launch_tile_256x256(epi, g, tiles, s);
    case kTile256x192: return launch_tile_256x192(epi, g, tiles, s);
    case kTile64: return launch_tile_64x64(epi, g, tiles, s);        // (no LoRA phase: planned with the 256-row tiles only)
    default: return launch_tile_128x128(epi, g, tiles, s);
    }
}

hipError_t launch_gemm(const uint8_t *codesA, const uint8_t *scalesA, const float *gsA,
                       const uint8_t *codesW, const uint8_t *scalesW, const float *gsW, int64_t M,
                       int64_t N, int64_t K, const GemmEpilogue &ep, int *n_wg, hipStream_t s,
                       const LoraBranch &lora)
{
    GemmArgs g{codesA, scalesA, codesW, scalesW, gsA, gsW, M, N, K, ep, 0, N, 0, lora.t, lora.b, lora.scale};
    const bool with_lora = lora.t != nullptr;
    if (!tiled_ok(M, N, K)) {
        if (with_lora) return hipErrorInvalidValue;      // the untiled fallback has no LoRA phase (callers check gemm_is_tiled)
        if (n_wg) *n_wg = 0;
        const int64_t tiles = ((M + kEdgeTile - 1) / kEdgeTile) * ((N + kEdgeTile - 1) / kEdgeTile);
        gemm_edge_kernel<<<(unsigned)tiles, 256, 0, s>>>(g);
        return hipGetLastError();
    }
    // (the tiled fp32 output never carries an activation: nvfp4_gemm has none and the fused call emits bf16)
    const int out_kind = ep.q_scale ? kEpiQuant : (ep.out_dtype != 0 ? kEpiBF16 : kEpiF32);
    const int epi = out_kind | ((ep.act == 1 && out_kind != kEpiF32) ? kEpiGelu : 0);
    const int64_t kbytes = K >> 1, kblocks = K >> 4;
    const int64_t ysize = ep.out_dtype == 0 ? 4 : 2;
    int wg_total = 0;
    hipError_t err = hipSuccess;
    for_each_chunk(M, N, K, with_lora, [&](int64_t cm, int64_t, int64_t cn, int64_t, const LaunchPlan &plan) {
        for (int i = 0; i < plan.n && err == hipSuccess; ++i) {
            const SubLaunch &p = plan.part[i];
            const int64_t m_lo = cm + p.m_lo, n_lo = cn + p.n_lo;     // the sub-rectangle [m_lo, ..) x [n_lo, ..) as a problem of its own
            GemmArgs a = g;
            a.codesA = codesA + m_lo * kbytes;
            a.scalesA = scalesA + m_lo * kblocks;
            a.codesW = codesW + n_lo * kbytes;
            a.scalesW = scalesW + n_lo * kblocks;
            a.M = p.m_hi - p.m_lo;
            a.N = p.n_hi - p.n_lo;
            if (ep.Y) a.ep.Y = (uint8_t *)ep.Y + (m_lo * ep.ldy + n_lo) * ysize;
            if (ep.q_codes) {
                a.ep.q_codes = ep.q_codes + m_lo * (N >> 1) + (n_lo >> 1);
                a.ep.q_scales = ep.q_scales + m_lo * (N >> 4) + (n_lo >> 4);
            }
            a.q_pitch = N;
            a.partial_base = wg_total;
            if (with_lora) {
                a.lora_t = lora.t + m_lo * kLoraRank;
                a.lora_b = lora.b + n_lo * kLoraRank;
            }
            err = launch_kind(p.kind, epi | (with_lora ? kEpiLora : 0), a, p.tiles, s);
            wg_total += (int)p.tiles;
        }
    });
    if (err != hipSuccess) return err;
    if (n_wg) *n_wg = wg_total;
    return hipSuccess;
}

// K is cut into `splits` ranges of whole 64-k steps so that about one workgroup per compute unit runs
static void lora_down_plan(int64_t M, int64_t K, int *splits, int *steps_per_split, int64_t *m_pad)
{
    const int64_t row_tiles = (M + kLdRows - 1) / kLdRows;
    const int ksteps = (int)((K + 63) >> 6);
    int want = (int)std::max<int64_t>(1, std::min<int64_t>(16, kCUs / row_tiles));
    *steps_per_split = (ksteps + want - 1) / want;
    *splits = (ksteps + *steps_per_split - 1) / *steps_per_split;
    *m_pad = row_tiles * kLdRows;
}

size_t lora_down_workspace_bytes(int64_t M, int64_t K)
{
    int splits, sps;
    int64_t m_pad;
    lora_down_plan(M, K, &splits, &sps, &m_pad);
    return (size_t)splits * (size_t)m_pad * kLoraRank * sizeof(float);
}

hipError_t launch_lora_down(const uint16_t *x, int64_t M, int64_t K, int64_t ldx, const uint16_t *a,
                            uint16_t *t, float *workspace, hipStream_t s)
{
    int splits, sps;
    int64_t m_pad;
    lora_down_plan(M, K, &splits, &sps, &m_pad);
    dim3 grid((unsigned)(m_pad / kLdRows), (unsigned)splits);
    lora_down_partial_kernel<<<grid, 256, 2 * (kLdRows + kLoraRank) * ROW_BYTES, s>>>(x, M, K, ldx, a, sps, workspace, m_pad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    lora_down_reduce_kernel<<<(unsigned)((M * kLoraRank / 4 + 255) / 256), 256, 0, s>>>(workspace, splits, m_pad, M, t);
    return hipGetLastError();
}

}  // namespace nvfp4
