// NVFP4 quantizer and KV-cache kernels for gfx950 (Sec. 2.2, Eq. 2; Appendix
// on scale search, Eq. 12 with target 6; Sec. 3.2, Eq. 5).  All of them are
// streaming kernels bound by HBM: 2 B read + 0.5625 B written per element
// (quantize), 0.5625 B read + 2 B written (KV reconstruction).
#include "nvfp4_device.h"

#include <algorithm>
#include "nvfp4_kernels.h"

namespace nvfp4 {

// blocks in flight per lane and the largest grids of the streaming kernels (measured choices)
constexpr int kQuantUnroll = 2, kDequantUnroll = 4, kQuantMaxGrid = 16384, kDequantMaxGrid = 8192;

// --------------------------------------------------------------------------
// Pass 1: per-workgroup partial amax (largest |bf16| bit pattern).
// x is [R, C] with row stride ld; C % 8 == 0.  partial[blockIdx.x] is written
// by every workgroup (no atomics, nothing to clear).
// --------------------------------------------------------------------------
// 1024 threads per workgroup: one workgroup per compute unit keeps sixteen waves of loads in
// flight and leaves at most 256 partial maxima for every pass-2 workgroup to reduce again.
constexpr int kAmaxThreads = 1024, kAmaxGrid = 256;
// STREAM: the tensor is larger than the 256 MB Infinity Cache, so nothing pass 2 reads would still be there:
// the loads bypass the caches (on the 505 MB gradient the transposed quantizer gains 5 %); smaller tensors are read
// with ordinary loads, and pass 2 finds them in the cache.
template <bool CONTIG, bool STREAM>
__global__ __launch_bounds__(kAmaxThreads) void amax_partial_kernel(const uint16_t *__restrict__ x, int64_t R,
                                                                    int64_t C, int64_t ld,
                                                                    uint32_t *__restrict__ partial)
{
    __shared__ uint32_t wave_max[kAmaxThreads / 64];
    const int64_t vec_per_row = C >> 3;
    const int64_t nvec = R * vec_per_row;
    // a workgroup reads one contiguous stretch of the tensor, four vectors per lane in flight (contiguous stretches
    // per workgroup stream about a fifth faster than a grid-wide stride)
    const int64_t per = (nvec + gridDim.x - 1) / gridDim.x, begin = per * blockIdx.x, end = min(nvec, begin + per);
    auto offset_of = [&](int64_t i) {
        if (CONTIG) return i << 3;
        const int64_t r = i / vec_per_row;
        return r * ld + ((i - r * vec_per_row) << 3);
    };
    uint32_t acc = 0;
    auto take = [&](uint4v v) {
        acc = pk_absmax_u16(acc, v.x);
        acc = pk_absmax_u16(acc, v.y);
        acc = pk_absmax_u16(acc, v.z);
        acc = pk_absmax_u16(acc, v.w);
    };
    auto fetch = [&](int64_t k) {
        const uint4v *p = (const uint4v *)(x + offset_of(k));
        return STREAM ? __builtin_nontemporal_load(p) : *p;
    };
    int64_t i = begin + threadIdx.x;
    for (; i + 3 * kAmaxThreads < end; i += 4 * kAmaxThreads) {
        const uint4v a = fetch(i), b = fetch(i + kAmaxThreads), c = fetch(i + 2 * kAmaxThreads), d = fetch(i + 3 * kAmaxThreads);
        take(a);
        take(b);
        take(c);
        take(d);
    }
    for (; i < end; i += kAmaxThreads) take(fetch(i));
    uint32_t m = wave_max_u32(pk_hmax_u16(acc));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t all = 0;
        for (int w = 0; w < kAmaxThreads / 64; ++w) all = max(all, wave_max[w]);
        partial[blockIdx.x] = all;
    }
}

// --------------------------------------------------------------------------
// Pass 1 of the smoothed key cache (Sec. 3.2, Eq. 6): per row of d features (one token, one
// head) the mean over the features, rounded to bf16 and stored, and the partial amax of the
// smoothed values RN_bf16(x - mean).  One lane per 16-element block; the d/16 lanes of a row
// are neighbours (d/16 a power of two up to 64) and add their fp64 partial sums by shuffles.
// --------------------------------------------------------------------------
__global__ __launch_bounds__(kAmaxThreads) void amax_smooth_kernel(const uint16_t *__restrict__ x, int64_t rows,
                                                          int log2_nb_row, uint16_t *__restrict__ mean_out,
                                                          uint32_t *__restrict__ partial)
{
    __shared__ uint32_t wave_max[kAmaxThreads / 64];
    const int nb_row = 1 << log2_nb_row;                        // blocks per row, d = 16 nb_row
    const double inv_d = 1.0 / (double)(16 << log2_nb_row);    // a power of two: the quotient below is exact
    const int64_t nblk = rows << log2_nb_row;
    const int64_t stride = (int64_t)gridDim.x * kAmaxThreads;  // a multiple of nb_row
    uint32_t acc = 0;
    // the trip count is the same for all lanes of a wave up to the tail, where lanes past the end
    // contribute zeros to the shuffles (their rows do not exist)
    for (int64_t g0 = (int64_t)blockIdx.x * kAmaxThreads; g0 < nblk; g0 += stride) {
        const int64_t g = g0 + threadIdx.x;
        const bool live = g < nblk;
        uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (live) {
            const uint4v *p = (const uint4v *)(x + (g << 4));
            const uint4v v0 = p[0], v1 = p[1];                 // ordinary loads: pass 2 re-reads x
            w[0] = v0.x; w[1] = v0.y; w[2] = v0.z; w[3] = v0.w;
            w[4] = v1.x; w[5] = v1.y; w[6] = v1.z; w[7] = v1.w;
        }
        double sum = 0.0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            sum += (double)bf16lo_to_f32(w[i]);
            sum += (double)bf16hi_to_f32(w[i]);
        }
        for (int m = 1; m < nb_row; m <<= 1) sum += __shfl_xor(sum, m, 64);
        const uint32_t mean_bits = bf16_rne_signed_from_f64(sum * inv_d);
        if (live) {
            if ((g & (nb_row - 1)) == 0) mean_out[g >> log2_nb_row] = (uint16_t)mean_bits;
            smooth_block16(w, __uint_as_float(mean_bits << 16));
#pragma unroll
            for (int i = 0; i < 8; ++i) acc = pk_absmax_u16(acc, w[i]);
        }
    }
    uint32_t m = wave_max_u32(pk_hmax_u16(acc));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t all = 0;
        for (int w = 0; w < kAmaxThreads / 64; ++w) all = max(all, wave_max[w]);
        partial[blockIdx.x] = all;
    }
}

// Every workgroup of a pass-2 kernel reduces the partials again (a few KB out
// of L2) and so knows the tensor scale without a third launch.
__device__ __forceinline__ float resolve_global_scale(const float *gs_in, const uint32_t *partial,
                                                      int n_partial, float *gs_out, uint32_t *lds4)
{
    float sg;
    if (gs_in) {
        sg = *gs_in;
    } else {
        uint32_t acc = 0;
        for (int i = threadIdx.x; i < n_partial; i += blockDim.x) acc = max(acc, partial[i]);
        uint32_t m = wave_max_u32(acc);
        if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = m;
        __syncthreads();
        m = 0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) m = max(m, lds4[w]);
        sg = global_scale_from_amax_bits(m);
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *gs_out = sg;
    return sg;
}

// The tensor scale alone, from partial maxima that something else produced (a GEMM epilogue, an amax pass): one
// workgroup, one float.  What a later quantizer call takes as its given scale.
__global__ __launch_bounds__(256) void scale_from_partials_kernel(const uint32_t *__restrict__ partial, int n_partial,
                                                                  float *__restrict__ gs_out)
{
    __shared__ uint32_t lds4[4];
    (void)resolve_global_scale(nullptr, partial, n_partial, gs_out, lds4);
}

// --------------------------------------------------------------------------
// Pass 2, blocks along the contiguous axis: one lane per 16-element block
// (two 128-bit loads, one 64-bit code store, one scale byte).
// SEARCH: the Four-over-Six scale search of Eq. 12-13 instead of the plain max -> 6 rule.
// SMOOTH: the row means of Eq. 6 (row_mean, one bf16 per row) are removed first.
// slab_heads > 0: the rows are (token, head) pairs of a [T, H, d] tensor and the output is
// regrouped into H / slab_heads slabs of slab_heads heads each, [slab][token][head in slab]
// (what the pre-attention all-to-all of sequence-parallel inference sends to each peer).
// --------------------------------------------------------------------------
template <bool CONTIG, bool SEARCH = false, bool SMOOTH = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4)))   // at most 128 registers: four waves per SIMD
void quantize_rows_kernel(const uint16_t *__restrict__ x, int64_t R,
                                                            int64_t C, int64_t ld,
                                                            const float *__restrict__ gs_in,
                                                            const uint32_t *__restrict__ partial,
                                                            int n_partial, uint8_t *__restrict__ codes,
                                                            uint8_t *__restrict__ scales,
                                                            float *__restrict__ gs_out,
                                                            const uint16_t *__restrict__ row_mean = nullptr,
                                                            int heads = 0, int slab_heads = 0, int row_shift = 0)
{
    __shared__ uint32_t lds4[4];
    const int64_t nb_row = C >> 4;
    const int64_t nblk = R * nb_row;
    const int64_t stride = (int64_t)gridDim.x * 256;
    constexpr int U = kQuantUnroll;              // blocks in flight per lane
    uint4v v0[U], v1[U];
    auto fetch = [&](int64_t g0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t g = g0 + u * stride;
            if (g < nblk) {
                int64_t off;
                if (CONTIG) off = g << 4;
                else {
                    int64_t r = g / nb_row;
                    off = r * ld + ((g - r * nb_row) << 4);
                }
                const uint4v *p = (const uint4v *)(x + off);
                v0[u] = __builtin_nontemporal_load(p);
                v1[u] = __builtin_nontemporal_load(p + 1);
            }
        }
    };
    // the first loads do not depend on the tensor scale: they are in flight while the workgroup
    // reduces the partial maxima (not in the scale-search variants: they are bound by VALU work,
    // and the registers held across the reduction would cost them a wave of occupancy)
    const int64_t first = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if constexpr (!SEARCH) fetch(first);
    const float sg = resolve_global_scale(gs_in, partial, n_partial, gs_out, lds4);
    if constexpr (SEARCH) fetch(first);
    const float shift = range_shift(sg), sgq = sg * shift;      // (1 and s_g unless the tensor scale is out of the fp32-safe range)
    const float inv_6sg = 1.0f / (6.0f * sgq);
    const float inv_4sg = 1.0f / (4.0f * sgq);
    for (int64_t g0 = first; g0 < nblk; g0 += stride * U) {
        if (g0 != first) fetch(g0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t g = g0 + u * stride;
            if (g < nblk) {
                uint32_t w[8] = {v0[u].x, v0[u].y, v0[u].z, v0[u].w, v1[u].x, v1[u].y, v1[u].z, v1[u].w};
                // SMOOTH: C / 16 = 1 << row_shift blocks per row
                if constexpr (SMOOTH) smooth_block16(w, __uint_as_float((uint32_t)row_mean[g >> row_shift] << 16));
                if (__builtin_expect(shift != 1.0f, 0)) rescale_block16(w, shift);
                uint32_t sbyte, c0, c1;
                if (SEARCH && __builtin_expect(shift == 1.0f, 1)) {
                    // the straight-line form: the candidates compared on one bracket end, the winner settled
                    quantize_block16_4over6_inline(w, sgq, inv_6sg, inv_4sg, sbyte, c0, c1);
                } else {
                    uint32_t acc = 0;
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc = pk_absmax_u16(acc, w[i]);
                    const float bmax = __uint_as_float(pk_hmax_u16(acc) << 16);
                    if constexpr (SEARCH) {
                        encode_block16_4over6(w, bmax, sgq, inv_6sg, inv_4sg, sbyte, c0, c1);
                    } else {
                        sbyte = block_scale_exact(bmax, sgq, inv_6sg);
                        encode_block16(w, e4m3_to_f32(sbyte), sgq, c0, c1);
                    }
                }
                uint2v cc = {c0, c1};
                int64_t go = g;                       // output block index
                if (slab_heads > 0) {
                    const int64_t row = g / nb_row, b = g - row * nb_row;
                    const int64_t t = row / heads, h = row - t * heads;
                    const int64_t slab = h / slab_heads, hl = h - slab * slab_heads;
                    go = ((slab * (R / heads) + t) * slab_heads + hl) * nb_row + b;
                }
                __builtin_nontemporal_store(cc, (uint2v *)(codes + (go << 3)));
                scales[go] = (uint8_t)sbyte;
            }
        }
    }
}

// --------------------------------------------------------------------------
// Pass 2, blocks along the ROW axis (the operand re-quantized along its other
// axis for dgrad / wgrad).  x [R, C] -> codes [C, R/2], scales [C, R/16].
// A workgroup takes a tile of 128 rows x 256 columns: thread (rb, cg) loads 16
// rows x 8 columns (sixteen 128-bit loads, coalesced along C), owns 8 whole
// blocks (one per column), and the packed results go through LDS so that every
// output row is written in 64-byte runs.
// --------------------------------------------------------------------------
constexpr int kTR = 128, kTC = 256;

// a thread's 16 rows x 8 columns -> column j as eight packed pairs (rows 2i in the low half)
__device__ __forceinline__ void column_of(const uint4v (&v)[16], int j, uint32_t (&w)[8])
{
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t a = v[2 * i][j >> 1], b = v[2 * i + 1][j >> 1];
        w[i] = (j & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
    }
}

// the same for a column index known only at run time (the rare path of the Hadamard kernels)
__device__ __forceinline__ void column_of_dyn(const uint4v (&v)[16], int j, uint32_t (&w)[8])
{
    const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;     // high halves / low halves of (a, b)
    const bool c1 = (j & 2) != 0, c2 = (j & 4) != 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint4v va = v[2 * i], vb = v[2 * i + 1];
        const uint32_t a = c2 ? (c1 ? va.w : va.z) : (c1 ? va.y : va.x), b = c2 ? (c1 ? vb.w : vb.z) : (c1 ? vb.y : vb.x);
        w[i] = __builtin_amdgcn_perm(b, a, sel);
    }
}

// ---- the groups of the Hadamard kernels that the fp32 transform is not exact for -----------------------
// About one group in a hundred of Gaussian data.  They are not redone where the sweep over a tile finds them, which
// would hold up the whole wave for the few lanes that have one and keep the loaded tile in registers next to the
// slower forms' own: they go into a list of the workgroup (eight words and a word that says where the group belongs),
// and after the sweep the list is worked off with one group per lane, so that a tile's twenty-odd such groups cost
// one pass of one wave.  When the list is full the lane notes the column (a bit of `noted`) instead; noted columns
// are read again from memory and listed in further rounds (data that spans many binades within most groups: slow,
// and as exact).
constexpr int kRhtQueue = 512;       // groups per round
struct RhtList {
    uint32_t q[kRhtQueue * 9];
    uint32_t n;
};
__device__ __forceinline__ bool rht_list(RhtList &l, const uint32_t (&raw)[8], uint32_t place)
{
    const uint32_t slot = atomicAdd(&l.n, 1u);
    if (slot >= (uint32_t)kRhtQueue) return false;
#pragma unroll
    for (int i = 0; i < 8; ++i) l.q[slot * 9 + i] = raw[i];
    l.q[slot * 9 + 8] = place;
    return true;
}
// Every lane of the workgroup calls this after its sweep (l.n was zeroed, behind a barrier, before it).  take(w,
// place) receives each listed group, transformed.  (r, c): the lane's first row and column, for the noted columns.
template <class Take>
__device__ __forceinline__ void rht_work_off(RhtList &l, uint32_t noted, uint32_t place, const RhtRows &h, uint32_t sign_mask,
                                             const uint16_t *__restrict__ x, int64_t r, int64_t c, int64_t ld, Take take)
{
    for (;;) {
        __syncthreads();
        const uint32_t n = min(l.n, (uint32_t)kRhtQueue);
        for (uint32_t e0 = threadIdx.x & ~63u; e0 < n; e0 += 256u) {      // (the same for the whole wave: matrix instructions inside)
            const uint32_t e = e0 + (threadIdx.x & 63u);
            const bool mine = e < n;
            uint32_t w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = mine ? l.q[e * 9 + i] : 0u;
            const uint32_t where = mine ? l.q[e * 9 + 8] : 0u;
            const bool settled = rht_block16_mfma_split(w, h);
            if (__builtin_expect(mine & !settled, 0)) rht_block16(w, sign_mask);
            if (mine) take(w, where);
        }
        if (!__syncthreads_or(noted != 0u)) break;
        if (threadIdx.x == 0) l.n = 0u;
        __syncthreads();
        if (noted != 0u) {                 // (only lanes inside the tensor note columns)
            const int j = __builtin_ctz(noted);
            uint32_t raw[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                raw[i] = (uint32_t)x[(r + 2 * i) * ld + c + j] | ((uint32_t)x[(r + 2 * i + 1) * ld + c + j] << 16);
            if (rht_list(l, raw, place + (uint32_t)j)) noted &= noted - 1u;
        }
    }
}

// Pass 1 for a weight-gradient operand that is Hadamard-transformed along its rows before it is
// quantized (Sec. 2.2): partial amax of the TRANSFORMED values, same tiles and thread layout as
// the pass-2 kernel below, tiles dealt over at most kMaxPartials workgroups.
template <bool STREAM>      // as in amax_partial_kernel: tensors beyond the Infinity Cache are read past the caches (-8 % on the 505 MB gradient)
__global__ __launch_bounds__(256, 4) void amax_rht_kernel(const uint16_t *__restrict__ x, int64_t R, int64_t C,
                                                       int64_t ld, uint32_t sign_mask,
                                                       uint32_t *__restrict__ partial, uint8_t *__restrict__ inexact)
{
    __shared__ uint32_t wave_max[4];
    __shared__ RhtList list;
    const int cg = threadIdx.x & 31, rb = threadIdx.x >> 5;
    const int64_t tiles_x = (C + kTC - 1) / kTC, tiles_y = (R + kTR - 1) / kTR;
    const RhtRows h = rht_rows(sign_mask, threadIdx.x);
    uint32_t acc = 0;
    float accf = 0.0f;
    for (int64_t tile = blockIdx.x; tile < tiles_x * tiles_y; tile += gridDim.x) {      // (as many turns for every lane)
        const int64_t r = (tile / tiles_x) * kTR + rb * 16, c = (tile % tiles_x) * kTC + cg * 8;
        if (threadIdx.x == 0) list.n = 0u;
        __syncthreads();
        // lanes outside the tensor carry zeros through the same instructions (the matrix instructions below are
        // issued for whole waves); zeros transform to zeros and change no maximum
        uint4v v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = uint4v{0u, 0u, 0u, 0u};
        if (r < R && c < C) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint4v *p = (const uint4v *)(x + (r + i) * ld + c);
                v[i] = STREAM ? __builtin_nontemporal_load(p) : *p;
            }
        }
        // the fp32 transform for every group; the few groups it is not exact for are listed and redone after the sweep
        uint32_t inex = 0, noted = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t w[8];
            column_of(v, j, w);
            const bool exact = rht_fp32_is_exact(w);
            float y[16];
            rht_block16_mfma(w, h, y);
            float m = absmax16_tree(y);            // (rounding to bf16 is monotone: the maximum is rounded once, at the end)
            // one column at a time, its sixteen sums folded into one number before the next starts: eight columns
            // in flight would not fit the registers
            asm volatile("" : "+v"(m));
            __builtin_amdgcn_sched_barrier(0);
            accf = exact ? fmaxf(accf, m) : accf;
            if (__builtin_expect(!exact, 0)) {
                inex |= 1u << j;
                if (!rht_list(list, w, 0u)) noted |= 1u << j;
            }
        }
        // which of the lane's eight groups were inexact: pass 2 (same tiles, same lanes) need not test them again
        if (inexact) inexact[tile * 256 + threadIdx.x] = (uint8_t)inex;
        rht_work_off(list, noted, 0u, h, sign_mask, x, r, c, ld, [&](const uint32_t (&w)[8], uint32_t) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc = pk_absmax_u16(acc, w[i]);
        });
    }
    uint32_t m = wave_max_u32(max(pk_hmax_u16(acc), pack_bf16x2(accf, 0.0f) & 0xFFFFu));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0)
        partial[blockIdx.x] = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
}

// RHT: every 16-row group of a column goes through the random Hadamard transform first.
template <bool RHT = false>
__global__ __launch_bounds__(256, 3) void quantize_cols_kernel(const uint16_t *__restrict__ x, int64_t R,
                                                            int64_t C, int64_t ld,
                                                            const float *__restrict__ gs_in,
                                                            const uint32_t *__restrict__ partial,
                                                            int n_partial, uint8_t *__restrict__ codes,
                                                            uint8_t *__restrict__ scales,
                                                            float *__restrict__ gs_out,
                                                            uint32_t sign_mask = 0,
                                                            const uint8_t *__restrict__ inexact = nullptr)
{
    __shared__ uint32_t lds4[4];
    __shared__ uint2v lds_codes[kTC][kTR / 16 + 1];     // [column][row block], padded
    __shared__ uint8_t lds_scales[kTC][kTR / 16];
    __shared__ uint32_t list_words[RHT ? sizeof(RhtList) / 4 : 1];       // RHT: the groups left for after the sweep
    const int cg = threadIdx.x & 31, rb = threadIdx.x >> 5;
    const int64_t r0 = (int64_t)blockIdx.y * kTR, c0 = (int64_t)blockIdx.x * kTC;
    const int64_t r = r0 + rb * 16, c = c0 + cg * 8;
    const bool live = (r < R) && (c < C);      // R % 16 == 0 and C % 8 == 0: whole blocks only
    // the loads do not depend on the tensor scale: they are in flight while the partial maxima are reduced
    uint4v v[16];
    if constexpr (RHT) {                       // (lanes outside the tensor carry zeros through the transform)
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = uint4v{0u, 0u, 0u, 0u};
    }
    if (live) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            v[i] = __builtin_nontemporal_load((const uint4v *)(x + (r + i) * ld + c));
    }
    const float sg = resolve_global_scale(gs_in, partial, n_partial, gs_out, lds4);
    const float shift = range_shift(sg), sgq = sg * shift;      // (1 and s_g unless the tensor scale is out of the fp32-safe range)
    const float inv_6sg = 1.0f / (6.0f * sgq);
    auto group_max = [](const uint32_t (&w)[8]) {
        uint32_t acc = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = pk_absmax_u16(acc, w[i]);
        return __uint_as_float(pk_hmax_u16(acc) << 16);
    };
    // (transformed) group and its largest magnitude -> codes and scale of column c0 + col
    auto encode_group = [&](uint32_t (&w)[8], float bmax, int col, int rbx) {
        if (__builtin_expect(shift != 1.0f, 0)) {
            rescale_block16(w, shift);
            bmax = group_max(w);
        }
        uint32_t sbyte = block_scale_exact(bmax, sgq, inv_6sg);
        uint32_t k0, k1;
        encode_block16(w, e4m3_to_f32(sbyte), sgq, k0, k1);
        uint2v cc = {k0, k1};
        lds_codes[col][rbx] = cc;
        lds_scales[col][rbx] = (uint8_t)sbyte;
    };
    if constexpr (RHT) {
        // Every lane of the wave runs the transform (matrix instructions are issued for whole waves; lanes outside
        // the tensor encode zeros into staging rows that are not stored).
        RhtList &list = *reinterpret_cast<RhtList *>(list_words);
        const RhtRows h = rht_rows(sign_mask, threadIdx.x);
        if (threadIdx.x == 0) list.n = 0u;
        __syncthreads();
        // (pass 1, when it ran and had room for them, left the outcome of the exactness test of this lane's groups)
        const uint32_t known = inexact ? inexact[((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x] : 0u;
        const uint32_t place = (uint32_t)(cg * 8) | ((uint32_t)rb << 16);
        uint32_t noted = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {      // column c + j: element j of every loaded vector
            uint32_t raw[8], w[8];
            column_of(v, j, raw);
            const bool exact = inexact ? ((known >> j) & 1u) == 0u : rht_fp32_is_exact(raw);
            float y[16];
            rht_block16_mfma(raw, h, y);
            pack16(y, w);
            // (rounding to bf16 is monotone: the largest of the rounded values is the rounded largest value.  A group
            //  that is listed is encoded here all the same, and again, into the same place, after the sweep.)
            encode_group(w, __uint_as_float(pack_bf16x2(absmax16_tree(y), 0.0f) << 16), cg * 8 + j, rb);
            if (__builtin_expect(!exact, 0))
                if (!rht_list(list, raw, place + (uint32_t)j)) noted |= 1u << j;
        }
        rht_work_off(list, noted, place, h, sign_mask, x, r, c, ld, [&](uint32_t (&w)[8], uint32_t where) {
            encode_group(w, group_max(w), (int)(where & 0xFFFFu), (int)(where >> 16));
        });
    } else if (live) {
        if (__builtin_expect(shift == 1.0f, 1)) {          // two columns side by side (see quantize_pair16)
#pragma unroll
            for (int j = 0; j < 8; j += 2) {               // columns c + j, c + j + 1: elements j, j + 1 of every loaded vector
                uint32_t wa[8], wb[8], sa, a0, a1, sb, b0, b1;
                column_of(v, j, wa);
                column_of(v, j + 1, wb);
                quantize_pair16(wa, wb, sg, inv_6sg, sa, a0, a1, sb, b0, b1);
                lds_codes[cg * 8 + j][rb] = uint2v{a0, a1};
                lds_scales[cg * 8 + j][rb] = (uint8_t)sa;
                lds_codes[cg * 8 + j + 1][rb] = uint2v{b0, b1};
                lds_scales[cg * 8 + j + 1][rb] = (uint8_t)sb;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t w[8];
                column_of(v, j, w);
                encode_group(w, group_max(w), cg * 8 + j, rb);
            }
        }
    }
    __syncthreads();
    // cooperative store: per column 8 row blocks = 64 B of codes + 8 B of scales
    const int64_t rows_here = min((int64_t)kTR, R - r0);          // multiple of 16
    const int nrb = (int)(rows_here >> 4);
    for (int t = threadIdx.x; t < kTC * (kTR / 16); t += 256) {
        int col = t >> 3, b = t & 7;
        if (c0 + col < C && b < nrb) {
            *(uint2v *)(codes + (c0 + col) * (R >> 1) + (r0 >> 1) + b * 8) = lds_codes[col][b];
            scales[(c0 + col) * (R >> 4) + (r0 >> 4) + b] = lds_scales[col][b];
        }
    }
}

// --------------------------------------------------------------------------
// 2-D block scaling for weights (Sec. 2.2, the training recipe): one scale per 16x16 tile,
// so that the operand [R, C] (blocks along C) and the operand [C, R] (blocks along R) hold
// the same quantized values.  A lane owns a whole tile (sixteen 32-byte row loads, 128
// registers), a workgroup a square of 16 x 16 tiles; lane = 16 tj + ti, so the transposed
// output leaves in 128-byte runs (ti fastest) and the plain one in 32-byte runs that
// neighbouring waves complete in the cache.
// --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void quantize_tiles_kernel(const uint16_t *__restrict__ x, int64_t R,
                                                             int64_t C, int64_t ld,
                                                             const float *__restrict__ gs_in,
                                                             const uint32_t *__restrict__ partial,
                                                             int n_partial, uint8_t *__restrict__ codes,
                                                             uint8_t *__restrict__ scales,
                                                             uint8_t *__restrict__ codes_t,
                                                             uint8_t *__restrict__ scales_t,
                                                             float *__restrict__ gs_out,
                                                             float *__restrict__ gs_out_t)
{
    __shared__ uint32_t lds4[4];
    const int64_t I = (int64_t)blockIdx.y * 16 + (threadIdx.x & 15), J = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int64_t tr = R >> 4, tc = C >> 4;
    const bool live = I < tr && J < tc;
    // the tile is loaded (and its maximum taken) while the partial maxima of the tensor are reduced
    uint32_t w[16][8];
    uint32_t acc = 0;
    if (live) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint4v *p = (const uint4v *)(x + (16 * I + i) * ld + 16 * J);
            const uint4v v0 = __builtin_nontemporal_load(p), v1 = __builtin_nontemporal_load(p + 1);
            w[i][0] = v0.x; w[i][1] = v0.y; w[i][2] = v0.z; w[i][3] = v0.w;
            w[i][4] = v1.x; w[i][5] = v1.y; w[i][6] = v1.z; w[i][7] = v1.w;
        }
    }
    const float sg = resolve_global_scale(gs_in, partial, n_partial, gs_out, lds4);
    if (gs_out_t && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *gs_out_t = sg;
    const float shift = range_shift(sg), sgq = sg * shift;      // (1 and s_g unless the tensor scale is out of the fp32-safe range)
    const float inv_6sg = 1.0f / (6.0f * sgq);
    if (!live) return;
    if (__builtin_expect(shift != 1.0f, 0)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) rescale_block16(w[i], shift);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc = pk_absmax_u16(acc, w[i][k]);
    const float bmax = __uint_as_float(pk_hmax_u16(acc) << 16);
    const uint32_t sbyte = block_scale_exact(bmax, sgq, inv_6sg);
    const float sb = e4m3_to_f32(sbyte);
    uint32_t c0[16], c1[16];                       // row i of the tile: codes of columns 0-7, 8-15
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        encode_block16(w[i], sb, sgq, c0[i], c1[i]);
        const int64_t row = 16 * I + i;
        *(uint2v *)(codes + row * (C >> 1) + 8 * J) = uint2v{c0[i], c1[i]};
        scales[row * tc + J] = (uint8_t)sbyte;
    }
    if (codes_t) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            // column j of the tile = 16 codes of row 16 J + j of the transposed operand
            uint32_t t0 = 0, t1 = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                t0 |= (((j < 8 ? c0[i] : c1[i]) >> (4 * (j & 7))) & 15u) << (4 * i);
                t1 |= (((j < 8 ? c0[i + 8] : c1[i + 8]) >> (4 * (j & 7))) & 15u) << (4 * i);
            }
            const int64_t row = 16 * J + j;
            *(uint2v *)(codes_t + row * (R >> 1) + 8 * I) = uint2v{t0, t1};
            scales_t[row * tr + I] = (uint8_t)sbyte;
        }
    }
}

// --------------------------------------------------------------------------
// KV-cache reconstruction: x^ = RN_bf16(code * s_b * s_g), the product exact,
// one rounding.  For a given tensor there are only 127 * 8 distinct magnitudes,
// so each workgroup builds that table exactly (fp64) in LDS once, split into a
// low-byte and a high-byte plane per scale, and every element is then two
// byte-permute lookups.  One lane per half block (8 elements): a wave's loads and
// stores are then each one contiguous stretch (256 bytes of codes in, 1 KB of bf16
// out), which is worth a fifth more bandwidth than 32 bytes per lane in two pieces.
// --------------------------------------------------------------------------
// table[scale byte] = {low bytes of magnitudes 0-3, low bytes 4-7, high bytes 0-3, high bytes 4-7}
__device__ __forceinline__ void build_dequant_table(uint4v *table, double sg)
{
    if (threadIdx.x < 128) {
        const uint32_t s = threadIdx.x;
        const double sb = (double)e4m3_to_f32(s < 127u ? s : 0u);
        uint32_t lo0 = 0, lo1 = 0, hi0 = 0, hi1 = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const double mag = i < 4 ? 0.5 * i : (i == 4 ? 2.0 : (i == 5 ? 3.0 : (i == 6 ? 4.0 : 6.0)));
            uint32_t h = bf16_rne_from_f64(mag * sb * sg);   // mag*sb: 6 bits, times 24 bits: exact
            if (i < 4) { lo0 |= (h & 0xFFu) << (8 * i); hi0 |= (h >> 8) << (8 * i); }
            else { lo1 |= (h & 0xFFu) << (8 * (i - 4)); hi1 |= (h >> 8) << (8 * (i - 4)); }
        }
        uint4v e = {lo0, lo1, hi0, hi1};
        table[s] = e;
    }
}

// eight codes (one dword) -> eight bf16 (four dwords) through the table row t of their scale
__device__ __forceinline__ void dequant_half_lookup(uint32_t cw, uint4v t, uint32_t (&o)[4])
{
    // selectors: magnitude index of the even / odd elements, one per byte
    uint32_t se = cw & 0x07070707u, so = (cw >> 4) & 0x07070707u;
    uint32_t lo_e = __builtin_amdgcn_perm(t.y, t.x, se), lo_o = __builtin_amdgcn_perm(t.y, t.x, so);
    uint32_t hi_e = __builtin_amdgcn_perm(t.w, t.z, se), hi_o = __builtin_amdgcn_perm(t.w, t.z, so);
    hi_e |= (cw << 4) & 0x80808080u;      // sign of even elements: bit 3 of each byte
    hi_o |= cw & 0x80808080u;             // sign of odd elements: bit 7
    // element 2b = (hi_e.b, lo_e.b), element 2b+1 = (hi_o.b, lo_o.b); dword b = elems 2b, 2b+1
    uint32_t e01 = __builtin_amdgcn_perm(hi_e, lo_e, 0x05010400u);  // even elems of bytes 0, 1
    uint32_t e23 = __builtin_amdgcn_perm(hi_e, lo_e, 0x07030602u);
    uint32_t o01 = __builtin_amdgcn_perm(hi_o, lo_o, 0x05010400u);
    uint32_t o23 = __builtin_amdgcn_perm(hi_o, lo_o, 0x07030602u);
    o[0] = __builtin_amdgcn_perm(o01, e01, 0x05040100u);
    o[1] = __builtin_amdgcn_perm(o01, e01, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(o23, e23, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(o23, e23, 0x07060302u);
}

__global__ __launch_bounds__(256) void dequant_bf16_kernel(const uint8_t *__restrict__ codes,
                                                           const uint8_t *__restrict__ scales,
                                                           const float *__restrict__ gs, int64_t nblk,
                                                           uint16_t *__restrict__ out)
{
    __shared__ uint4v table[128];
    build_dequant_table(table, (double)*gs);
    __syncthreads();
    // One lane per half block (eight codes in, sixteen bytes out): every load and every store instruction of a wave
    // covers one contiguous stretch.  The stores are streaming ones: 7 % faster here, and a consumer that reads the
    // window right afterwards loses as much again, so the pair costs the same either way (measured with a plain read).  A workgroup takes the units of 256 * U half blocks at a grid-wide stride.
    constexpr int U = kDequantUnroll;             // half blocks in flight per lane
    const int64_t nhalf = nblk << 1;
    for (int64_t h0 = (int64_t)blockIdx.x * (256 * U) + threadIdx.x; h0 < nhalf; h0 += (int64_t)gridDim.x * (256 * U)) {
        uint32_t cws[U], sbs[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t h = h0 + u * 256;
            if (h < nhalf) {
                cws[u] = __builtin_nontemporal_load((const uint32_t *)codes + h);
                sbs[u] = scales[h >> 1];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t h = h0 + u * 256;
            if (h >= nhalf) continue;
            uint32_t o[4];
            dequant_half_lookup(cws[u], table[sbs[u] & 0x7Fu], o);
            __builtin_nontemporal_store(uint4v{o[0], o[1], o[2], o[3]}, (uint4v *)(out + (h << 3)));
        }
    }
}

// --------------------------------------------------------------------------
// Gathered reconstruction (Sec. 3.2: with sink tokens and a sliding window an attention step
// reads several cached chunks): up to kMaxKvChunks NVFP4 chunks, each with its own tensor
// scale and, for smoothed keys, its row means, are written back to back into one bf16
// [sum T_c, H, d] buffer by ONE launch.  A workgroup works inside one chunk (it owns
// kGatherBlocksPerWg consecutive blocks of it), so the table of the plain path is built once
// per workgroup; a smoothed chunk adds its row mean before the single rounding,
// RN_bf16(code * s_b * s_g + mean), which takes the exact product and sum in fp64.
// --------------------------------------------------------------------------
constexpr int kGatherBlocksPerWg = 256 * 2;    // small workgroups: many loads in flight chip-wide matter more than table reuse
struct GatherTable {
    const uint8_t *codes[kMaxKvChunks];
    const uint8_t *scales[kMaxKvChunks];
    const float *gs[kMaxKvChunks];
    const uint16_t *mean[kMaxKvChunks];           // nullptr: not smoothed
    int64_t blk_start[kMaxKvChunks + 1];          // first block (16 elements) of chunk c in the output
    int wg_start[kMaxKvChunks + 1];               // first workgroup of chunk c
    int n_chunks;
    int nb_row;                                    // blocks per row (d / 16)
    int row_shift;                                 // log2(nb_row) when that is a power of two, else -1
};

// One unit of a chunk: 256 * U half blocks from half block h0 (this lane's first) on.  Every load of the unit is
// issued before the first result is used (indices past the end of the chunk are clamped, their results dropped), so a
// workgroup waits for memory once.
template <bool SMOOTH>
__device__ __forceinline__ void gather_unit(const uint4v *table, const uint8_t *__restrict__ codes,
                                            const uint8_t *__restrict__ scales, const uint16_t *__restrict__ mean,
                                            double sg, int64_t nhalf, int64_t h0, int nb_row, int row_shift,
                                            uint16_t *__restrict__ dst)
{
    constexpr int U = 4;                                   // half blocks in flight per lane
    uint32_t cws[U], sbs[U], mus[U];
    int64_t hc[U], row[U];
#pragma unroll
    for (int u = 0; u < U; ++u) hc[u] = min(h0 + u * 256, nhalf - 1);
    if constexpr (SMOOTH) {                                // row of the half block: its mean (a shift when d / 16 is a power of two)
        if (row_shift >= 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) row[u] = hc[u] >> (row_shift + 1);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) row[u] = (hc[u] >> 1) / nb_row;
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        cws[u] = __builtin_nontemporal_load((const uint32_t *)codes + hc[u]);
        sbs[u] = scales[hc[u] >> 1] & 0x7Fu;
        if constexpr (SMOOTH) mus[u] = mean[row[u]];
    }
    const float sgf = (float)sg;                           // (the chunk's tensor scale is an fp32 number)
    const bool sg_mid = sgf >= 0x1p-60f && sgf <= 0x1p60f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t h = h0 + u * 256;
        if (h >= nhalf) continue;
        const uint32_t cw = cws[u];
        uint32_t o[4];
        if constexpr (!SMOOTH) {
            dequant_half_lookup(cw, table[sbs[u]], o);
        } else {
            // RN_bf16(code s_b s_g + mean), the exact sum rounded once.  code s_b is exact in fp32 (2 + 4 bits), and
            // the fused multiply-add rounds (code s_b) s_g + mean once, to fp32: the result lies within half an
            // fp32 ulp of the exact sum, and rounding to bf16 is constant between consecutive bf16 midpoints, which
            // are fp32 numbers -- so the two round alike unless the fp32 result is itself a midpoint (low sixteen
            // bits 0x8000: one element in 65 536).  With the tensor scale and the mean in [2^-60, 2^60] (or a mean
            // of zero) every non-zero sum is a multiple of 2^-93 below 2^73: nothing overflows or goes subnormal.
            // The rest takes the sum in fp64.
            typedef float float2v __attribute__((ext_vector_type(2)));
            const float muf = __uint_as_float(mus[u] << 16), amu = fabsf(muf);
            const float sbf = e4m3_to_f32(sbs[u]);
            uint32_t hit = 0xFFFFFFFFu;
#define NVFP4_GATHER_PAIR(I, SEL)                                                                 \
    {                                                                                             \
        const float2v q = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(cw, 1.0f, SEL);                \
        const float y0 = __builtin_fmaf(q.x * sbf, sgf, muf), y1 = __builtin_fmaf(q.y * sbf, sgf, muf); \
        const uint32_t low = __builtin_amdgcn_perm(__float_as_uint(y1), __float_as_uint(y0), 0x05040100u) ^ 0x80008000u; \
        hit = __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(ushort2v, hit), __builtin_bit_cast(ushort2v, low))); \
        o[I] = pack_bf16x2(y0, y1);                                                               \
    }
            NVFP4_GATHER_PAIR(0, 0) NVFP4_GATHER_PAIR(1, 1) NVFP4_GATHER_PAIR(2, 2) NVFP4_GATHER_PAIR(3, 3)
#undef NVFP4_GATHER_PAIR
            const bool sure = sg_mid & ((hit & 0xFFFFu) != 0u) & ((hit >> 16) != 0u) &
                              ((amu == 0.0f) | ((amu >= 0x1p-60f) & (amu <= 0x1p60f)));
            if (__builtin_expect(!sure, 0)) {
                const double mu = (double)muf;
                const double den = (double)sbf * sg;                // exact
#define NVFP4_GATHER_PAIR(I, SEL)                                                                 \
    {                                                                                             \
        const float2v q = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(cw, 1.0f, SEL);                \
        o[I] = bf16_rne_signed_from_f64((double)q.x * den + mu) |                                 \
               (bf16_rne_signed_from_f64((double)q.y * den + mu) << 16);                          \
    }
                NVFP4_GATHER_PAIR(0, 0) NVFP4_GATHER_PAIR(1, 1) NVFP4_GATHER_PAIR(2, 2) NVFP4_GATHER_PAIR(3, 3)
#undef NVFP4_GATHER_PAIR
            }
        }
        __builtin_nontemporal_store(uint4v{o[0], o[1], o[2], o[3]}, (uint4v *)(dst + (h << 3)));
    }
}

__global__ __launch_bounds__(256) void dequant_gather_kernel(GatherTable t, uint16_t *__restrict__ out)
{
    __shared__ uint4v table[128];
    // this workgroup's chunk: the last c with wg_start[c] <= blockIdx.x, by bisection (uniform; a linear walk over
    // the table costs a dependent scalar load per chunk before the first byte of data is requested)
    int c = 0, hi = t.n_chunks - 1;
    while (c < hi) {
        const int mid = (c + hi + 1) >> 1;
        if ((int)blockIdx.x >= t.wg_start[mid]) c = mid;
        else hi = mid - 1;
    }
    const uint8_t *__restrict__ codes = t.codes[c];
    const uint8_t *__restrict__ scales = t.scales[c];
    const uint16_t *__restrict__ mean = t.mean[c];
    const double sg = (double)*t.gs[c];
    const int64_t nblk = t.blk_start[c + 1] - t.blk_start[c];
    const int64_t first = (int64_t)((int)blockIdx.x - t.wg_start[c]) * kGatherBlocksPerWg;
    uint16_t *dst = out + (t.blk_start[c] << 4);
    const int64_t nhalf = nblk << 1;
    if (!mean) {
        build_dequant_table(table, sg);
        __syncthreads();
    }
    for (int it = 0; it < 2 * kGatherBlocksPerWg / (256 * 4); ++it) {
        const int64_t h0 = 2 * first + it * (256 * 4) + threadIdx.x;
        if (h0 - threadIdx.x >= nhalf) break;             // (the same for the whole workgroup)
        if (mean) gather_unit<true>(table, codes, scales, mean, sg, nhalf, h0, t.nb_row, t.row_shift, dst);
        else gather_unit<false>(table, codes, scales, mean, sg, nhalf, h0, t.nb_row, t.row_shift, dst);
    }
}

// --------------------------------------------------------------------------
static int grid_for(int64_t work_items, int max_grid)
{
    int64_t g = (work_items + 255) / 256;
    if (g < 1) g = 1;
    return (int)(g < max_grid ? g : max_grid);
}

hipError_t launch_amax(const uint16_t *x, int64_t R, int64_t C, int64_t ld, uint32_t *partial,
                       int *n_partial, hipStream_t s)
{
    const int64_t want = (R * (C >> 3) + kAmaxThreads - 1) / kAmaxThreads;
    const int grid = (int)std::max<int64_t>(1, std::min<int64_t>(want, kAmaxGrid));
    *n_partial = grid;
    const bool stream = (uint64_t)R * (uint64_t)C * 2u > (256ull << 20);
    if (ld == C) {
        if (stream) amax_partial_kernel<true, true><<<grid, kAmaxThreads, 0, s>>>(x, R, C, ld, partial);
        else amax_partial_kernel<true, false><<<grid, kAmaxThreads, 0, s>>>(x, R, C, ld, partial);
    } else {
        if (stream) amax_partial_kernel<false, true><<<grid, kAmaxThreads, 0, s>>>(x, R, C, ld, partial);
        else amax_partial_kernel<false, false><<<grid, kAmaxThreads, 0, s>>>(x, R, C, ld, partial);
    }
    return hipGetLastError();
}

hipError_t launch_scale_from_partials(const uint32_t *partial, int n_partial, float *gs_out, hipStream_t s)
{
    scale_from_partials_kernel<<<1, 256, 0, s>>>(partial, n_partial, gs_out);
    return hipGetLastError();
}

hipError_t launch_quantize_rows(const uint16_t *x, int64_t R, int64_t C, int64_t ld, const float *gs_in,
                                const uint32_t *partial, int n_partial, uint8_t *codes, uint8_t *scales,
                                float *gs_out, hipStream_t s, bool scale_search)
{
    int grid = grid_for(R * (C >> 4), kQuantMaxGrid);
    if (scale_search) {
        if (ld == C)
            quantize_rows_kernel<true, true><<<grid, 256, 0, s>>>(x, R, C, ld, gs_in, partial, n_partial, codes,
                                                                  scales, gs_out);
        else
            quantize_rows_kernel<false, true><<<grid, 256, 0, s>>>(x, R, C, ld, gs_in, partial, n_partial, codes,
                                                                   scales, gs_out);
    } else if (ld == C)
        quantize_rows_kernel<true><<<grid, 256, 0, s>>>(x, R, C, ld, gs_in, partial, n_partial, codes,
                                                        scales, gs_out);
    else
        quantize_rows_kernel<false><<<grid, 256, 0, s>>>(x, R, C, ld, gs_in, partial, n_partial, codes,
                                                         scales, gs_out);
    return hipGetLastError();
}

hipError_t launch_quantize_cols(const uint16_t *x, int64_t R, int64_t C, int64_t ld, const float *gs_in,
                                const uint32_t *partial, int n_partial, uint8_t *codes, uint8_t *scales,
                                float *gs_out, hipStream_t s)
{
    dim3 grid((unsigned)((C + kTC - 1) / kTC), (unsigned)((R + kTR - 1) / kTR));
    quantize_cols_kernel<false><<<grid, 256, 0, s>>>(x, R, C, ld, gs_in, partial, n_partial, codes, scales, gs_out);
    return hipGetLastError();
}

size_t rht_inexact_bytes(int64_t R, int64_t C) { return (size_t)(((C + kTC - 1) / kTC) * ((R + kTR - 1) / kTR)) * 256; }

hipError_t launch_amax_rht(const uint16_t *x, int64_t R, int64_t C, int64_t ld, uint32_t sign_mask,
                           uint32_t *partial, int *n_partial, uint8_t *inexact, hipStream_t s)
{
    const int64_t tiles = ((C + kTC - 1) / kTC) * ((R + kTR - 1) / kTR);
    const int grid = (int)(tiles < kMaxPartials ? tiles : kMaxPartials);
    *n_partial = grid;
    if ((uint64_t)R * (uint64_t)C * 2u > (256ull << 20)) amax_rht_kernel<true><<<grid, 256, 0, s>>>(x, R, C, ld, sign_mask, partial, inexact);
    else amax_rht_kernel<false><<<grid, 256, 0, s>>>(x, R, C, ld, sign_mask, partial, inexact);
    return hipGetLastError();
}

hipError_t launch_quantize_cols_rht(const uint16_t *x, int64_t R, int64_t C, int64_t ld, uint32_t sign_mask,
                                    const float *gs_in, const uint32_t *partial, int n_partial,
                                    uint8_t *codes, uint8_t *scales, float *gs_out, const uint8_t *inexact, hipStream_t s)
{
    dim3 grid((unsigned)((C + kTC - 1) / kTC), (unsigned)((R + kTR - 1) / kTR));
    quantize_cols_kernel<true><<<grid, 256, 0, s>>>(x, R, C, ld, gs_in, partial, n_partial, codes, scales,
                                                    gs_out, sign_mask, inexact);
    return hipGetLastError();
}

hipError_t launch_dequant_bf16(const uint8_t *codes, const uint8_t *scales, const float *gs, int64_t rows,
                               int64_t K, uint16_t *out, hipStream_t s)
{
    int64_t nblk = rows * (K >> 4);
    int grid = grid_for((2 * nblk + kDequantUnroll - 1) / kDequantUnroll, kDequantMaxGrid);      // at most one workgroup per unit
    dequant_bf16_kernel<<<grid, 256, 0, s>>>(codes, scales, gs, nblk, out);
    return hipGetLastError();
}

hipError_t launch_quantize_tiles(const uint16_t *x, int64_t R, int64_t C, int64_t ld, const float *gs_in,
                                 const uint32_t *partial, int n_partial, uint8_t *codes, uint8_t *scales,
                                 uint8_t *codes_t, uint8_t *scales_t, float *gs_out, float *gs_out_t,
                                 hipStream_t s)
{
    dim3 grid((unsigned)((C + 255) / 256), (unsigned)((R + 255) / 256));
    quantize_tiles_kernel<<<grid, 256, 0, s>>>(x, R, C, ld, gs_in, partial, n_partial, codes, scales, codes_t,
                                               scales_t, gs_out, gs_out_t);
    return hipGetLastError();
}

hipError_t launch_quantize_rows_slabs(const uint16_t *x, int64_t T, int64_t H, int64_t d, int slab_heads,
                                      const float *gs_in, const uint32_t *partial, int n_partial,
                                      uint8_t *codes, uint8_t *scales, float *gs_out, hipStream_t s)
{
    int grid = grid_for(T * H * (d >> 4), kQuantMaxGrid);
    quantize_rows_kernel<true, false, false><<<grid, 256, 0, s>>>(x, T * H, d, d, gs_in, partial, n_partial, codes,
                                                                  scales, gs_out, nullptr, (int)H, slab_heads);
    return hipGetLastError();
}

hipError_t launch_amax_smooth(const uint16_t *x, int64_t rows, int d, uint16_t *mean_out, uint32_t *partial,
                              int *n_partial, hipStream_t s)
{
    const int64_t want = (rows * (d >> 4) + kAmaxThreads - 1) / kAmaxThreads;
    const int grid = (int)std::max<int64_t>(1, std::min<int64_t>(want, kAmaxGrid));
    *n_partial = grid;
    amax_smooth_kernel<<<grid, kAmaxThreads, 0, s>>>(x, rows, __builtin_ctz((unsigned)(d >> 4)), mean_out, partial);
    return hipGetLastError();
}

hipError_t launch_quantize_rows_smooth(const uint16_t *x, int64_t rows, int d, const uint16_t *row_mean,
                                       const uint32_t *partial, int n_partial, uint8_t *codes,
                                       uint8_t *scales, float *gs_out, hipStream_t s)
{
    int grid = grid_for(rows * (d >> 4), kQuantMaxGrid);
    quantize_rows_kernel<true, true, true><<<grid, 256, 0, s>>>(x, rows, d, d, nullptr, partial, n_partial, codes,
                                                                scales, gs_out, row_mean, 0, 0,
                                                                __builtin_ctz((unsigned)(d >> 4)));
    return hipGetLastError();
}

hipError_t launch_dequant_gather(const KvChunkDesc *chunks, int n_chunks, int64_t H, int64_t d, uint16_t *out,
                                 hipStream_t s)
{
    GatherTable t{};
    t.n_chunks = n_chunks;
    t.nb_row = (int)(d >> 4);
    t.row_shift = (t.nb_row & (t.nb_row - 1)) == 0 ? __builtin_ctz((unsigned)t.nb_row) : -1;
    int64_t blk = 0;
    int wg = 0;
    for (int c = 0; c < n_chunks; ++c) {
        t.codes[c] = chunks[c].codes;
        t.scales[c] = chunks[c].scales;
        t.gs[c] = chunks[c].global_scale;
        t.mean[c] = chunks[c].row_mean;
        t.blk_start[c] = blk;
        t.wg_start[c] = wg;
        const int64_t nblk = chunks[c].T * H * (d >> 4);
        blk += nblk;
        wg += (int)((nblk + kGatherBlocksPerWg - 1) / kGatherBlocksPerWg);
    }
    t.blk_start[n_chunks] = blk;
    t.wg_start[n_chunks] = wg;
    dequant_gather_kernel<<<wg, 256, 0, s>>>(t, out);
    return hipGetLastError();
}

}  // namespace nvfp4
