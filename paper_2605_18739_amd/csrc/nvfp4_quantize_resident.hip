// One-launch row quantizer for tensors that fit on the chip (Sec. 2.2, Eq. 2; Appendix Eq. 12-13;
// Sec. 3.2, Eq. 5-6).
//
// The tensor scale needs the tensor's largest magnitude before the first code can be written, which
// is why the streaming quantizer reads its input twice.  An MI355X holds about 170 MB in registers
// and LDS (256 compute units x (512 KB + 160 KB)), so a KV window, an activation or a weight matrix
// of up to ~120 MB can stay there between the two steps: every workgroup loads its slice ONCE into
// registers (and LDS), publishes the slice's maximum, waits until all workgroups have done so, and
// encodes from the on-chip copy.  HBM traffic is the algorithmic 2 + 0.5625 bytes per element.
//
// The wait is bounded.  A workgroup that gives up (another kernel holding compute units so that
// part of this grid cannot become resident, or the test hook that sets the limit to zero) derives
// the tensor maximum itself by scanning the whole tensor, so the result never depends on the wait.
// Every workgroup reaches the end of the kernel whatever the others do.
#include "nvfp4_device.h"

#include <algorithm>
#include "nvfp4_kernels.h"

#include <type_traits>

namespace nvfp4 {

constexpr int kResThreads = 512;          // 8 waves, two per SIMD, up to 256 registers each
constexpr int kResRegSlots = 20;          // 16-element blocks a lane keeps in registers (160 registers)
constexpr int kResLdsSlots = 9;           // ... and in LDS (9 x 16 KB)
constexpr int kResSlots = kResRegSlots + kResLdsSlots;
constexpr int kResLdsBytes = kResLdsSlots * kResThreads * 32 + 64;   // blocks, reduction words
constexpr int kResMaxGrid = 256;          // one workgroup per compute unit

// The grid-wide exchange of the workgroups' maxima: one 64-bit word per workgroup and call in flight,
// (epoch << 32) | maximum, in memory the library owns.  A workgroup publishes its word with one store
// and then watches the others' words until each carries the epoch of this launch; epochs of a slot never
// repeat (32 bits), so words left by earlier launches are never mistaken for this one's, nothing has to be
// cleared, and no workgroup waits on a counter.
// The epoch is counted ON THE DEVICE, so that a launch replayed from a captured graph (the same kernel
// arguments every time) still gets a fresh one: every workgroup reads the slot's counter and then registers
// itself; the last to register advances the counter for the NEXT launch on the slot, which stream order
// places after this one.  Launches that overlap on one slot (more than 64 calls in flight at once, or one
// captured graph replayed concurrently with itself) would race.
constexpr int kSyncSlots = 64;
static __device__ unsigned long long g_grid_words[kSyncSlots][kResMaxGrid];
static __device__ uint32_t g_slot_epoch[kSyncSlots], g_slot_arrivals[kSyncSlots];

template <int First, int Last, class F>
__device__ __forceinline__ void static_for_slots(F &&f)
{
    if constexpr (First < Last) {
        f(std::integral_constant<int, First>{});
        static_for_slots<First + 1, Last>(f);
    }
}

struct ResidentArgs {
    const uint16_t *x;          // [rows, C] contiguous
    int64_t nblk;               // rows * C / 16
    int row_shift;              // SMOOTH: log2(C / 16)
    int sync_slot;
    uint32_t spin_limit;        // bound of the grid-wide wait in 10 ns ticks
    uint8_t *codes, *scales;
    float *gs_out;
    uint16_t *mean_out;         // SMOOTH: [rows] bf16 row means
    // slab_heads > 0: the rows are (token, head) pairs of a [T, H, d] tensor and the output is regrouped into
    // H / slab_heads slabs of slab_heads heads each, [slab][token][head in slab] (the all-to-all send buffers)
    uint32_t nb_row, heads, slab_heads, tokens;
};

// output block index of input block g (fewer than 2^32 blocks fit on the chip: 32-bit arithmetic)
__device__ __forceinline__ uint32_t output_block(uint32_t g, const ResidentArgs &a)
{
    if (a.slab_heads == 0) return g;
    const uint32_t row = g / a.nb_row, b = g - row * a.nb_row;
    const uint32_t t = row / a.heads, h = row - t * a.heads;
    const uint32_t slab = h / a.slab_heads, hl = h - slab * a.slab_heads;
    return ((slab * a.tokens + t) * a.slab_heads + hl) * a.nb_row + b;
}

// maximum of two pairs of 16-bit patterns, half by half
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2v, a), __builtin_bit_cast(ushort2v, b)));
}

// One block's share of pass 1: (SMOOTH: remove the row mean, in place;) largest |bf16| pattern.
// live: the block exists (lanes past the end hold zeros and only take part in the shuffles).
template <bool SMOOTH, bool WRITE_MEAN = true>
__device__ __forceinline__ uint32_t block_pass1(uint32_t (&w)[8], bool live, int64_t g, const ResidentArgs &a)
{
    if constexpr (SMOOTH) {
        const int nb_row = 1 << a.row_shift;
        double sum = 0.0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            sum += (double)bf16lo_to_f32(w[i]);
            sum += (double)bf16hi_to_f32(w[i]);
        }
        for (int m = 1; m < nb_row; m <<= 1) sum += __shfl_xor(sum, m, 64);
        const double inv_d = 1.0 / (double)(16 << a.row_shift);           // a power of two: the quotient is exact
        const uint32_t mean_bits = bf16_rne_signed_from_f64(sum * inv_d);
        if (live) {
            if (WRITE_MEAN && (g & (nb_row - 1)) == 0) a.mean_out[g >> a.row_shift] = (uint16_t)mean_bits;
            smooth_block16(w, __uint_as_float(mean_bits << 16));
        }
    }
    (void)live; (void)g; (void)a;
    uint32_t acc = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc = pk_absmax_u16(acc, w[i]);
    return acc;
}

struct Pass2Out {
    __amdgpu_buffer_rsrc_t rcodes, rscales;        // the outputs as buffers of nblk * 8 and nblk bytes
};

// Two blocks through one straight-line stretch of code.  The stores go through buffer descriptors sized to
// the outputs: a block past the end of the tensor gets an offset outside the descriptor's range, which the
// hardware drops, so no branch surrounds the stores and the compiler can schedule across them.
template <bool SEARCH>
__device__ __forceinline__ void pair_pass2(const uint32_t (&wa)[8], const uint32_t (&wb)[8], int64_t ga, int64_t gb, int64_t nblk,
                                           float sg, float inv_6sg, float inv_4sg, const Pass2Out &out, const ResidentArgs &a)
{
    uint32_t sa, a0, a1, sb, b0, b1;
    if constexpr (SEARCH) {
        quantize_block16_4over6_inline(wa, sg, inv_6sg, inv_4sg, sa, a0, a1);
        quantize_block16_4over6_inline(wb, sg, inv_6sg, inv_4sg, sb, b0, b1);
    } else {
        quantize_pair16(wa, wb, sg, inv_6sg, sa, a0, a1, sb, b0, b1);
    }
    constexpr uint32_t kDropped = 0x80000000u;
    const bool live_a = ga < nblk, live_b = gb < nblk;
    const uint32_t oa = live_a ? output_block((uint32_t)ga, a) : 0u, ob = live_b ? output_block((uint32_t)gb, a) : 0u;
    __builtin_amdgcn_raw_buffer_store_b64(uint2v{a0, a1}, out.rcodes, live_a ? oa << 3 : kDropped, 0, 2 /* nontemporal */);
    __builtin_amdgcn_raw_buffer_store_b8((uint8_t)sa, out.rscales, live_a ? oa : kDropped, 0, 0);
    __builtin_amdgcn_raw_buffer_store_b64(uint2v{b0, b1}, out.rcodes, live_b ? ob << 3 : kDropped, 0, 2);
    __builtin_amdgcn_raw_buffer_store_b8((uint8_t)sb, out.rscales, live_b ? ob : kDropped, 0, 0);
}

template <bool SEARCH, bool SMOOTH>
__global__ __launch_bounds__(kResThreads) void quantize_rows_resident_kernel(ResidentArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint4v *lds_blk = (uint4v *)lds;                                   // [slot][half][thread]
    uint32_t *lds_red = (uint32_t *)(lds + kResLdsSlots * kResThreads * 32);   // 16 words
    const Pass2Out out{__builtin_amdgcn_make_buffer_rsrc((void *)a.codes, 0, (int)(a.nblk << 3), 0x00020000),
                       __builtin_amdgcn_make_buffer_rsrc((void *)a.scales, 0, (int)a.nblk, 0x00020000)};
    const int tid = threadIdx.x, G = gridDim.x;
    // A workgroup owns a contiguous stretch of the tensor: the tensor's units of 512 blocks (one slot of one
    // workgroup, 16 KB of input) are dealt out in order, 27 or 28 to each for the KV window.  (Contiguous stretches per
    // workgroup move about a fifth more bytes per second through HBM than a grid-wide stride does.)
    const int64_t n_units = (a.nblk + kResThreads - 1) / kResThreads;
    const int64_t unit0 = n_units * blockIdx.x / G, unit1 = n_units * (blockIdx.x + 1) / G;
    const int nb = (int)(unit1 - unit0);                               // slots this workgroup uses (at most kResSlots)
    const int64_t wg_first = unit0 * kResThreads;
    const int nr = min(nb, kResRegSlots), nl = nb - nr;                // register slots / LDS slots in use
    auto block_of = [&](int slot) { return wg_first + (int64_t)slot * kResThreads + tid; };
    uint32_t *queue_head = lds_red + 12;                               // tickets for the LDS slots in pass 2
    uint32_t epoch = 0, arrival = 0;                                   // (lane 0 of the workgroup only)
    if (tid == 0) {
        *queue_head = 0;
        epoch = __hip_atomic_load(&g_slot_epoch[a.sync_slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
        if (epoch == 0u) epoch = 1u;                                   // (0 is what never-written words hold)
    }

    // ---- pass 1: load every block once; registers first (all loads in flight together), then LDS slots
    uint4v r0[kResRegSlots], r1[kResRegSlots];
    static_for_slots<0, kResRegSlots>([&](auto i_c) {
        constexpr int i = decltype(i_c)::value;
        r0[i] = uint4v{0, 0, 0, 0};
        r1[i] = uint4v{0, 0, 0, 0};
        if (i < nr) {
            const int64_t g = block_of(i);
            if (g < a.nblk) {
                const uint4v *p = (const uint4v *)(a.x + (g << 4));
                r0[i] = __builtin_nontemporal_load(p);
                r1[i] = __builtin_nontemporal_load(p + 1);
            }
        }
    });
    if (tid == 0) {
        // register only once the counter has been read (the empty asm makes the increment depend on the value read;
        // the wait it costs is for that one load, the oldest in flight, not for the data loads issued since)
        uint32_t one = 1;
        asm volatile("" : "+v"(one) : "v"(epoch));
        arrival = atomicAdd(&g_slot_arrivals[a.sync_slot], one);
    }
    uint32_t amax = 0;                       // two running maxima of |bf16| patterns, one per half
    {   // LDS slots, two blocks in flight
        uint4v n0 = {0, 0, 0, 0}, n1 = {0, 0, 0, 0};
        auto fetch = [&](int s) {
            const int64_t g = block_of(kResRegSlots + s);
            n0 = uint4v{0, 0, 0, 0};
            n1 = uint4v{0, 0, 0, 0};
            if (g < a.nblk) {
                const uint4v *p = (const uint4v *)(a.x + (g << 4));
                n0 = __builtin_nontemporal_load(p);
                n1 = __builtin_nontemporal_load(p + 1);
            }
        };
        if (nl > 0) fetch(0);
        for (int s = 0; s < nl; ++s) {
            uint32_t w[8] = {n0.x, n0.y, n0.z, n0.w, n1.x, n1.y, n1.z, n1.w};
            const int64_t g = block_of(kResRegSlots + s);
            if (s + 1 < nl) fetch(s + 1);
            amax = pk_max_u16(amax, block_pass1<SMOOTH>(w, g < a.nblk, g, a));
            lds_blk[(2 * s) * kResThreads + tid] = uint4v{w[0], w[1], w[2], w[3]};
            lds_blk[(2 * s + 1) * kResThreads + tid] = uint4v{w[4], w[5], w[6], w[7]};
        }
    }
    static_for_slots<0, kResRegSlots>([&](auto i_c) {
        constexpr int i = decltype(i_c)::value;
        if (i < nr) {
            uint32_t w[8] = {r0[i].x, r0[i].y, r0[i].z, r0[i].w, r1[i].x, r1[i].y, r1[i].z, r1[i].w};
            const int64_t g = block_of(i);
            amax = pk_max_u16(amax, block_pass1<SMOOTH>(w, g < a.nblk, g, a));
            if constexpr (SMOOTH) {
                r0[i] = uint4v{w[0], w[1], w[2], w[3]};
                r1[i] = uint4v{w[4], w[5], w[6], w[7]};
            }
        }
    });

    // ---- this workgroup's maximum, then the grid-wide exchange.  The words are agent-scope atomics (they
    // bypass the per-XCD caches by themselves): no cache write-back or invalidation is needed around them.
    uint32_t m = wave_max_u32(pk_hmax_u16(amax));
    if ((tid & 63) == 0) lds_red[tid >> 6] = m;
    if (tid == 0) {
        lds_red[11] = epoch;
        if (arrival == (uint32_t)G - 1u) {          // every workgroup of this launch has read the counter: advance it
            __hip_atomic_store(&g_slot_arrivals[a.sync_slot], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&g_slot_epoch[a.sync_slot], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    epoch = lds_red[11];
    unsigned long long *words = g_grid_words[a.sync_slot];
    if (tid == 0) {
        uint32_t all = 0;
#pragma unroll
        for (int w = 0; w < kResThreads / 64; ++w) all = max(all, lds_red[w]);
        __hip_atomic_store(&words[blockIdx.x], ((unsigned long long)epoch << 32) | all, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    // lane t watches workgroup t's word; the wait is bounded
    uint32_t tmax = 0;
    bool seen = true;
    if (tid < G) {
        const uint64_t t0 = wall_clock64();
        seen = false;
        for (;;) {
            const unsigned long long v = __hip_atomic_load(&words[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((uint32_t)(v >> 32) == epoch) {
                tmax = (uint32_t)v;
                seen = true;
                break;
            }
            if (wall_clock64() - t0 > (uint64_t)a.spin_limit) break;
            __builtin_amdgcn_s_sleep(1);
        }
    }
    const bool arrived = __syncthreads_and(seen) != 0;
    if (!arrived) {
        // gave up waiting: the tensor maximum from the tensor itself, this workgroup alone
        tmax = 0;
        for (int64_t g0 = 0; g0 < a.nblk; g0 += kResThreads) {
            const int64_t g = g0 + tid;
            uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (g < a.nblk) {
                const uint4v *p = (const uint4v *)(a.x + (g << 4));
                const uint4v v0 = p[0], v1 = p[1];
                w[0] = v0.x; w[1] = v0.y; w[2] = v0.z; w[3] = v0.w;
                w[4] = v1.x; w[5] = v1.y; w[6] = v1.z; w[7] = v1.w;
            }
            tmax = max(tmax, pk_hmax_u16(block_pass1<SMOOTH, false>(w, g < a.nblk, g, a)));   // (the means are written by the rows' owners)
        }
    }
    tmax = wave_max_u32(tmax);
    if ((tid & 63) == 0) lds_red[tid >> 6] = tmax;     // (the first reduction's words were read before the barrier above)
    __syncthreads();
    tmax = 0;
#pragma unroll
    for (int w = 0; w < kResThreads / 64; ++w) tmax = max(tmax, lds_red[w]);
    const float sg = global_scale_from_amax_bits(tmax);
    if (blockIdx.x == 0 && tid == 0) *a.gs_out = sg;
    const float inv_6sg = 1.0f / (6.0f * sg), inv_4sg = 1.0f / (4.0f * sg);
    if (__builtin_expect(scale_out_of_range(sg), 0)) {
        // A tensor scale outside the range in which fp32 quotients are safe: every block one at a time with the
        // tensor and its scale shifted back into range, from
        // memory (the smoothed keys re-derive the block from the stored mean, which a lane of this workgroup wrote
        // in pass 1: the fence and the barrier order that store before the loads).  Slow, and only for such tensors.
        if constexpr (SMOOTH) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __syncthreads();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        }
        const float shift = range_shift(sg), sgq = sg * shift;
        for (int slot = 0; slot < nb; ++slot) {
            const int64_t g = block_of(slot);
            if (g >= a.nblk) continue;
            const uint4v *p = (const uint4v *)(a.x + (g << 4));
            const uint4v v0 = p[0], v1 = p[1];
            uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
            if constexpr (SMOOTH) smooth_block16(w, __uint_as_float((uint32_t)a.mean_out[g >> a.row_shift] << 16));
            uint32_t sbyte, c0, c1;
            if constexpr (SEARCH) quantize_block16_4over6_exact(w, shift, sgq, 1.0f / (6.0f * sgq), 1.0f / (4.0f * sgq), sbyte, c0, c1);
            else quantize_block16_exact(w, shift, sgq, 1.0f / (6.0f * sgq), sbyte, c0, c1);
            const int64_t go = output_block((uint32_t)g, a);
            *(uint2v *)(a.codes + (go << 3)) = uint2v{c0, c1};
            a.scales[go] = (uint8_t)sbyte;
        }
        return;
    }
    // ---- pass 2: encode from the on-chip copy, two blocks at a time
    static_for_slots<0, kResRegSlots / 2>([&](auto p_c) {
        constexpr int i = 2 * decltype(p_c)::value;
        if (i < nr) {
            const uint32_t wa[8] = {r0[i].x, r0[i].y, r0[i].z, r0[i].w, r1[i].x, r1[i].y, r1[i].z, r1[i].w};
            const uint32_t wb[8] = {r0[i + 1].x, r0[i + 1].y, r0[i + 1].z, r0[i + 1].w, r1[i + 1].x, r1[i + 1].y, r1[i + 1].z, r1[i + 1].w};
            // (slot i + 1 beyond the slots in use holds zeros and lies past the end of the tensor)
            pair_pass2<SEARCH>(wa, wb, block_of(i), i + 1 < nr ? block_of(i + 1) : a.nblk, a.nblk, sg, inv_6sg, inv_4sg, out, a);
        }
    });
    // The blocks in LDS belong to no wave in particular, so they are handed out from a queue: 64 lanes x 2 slots per
    // item.  The arbiter favours the older of the two waves on a SIMD, which therefore finishes its register slots
    // first and takes more of these items, and the two reach the end of the kernel together.
    const int lane = tid & 63, n_items = ((nl + 1) >> 1) * (kResThreads / 64);
    for (;;) {
        uint32_t ticket = 0;
        if (lane == 0) ticket = atomicAdd(queue_head, 1u);
        const int item = (int)__builtin_amdgcn_readfirstlane(ticket);
        if (item >= n_items) break;                                       // (every wave draws tickets until they run out)
        const int s = (item >> 3) << 1, t = ((item & 7) << 6) + lane;     // first slot of the pair, lane slot in the workgroup
        const uint4v z = {0, 0, 0, 0};
        const bool two = s + 1 < nl;
        const uint4v v0 = lds_blk[(2 * s) * kResThreads + t], v1 = lds_blk[(2 * s + 1) * kResThreads + t];
        const uint4v v2 = two ? lds_blk[(2 * s + 2) * kResThreads + t] : z, v3 = two ? lds_blk[(2 * s + 3) * kResThreads + t] : z;
        const uint32_t wa[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        const uint32_t wb[8] = {v2.x, v2.y, v2.z, v2.w, v3.x, v3.y, v3.z, v3.w};
        const int64_t ga = wg_first + (int64_t)(kResRegSlots + s) * kResThreads + t;
        pair_pass2<SEARCH>(wa, wb, ga, two ? ga + kResThreads : a.nblk, a.nblk, sg, inv_6sg, inv_4sg, out, a);
    }
}

// ---- host side ------------------------------------------------------------------------------------
static uint32_t g_spin_limit = 200000;        // 2 ms in 10 ns ticks
static unsigned g_next_sync_slot = 0;

void set_resident_spin_limit(uint32_t ticks) { g_spin_limit = ticks; }
uint32_t resident_spin_limit() { return g_spin_limit; }

// Whether [rows, C] fits the on-chip path: contiguous rows of whole blocks, at most kResSlots blocks per
// lane on one workgroup per compute unit; smoothing wants a row's blocks inside one wave (as the
// two-pass path does).
bool quantize_rows_resident_fits(int64_t rows, int64_t C, int64_t ld, bool smooth)
{
    if (ld != C || (C & 15) != 0 || rows <= 0) return false;
    const int64_t nblk = rows * (C >> 4);
    if (smooth) {
        const int64_t nb_row = C >> 4;
        if (nb_row > 64 || (nb_row & (nb_row - 1)) != 0) return false;
    }
    return nblk <= (int64_t)kResMaxGrid * kResThreads * kResSlots;
}

// Whether the one-launch form is taken for a tensor that fits.  It fetches the tensor once where the two passes
// fetch it twice, but its encoding runs at two waves per SIMD where the streaming pass has six to eight, and
// measured back to back on cache-like data: for the scale search and the smoothed keys, whose encoding is the
// heavier, the two passes are faster at every size (by 7-14 % from 1 M blocks up to the largest tensor that
// fits); for the plain rule they are faster by 5-11 % from about 0.5 M to 2.5 M blocks, below 0.4 M blocks the
// one launch gains the second launch it does not make, and from 2.5 M blocks (80 MB) on the two forms take the
// same time and the single fetch decides.  mode 1: whenever it fits; mode 2: never.
static int g_one_launch_mode = 0;
void set_one_launch_mode(int mode) { g_one_launch_mode = mode; }
bool quantize_rows_resident_pays(int64_t nblk, bool search_or_smooth)
{
    if (g_one_launch_mode == 1) return true;
    if (g_one_launch_mode == 2) return false;
    constexpr int64_t kSmall = 400000, kLarge = 2500000;
    return !search_or_smooth && (nblk >= kLarge || nblk < kSmall);
}

template <bool SEARCH, bool SMOOTH>
static hipError_t launch_resident(const ResidentArgs &a, int grid, hipStream_t s)
{
    static uint64_t attr_set = 0;              // the dynamic LDS limit is raised once per kernel variant and device
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (((attr_set >> (dev & 63)) & 1u) == 0) {
        hipError_t e = hipFuncSetAttribute((const void *)quantize_rows_resident_kernel<SEARCH, SMOOTH>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kResLdsBytes);
        if (e != hipSuccess) return e;
        attr_set |= 1ull << (dev & 63);
    }
    quantize_rows_resident_kernel<SEARCH, SMOOTH><<<grid, kResThreads, kResLdsBytes, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_quantize_rows_resident(const uint16_t *x, int64_t rows, int64_t C, uint8_t *codes,
                                         uint8_t *scales, float *gs_out, bool scale_search, uint16_t *mean_out,
                                         hipStream_t s, int heads, int slab_heads)
{
    ResidentArgs a{};
    a.x = x;
    a.nblk = rows * (C >> 4);
    const int grid = (int)std::min<int64_t>(kResMaxGrid, (a.nblk + kResThreads - 1) / kResThreads);
    a.row_shift = mean_out ? __builtin_ctzll((unsigned long long)(C >> 4)) : 0;
    a.sync_slot = (int)(g_next_sync_slot++ % kSyncSlots);
    a.spin_limit = g_spin_limit;
    a.codes = codes;
    a.scales = scales;
    a.gs_out = gs_out;
    a.mean_out = mean_out;
    a.nb_row = (uint32_t)(C >> 4);
    a.heads = (uint32_t)heads;
    a.slab_heads = (uint32_t)slab_heads;
    a.tokens = heads > 0 ? (uint32_t)(rows / heads) : 0u;
    if (mean_out) return launch_resident<true, true>(a, grid, s);       // smoothed keys always take the scale search
    return scale_search ? launch_resident<true, false>(a, grid, s) : launch_resident<false, false>(a, grid, s);
}

}  // namespace nvfp4
