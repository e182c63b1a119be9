// Ceiling probes for the benchmark: what this GPU sustains for plain streaming reads, writes and
// copies of HBM, and for back-to-back v_mfma_f32_32x32x16_f16 on register-resident operands.  They
// are not part of the NVFP4 path; the streaming kernels and the GEMM are judged against them.
#include "nvfp4_device.h"
#include "nvfp4_kernels.h"

namespace nvfp4 {

// Each workgroup streams one contiguous stretch of the buffer, four 16-byte vectors per lane in flight.  Contiguous
// stretches per workgroup sustain about a fifth more than the same loop at a grid-wide stride (reads 6.9 against
// 5.7 TB/s, writes 5.9 against 4.4, copies 5.7 against 4.5 on the 1 GiB buffers of the benchmark), and the grids
// below are the best of 512 .. 16384 workgroups for each kind.
constexpr int kProbeThreads = 256, kProbeGridRead = 4096, kProbeGridWrite = 4096, kProbeGridCopy = 16384;

struct ProbeRange { int64_t begin, end; };
__device__ __forceinline__ ProbeRange probe_range(int64_t nvec)
{
    const int64_t per = (nvec + gridDim.x - 1) / gridDim.x, b = per * blockIdx.x;
    return {b, b + per < nvec ? b + per : nvec};
}

// every 16-byte vector of the buffer is read once; the XOR of what a workgroup read goes to sink[]
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const uint4v *__restrict__ src, int64_t nvec,
                                                                   uint32_t *__restrict__ sink)
{
    uint4v acc = {0, 0, 0, 0};
    const ProbeRange r = probe_range(nvec);
    int64_t i = r.begin + threadIdx.x;
    for (; i + 3 * kProbeThreads < r.end; i += 4 * kProbeThreads) {
        const uint4v a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + kProbeThreads);
        const uint4v c = __builtin_nontemporal_load(src + i + 2 * kProbeThreads), d = __builtin_nontemporal_load(src + i + 3 * kProbeThreads);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < r.end; i += kProbeThreads) acc ^= __builtin_nontemporal_load(src + i);
    const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9E3779B9u) sink[blockIdx.x] = x;                // practically never true: the loads cannot be dropped
}

__global__ __launch_bounds__(kProbeThreads) void probe_write_kernel(uint4v *__restrict__ dst, int64_t nvec, uint32_t seed)
{
    const ProbeRange r = probe_range(nvec);
    const uint4v v = {seed, seed + 1, seed + 2, seed + threadIdx.x};
    for (int64_t i = r.begin + threadIdx.x; i < r.end; i += kProbeThreads) dst[i] = v;
}

__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(const uint4v *__restrict__ src, uint4v *__restrict__ dst,
                                                                   int64_t nvec)
{
    const ProbeRange r = probe_range(nvec);
    int64_t i = r.begin + threadIdx.x;
    for (; i + 3 * kProbeThreads < r.end; i += 4 * kProbeThreads) {
        const uint4v a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + kProbeThreads);
        const uint4v c = __builtin_nontemporal_load(src + i + 2 * kProbeThreads), d = __builtin_nontemporal_load(src + i + 3 * kProbeThreads);
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + kProbeThreads);
        __builtin_nontemporal_store(c, dst + i + 2 * kProbeThreads);
        __builtin_nontemporal_store(d, dst + i + 3 * kProbeThreads);
    }
    for (; i < r.end; i += kProbeThreads) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// 64 MFMAs per iteration on sixteen accumulators; the operands are eight register-resident fragments, a
// different pair for every MFMA, holding what the GEMM feeds the matrix pipes: products of a pseudo-random
// E2M1 code and a pseudo-random E4M3 block scale (2^-4 .. 2^3), as f16.  The matrix pipes draw more power
// on changing operands than on constant ones, and the clock they sustain depends on it, so a ceiling
// measured on constants (or on full-mantissa noise) would not be the GEMM's.
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, uint32_t seed, float *__restrict__ sink)
{
    uint4v frag[8];
#pragma unroll
    for (int f = 0; f < 8; ++f) {
        uint32_t x = (seed + 977u * f + 40503u * threadIdx.x + 7919u * blockIdx.x) * 2654435761u;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
            const uint32_t sbyte = 24u + ((x >> 8) % 56u);                 // E4M3 2^-4 .. 2^3 with any mantissa
            const half2v sc = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(sbyte | (sbyte << 8), 1.0f, false);
            const half2v e = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(x, 1.0f, 0);
            frag[f][q] = __builtin_bit_cast(uint32_t, e * sc);
        }
    }
    float16v acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int rep = 0; rep < 4; ++rep)
#pragma unroll
            for (int t = 0; t < 16; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8v, frag[4 + (t >> 2)]),
                                                                __builtin_bit_cast(half8v, frag[(t + rep) & 3]), acc[t], 0, 0, 0);
#pragma unroll
        for (int f = 0; f < 8; ++f) asm volatile("" : "+v"(frag[f]));      // nothing of the loop body can be hoisted
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = s;
}

hipError_t launch_probe(int kind, const void *a, void *b, int64_t bytes, int iters, hipStream_t s)
{
    const int64_t nvec = bytes >> 4;
    switch (kind) {
    case 0: probe_read_kernel<<<kProbeGridRead, kProbeThreads, 0, s>>>((const uint4v *)a, nvec, (uint32_t *)b); break;
    case 1: probe_write_kernel<<<kProbeGridWrite, kProbeThreads, 0, s>>>((uint4v *)b, nvec, 0x01234567u); break;
    case 2: probe_copy_kernel<<<kProbeGridCopy, kProbeThreads, 0, s>>>((const uint4v *)a, (uint4v *)b, nvec); break;
    case 3: probe_mfma_kernel<<<256, 256, 0, s>>>(iters, 0x2545F491u, (float *)b); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace nvfp4
