// C ABI of the NVFP4 library: argument validation on the host, workspace
// carving, kernel launches on the caller's stream.  See include/nvfp4.h for the
// contract of every entry point.
#include "../../include/nvfp4.h"
#include "nvfp4_kernels.h"

#include <algorithm>
#include <mutex>
#include <vector>

using namespace nvfp4;

// Scratch memory of the allocation-free entry point (nvfp4_kv_quant_noalloc): the partial maxima
// that the ordinary entry points keep in the caller's workspace.  Every GPU the library runs on
// holds its own copy of this array at its own address; in host code the name is only a handle
// for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) uint32_t scratch[kMaxPartials];

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_tensor(const nvfp4_tensor *t)
{
    if (!t || !t->codes || !t->scales || !t->global_scale) return NVFP4_ERR_NULL;
    if (t->rows <= 0 || t->K <= 0 || (t->K & 15) != 0) return NVFP4_ERR_SHAPE;
    if (!aligned16(t->codes) || !aligned16(t->scales)) return NVFP4_ERR_ALIGN;
    return NVFP4_OK;
}

// ---- optional launch timing (benchmarks) -----------------------------------
// When enabled, every entry point records a pair of HIP events around its
// kernels on the caller's stream, tagged with its NVFP4_OP_* id.  Nothing is
// synchronised until nvfp4_timing_read() is called.
std::mutex g_mu;
uint32_t g_timing = 0;          // bit i: entry point i records events
constexpr int kMaxRecords = 8192;
struct Record { hipEvent_t e0, e1; int op; };
std::vector<Record> g_pool;     // events are created once and reused
int g_used = 0;

struct Timed {
    hipStream_t s;
    int slot;
    Timed(hipStream_t st, int op) : s(st), slot(-1)
    {
        if (((g_timing >> op) & 1u) == 0 || g_used >= kMaxRecords) return;
        if (g_used == (int)g_pool.size()) {
            Record r{nullptr, nullptr, op};
            if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return;
            g_pool.push_back(r);
        }
        slot = g_used++;
        g_pool[slot].op = op;
        (void)hipEventRecord(g_pool[slot].e0, s);
    }
    ~Timed()
    {
        if (slot >= 0) (void)hipEventRecord(g_pool[slot].e1, s);
    }
};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
constexpr size_t kPartialBytes = (size_t)kMaxPartials * sizeof(uint32_t);

// Room for one partial maximum per workgroup of the fused GEMM, whatever its launch plan: no
// more than one workgroup per 64 x 64 outputs, plus one extra tile row / column per row chunk
// (chunks are at least 256 rows).
size_t fused_partial_bytes(int64_t M, int64_t N)
{
    const int64_t tm = (M + 63) / 64 + (M + 255) / 256, tn = (N + 63) / 64 + (N + 255) / 256;
    return align_up((size_t)std::max<int64_t>(kMaxPartials, tm * tn) * 4, 256);
}

int quantize_impl(const void *x, int64_t R, int64_t C, int64_t ld, int block_axis,
                  const float *gs_in, nvfp4_tensor *out, void *ws, size_t ws_bytes, hipStream_t s,
                  bool scale_search = false)
{
    if (!x || !out) return NVFP4_ERR_NULL;
    if (int rc = check_tensor(out)) return rc;
    if (block_axis != 0 && block_axis != 1) return NVFP4_ERR_SHAPE;
    if (R <= 0 || C <= 0 || ld < C) return NVFP4_ERR_SHAPE;
    const int64_t rows = block_axis == 0 ? R : C, K = block_axis == 0 ? C : R;
    if ((K & 15) != 0 || (C & 7) != 0) return NVFP4_ERR_SHAPE;
    if (out->rows != rows || out->K != K) return NVFP4_ERR_SHAPE;
    if (!aligned16(x) || (ld & 7) != 0) return NVFP4_ERR_ALIGN;
    if (!gs_in && (!ws || ws_bytes < kPartialBytes)) return NVFP4_ERR_WORKSPACE;
    if (ws && (reinterpret_cast<uintptr_t>(ws) & 3u)) return NVFP4_ERR_ALIGN;

    const uint16_t *xb = static_cast<const uint16_t *>(x);
    uint32_t *partial = static_cast<uint32_t *>(ws);
    int n_partial = 0;
    if (!gs_in && block_axis == 0 && quantize_rows_resident_fits(R, C, ld, false) &&
        quantize_rows_resident_pays(R * (C >> 4), scale_search)) {
        // the tensor fits on the chip (and is of a size at which that pays): one launch, one pass over the input
        hipError_t e = launch_quantize_rows_resident(xb, R, C, out->codes, out->scales, out->global_scale,
                                                     scale_search, nullptr, s);
        return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
    }
    if (!gs_in) {
        if (launch_amax(xb, R, C, ld, partial, &n_partial, s) != hipSuccess) return NVFP4_ERR_LAUNCH;
    }
    hipError_t e = block_axis == 0
                       ? launch_quantize_rows(xb, R, C, ld, gs_in, partial, n_partial, out->codes,
                                              out->scales, out->global_scale, s, scale_search)
                       : launch_quantize_cols(xb, R, C, ld, gs_in, partial, n_partial, out->codes,
                                              out->scales, out->global_scale, s);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

// Device address of `scratch` on the current device, resolved once per device (first call there).
constexpr int kMaxDevices = 64;
uint32_t *g_scratch_ptr[kMaxDevices] = {};
int scratch_on_current_device(uint32_t **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return NVFP4_ERR_LAUNCH;
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return NVFP4_ERR_LAUNCH;
        g_scratch_ptr[dev] = static_cast<uint32_t *>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return NVFP4_OK;
}

int check_gemm(const nvfp4_tensor *A, const nvfp4_tensor *W)
{
    if (int rc = check_tensor(A)) return rc;
    if (int rc = check_tensor(W)) return rc;
    if (A->K != W->K) return NVFP4_ERR_SHAPE;
    return NVFP4_OK;
}

}  // namespace

extern "C" {

int nvfp4_quantize(const void *x_bf16, int64_t R, int64_t C, int64_t ld, int block_axis,
                   const float *global_scale_in, nvfp4_tensor *out, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    std::lock_guard<std::mutex> lk(g_mu);
    Timed t(static_cast<hipStream_t>(stream), NVFP4_OP_QUANTIZE);
    int rc = quantize_impl(x_bf16, R, C, ld, block_axis, global_scale_in, out, workspace, workspace_bytes,
                           static_cast<hipStream_t>(stream));
    return rc;
}

int nvfp4_kv_quant(const void *kv_bf16, int64_t T, int64_t H, int64_t d, nvfp4_tensor *out,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    if (T <= 0 || H <= 0 || d <= 0) return NVFP4_ERR_SHAPE;
    std::lock_guard<std::mutex> lk(g_mu);
    Timed t(static_cast<hipStream_t>(stream), NVFP4_OP_KV_QUANT);
    return quantize_impl(kv_bf16, T * H, d, d, 0, nullptr, out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(stream));
}

int nvfp4_kv_quant_noalloc(const void *kv_bf16, int64_t T, int64_t H, int64_t d, nvfp4_tensor *out,
                           void *stream)
{
    if (T <= 0 || H <= 0 || d <= 0) return NVFP4_ERR_SHAPE;
    // T * H * d <= NVFP4_NOALLOC_MAX_ELEMENTS, tested without forming a product that could overflow
    if (T > NVFP4_NOALLOC_MAX_ELEMENTS / H || T * H > NVFP4_NOALLOC_MAX_ELEMENTS / d) return NVFP4_ERR_SHAPE;
    std::lock_guard<std::mutex> lk(g_mu);
    uint32_t *ws = nullptr;
    if (int rc = scratch_on_current_device(&ws)) return rc;
    // no launch timing here: recording it would create events on first use
    return quantize_impl(kv_bf16, T * H, d, d, 0, nullptr, out, ws, kPartialBytes, static_cast<hipStream_t>(stream));
}

int nvfp4_quantize_4over6(const void *x_bf16, int64_t R, int64_t C, int64_t ld,
                          const float *global_scale_in, nvfp4_tensor *out, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    std::lock_guard<std::mutex> lk(g_mu);
    Timed t(static_cast<hipStream_t>(stream), NVFP4_OP_QUANTIZE_4OVER6);
    return quantize_impl(x_bf16, R, C, ld, 0, global_scale_in, out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(stream), true);
}

int nvfp4_kv_quant_4over6(const void *kv_bf16, int64_t T, int64_t H, int64_t d, nvfp4_tensor *out,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (T <= 0 || H <= 0 || d <= 0) return NVFP4_ERR_SHAPE;
    std::lock_guard<std::mutex> lk(g_mu);
    Timed t(static_cast<hipStream_t>(stream), NVFP4_OP_KV_QUANT_4OVER6);
    return quantize_impl(kv_bf16, T * H, d, d, 0, nullptr, out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(stream), true);
}

int nvfp4_quantize_for_all_to_all(const void *x_bf16, int64_t T, int64_t H, int64_t d, int64_t P,
                                  const float *global_scale_in, nvfp4_tensor *out, void *workspace,
                                  size_t workspace_bytes, void *stream)
{
    if (!x_bf16 || !out) return NVFP4_ERR_NULL;
    if (int rc = check_tensor(out)) return rc;
    if (T <= 0 || H <= 0 || d <= 0 || P <= 0 || (d & 15) != 0 || H % P != 0) return NVFP4_ERR_SHAPE;
    if (out->rows != T * H || out->K != d) return NVFP4_ERR_SHAPE;
    if (!aligned16(x_bf16)) return NVFP4_ERR_ALIGN;
    if (!global_scale_in && (!workspace || workspace_bytes < kPartialBytes)) return NVFP4_ERR_WORKSPACE;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 3u)) return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timed t(s, NVFP4_OP_QUANTIZE_A2A);
    const uint16_t *xb = static_cast<const uint16_t *>(x_bf16);
    uint32_t *partial = static_cast<uint32_t *>(workspace);
    int n_partial = 0;
    if (!global_scale_in && quantize_rows_resident_fits(T * H, d, d, false) && quantize_rows_resident_pays(T * H * (d >> 4), false)) {
        // small enough to stay on the chip between the maximum and the encoding: one launch
        hipError_t e1 = launch_quantize_rows_resident(xb, T * H, d, out->codes, out->scales, out->global_scale, false,
                                                      nullptr, s, (int)H, (int)(H / P));
        return e1 == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
    }
    if (!global_scale_in)
        if (launch_amax(xb, T * H, d, d, partial, &n_partial, s) != hipSuccess) return NVFP4_ERR_LAUNCH;
    hipError_t e = launch_quantize_rows_slabs(xb, T, H, d, (int)(H / P), global_scale_in, partial, n_partial,
                                              out->codes, out->scales, out->global_scale, s);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

int nvfp4_quantize_rht(const void *x_bf16, int64_t R, int64_t C, int64_t ld, uint32_t sign_mask,
                       const float *global_scale_in, nvfp4_tensor *out, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    if (!x_bf16 || !out) return NVFP4_ERR_NULL;
    if (int rc = check_tensor(out)) return rc;
    if (R <= 0 || C <= 0 || ld < C || (R & 15) != 0 || (C & 7) != 0 || (sign_mask >> 16) != 0) return NVFP4_ERR_SHAPE;
    if (out->rows != C || out->K != R) return NVFP4_ERR_SHAPE;
    if (!aligned16(x_bf16) || (ld & 7) != 0) return NVFP4_ERR_ALIGN;
    if (!global_scale_in && (!workspace || workspace_bytes < kPartialBytes)) return NVFP4_ERR_WORKSPACE;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 3u)) return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timed t(s, NVFP4_OP_QUANTIZE_RHT);
    const uint16_t *xb = static_cast<const uint16_t *>(x_bf16);
    uint32_t *partial = static_cast<uint32_t *>(workspace);
    // a workspace of the full size also carries the outcome of pass 1's exactness tests to pass 2
    uint8_t *inexact = (!global_scale_in && workspace_bytes >= kPartialBytes + rht_inexact_bytes(R, C))
                           ? static_cast<uint8_t *>(workspace) + kPartialBytes : nullptr;
    int n_partial = 0;
    if (!global_scale_in)
        if (launch_amax_rht(xb, R, C, ld, sign_mask, partial, &n_partial, inexact, s) != hipSuccess) return NVFP4_ERR_LAUNCH;
    hipError_t e = launch_quantize_cols_rht(xb, R, C, ld, sign_mask, global_scale_in, partial, n_partial,
                                            out->codes, out->scales, out->global_scale, inexact, s);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

int nvfp4_quantize_2d(const void *w_bf16, int64_t R, int64_t C, int64_t ld, const float *global_scale_in,
                      nvfp4_tensor *out, nvfp4_tensor *out_t, void *workspace, size_t workspace_bytes,
                      void *stream)
{
    if (!w_bf16 || !out) return NVFP4_ERR_NULL;
    if (int rc = check_tensor(out)) return rc;
    if (out_t)
        if (int rc = check_tensor(out_t)) return rc;
    if (R <= 0 || C <= 0 || ld < C || (R & 15) != 0 || (C & 15) != 0) return NVFP4_ERR_SHAPE;
    if (out->rows != R || out->K != C) return NVFP4_ERR_SHAPE;
    if (out_t && (out_t->rows != C || out_t->K != R)) return NVFP4_ERR_SHAPE;
    if (!aligned16(w_bf16) || (ld & 7) != 0) return NVFP4_ERR_ALIGN;
    if (!global_scale_in && (!workspace || workspace_bytes < kPartialBytes)) return NVFP4_ERR_WORKSPACE;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 3u)) return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timed t(s, NVFP4_OP_QUANTIZE_2D);
    const uint16_t *xb = static_cast<const uint16_t *>(w_bf16);
    uint32_t *partial = static_cast<uint32_t *>(workspace);
    int n_partial = 0;
    if (!global_scale_in)
        if (launch_amax(xb, R, C, ld, partial, &n_partial, s) != hipSuccess) return NVFP4_ERR_LAUNCH;
    if (launch_quantize_tiles(xb, R, C, ld, global_scale_in, partial, n_partial, out->codes, out->scales,
                              out_t ? out_t->codes : nullptr, out_t ? out_t->scales : nullptr,
                              out->global_scale, out_t ? out_t->global_scale : nullptr, s) != hipSuccess)
        return NVFP4_ERR_LAUNCH;
    return NVFP4_OK;
}

int nvfp4_kv_quant_k(const void *k_bf16, int64_t T, int64_t H, int64_t d, nvfp4_tensor *out,
                     void *row_mean_bf16_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!k_bf16 || !out || !row_mean_bf16_out) return NVFP4_ERR_NULL;
    if (int rc = check_tensor(out)) return rc;
    if (T <= 0 || H <= 0 || d <= 0 || (d & 15) != 0) return NVFP4_ERR_SHAPE;
    const int64_t nb = d >> 4;
    if (nb > 64 || (nb & (nb - 1)) != 0) return NVFP4_ERR_SHAPE;       // the lanes of a row reduce by shuffles
    if (out->rows != T * H || out->K != d) return NVFP4_ERR_SHAPE;
    if (!aligned16(k_bf16) || (reinterpret_cast<uintptr_t>(row_mean_bf16_out) & 1u)) return NVFP4_ERR_ALIGN;
    if (!workspace || workspace_bytes < kPartialBytes) return NVFP4_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 3u) return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timed t(s, NVFP4_OP_KV_QUANT_K);
    const uint16_t *x = static_cast<const uint16_t *>(k_bf16);
    uint16_t *mean = static_cast<uint16_t *>(row_mean_bf16_out);
    uint32_t *partial = static_cast<uint32_t *>(workspace);
    int n_partial = 0;
    if (quantize_rows_resident_fits(T * H, d, d, true) && quantize_rows_resident_pays(T * H * (d >> 4), true)) {
        hipError_t e = launch_quantize_rows_resident(x, T * H, d, out->codes, out->scales, out->global_scale, true,
                                                     mean, s);
        return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
    }
    if (launch_amax_smooth(x, T * H, (int)d, mean, partial, &n_partial, s) != hipSuccess) return NVFP4_ERR_LAUNCH;
    hipError_t e = launch_quantize_rows_smooth(x, T * H, (int)d, mean, partial, n_partial, out->codes,
                                               out->scales, out->global_scale, s);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

int nvfp4_kv_dequant_gather(const nvfp4_kv_chunk *chunks, int n_chunks, void *kv_bf16_out, int64_t H,
                            int64_t d, void *stream)
{
    if (!chunks || !kv_bf16_out) return NVFP4_ERR_NULL;
    if (n_chunks < 1 || n_chunks > NVFP4_KV_MAX_CHUNKS || H <= 0 || d <= 0) return NVFP4_ERR_SHAPE;
    if (!aligned16(kv_bf16_out)) return NVFP4_ERR_ALIGN;
    KvChunkDesc desc[NVFP4_KV_MAX_CHUNKS];
    int64_t blocks = 0;
    for (int c = 0; c < n_chunks; ++c) {
        if (int rc = check_tensor(&chunks[c].q)) return rc;
        if (chunks[c].T <= 0 || chunks[c].q.rows != chunks[c].T * H || chunks[c].q.K != d) return NVFP4_ERR_SHAPE;
        if (reinterpret_cast<uintptr_t>(chunks[c].row_mean_bf16) & 1u) return NVFP4_ERR_ALIGN;
        desc[c] = {chunks[c].q.codes, chunks[c].q.scales, chunks[c].q.global_scale,
                   static_cast<const uint16_t *>(chunks[c].row_mean_bf16), chunks[c].T};
        blocks += chunks[c].T * H * (d >> 4);
    }
    if (blocks / 512 + n_chunks > 0x7FFFFFFF) return NVFP4_ERR_SHAPE;       // one workgroup per 512 blocks
    std::lock_guard<std::mutex> lk(g_mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timed t(s, NVFP4_OP_KV_DEQUANT_GATHER);
    hipError_t e = launch_dequant_gather(desc, n_chunks, H, d, static_cast<uint16_t *>(kv_bf16_out), s);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

int nvfp4_kv_dequant(const nvfp4_tensor *in, void *kv_bf16_out, int64_t T, int64_t H, int64_t d,
                     void *stream)
{
    if (!kv_bf16_out) return NVFP4_ERR_NULL;
    if (int rc = check_tensor(in)) return rc;
    if (T <= 0 || H <= 0 || d <= 0 || in->rows != T * H || in->K != d) return NVFP4_ERR_SHAPE;
    if (!aligned16(kv_bf16_out)) return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    Timed t(static_cast<hipStream_t>(stream), NVFP4_OP_KV_DEQUANT);
    hipError_t e = launch_dequant_bf16(in->codes, in->scales, in->global_scale, in->rows, in->K,
                                       static_cast<uint16_t *>(kv_bf16_out), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

// Outputs larger than the 256 MB Infinity Cache leave through streaming stores: whoever reads them next would not find
// them cached anyway, and the GEMM gains 1-1.5 % (the training shapes write 0.5-1 GB).  Smaller outputs (the FFN's
// H, which the next kernel reads back at once) keep ordinary stores.
static int streams_out(int64_t M, int64_t N, int out_dtype)
{
    return (uint64_t)M * (uint64_t)N * (out_dtype == NVFP4_OUT_BF16 ? 2u : 4u) > (256ull << 20);
}

int nvfp4_gemm(const nvfp4_tensor *A, const nvfp4_tensor *W, void *Y, int64_t ldy, int out_dtype,
               void *stream)
{
    if (!Y) return NVFP4_ERR_NULL;
    if (int rc = check_gemm(A, W)) return rc;
    if (out_dtype != NVFP4_OUT_F32 && out_dtype != NVFP4_OUT_BF16) return NVFP4_ERR_SHAPE;
    if (ldy < W->rows) return NVFP4_ERR_SHAPE;
    // the tiled kernels store 16-byte vectors: every row of Y must start 16-byte aligned
    const bool vec_rows = gemm_is_tiled(A->rows, W->rows, A->K);
    if (!aligned16(Y) || (ldy & ((vec_rows && out_dtype == NVFP4_OUT_BF16) ? 7 : 3)) != 0) return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    Timed t(static_cast<hipStream_t>(stream), NVFP4_OP_GEMM);
    GemmEpilogue ep{};
    ep.out_dtype = out_dtype;
    ep.act = NVFP4_ACT_NONE;
    ep.Y = Y;
    ep.ldy = ldy;
    ep.stream_out = streams_out(A->rows, W->rows, out_dtype);
    hipError_t e = launch_gemm(A->codes, A->scales, A->global_scale, W->codes, W->scales, W->global_scale,
                               A->rows, W->rows, A->K, ep, nullptr, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

int nvfp4_gemm_scale_out(const nvfp4_tensor *A, const nvfp4_tensor *W, void *Y_bf16, int64_t ldy,
                         float *y_global_scale_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Y_bf16 || !y_global_scale_out) return NVFP4_ERR_NULL;
    if (int rc = check_gemm(A, W)) return rc;
    const int64_t M = A->rows, N = W->rows;
    if (ldy < N) return NVFP4_ERR_SHAPE;
    const bool tiled = gemm_is_tiled(M, N, A->K);
    if (!aligned16(Y_bf16) || (ldy & 7) != 0 || (reinterpret_cast<uintptr_t>(y_global_scale_out) & 3u)) return NVFP4_ERR_ALIGN;
    if (!workspace || workspace_bytes < fused_partial_bytes(M, N)) return NVFP4_ERR_WORKSPACE;
    if (!aligned16(workspace)) return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timed t(s, NVFP4_OP_GEMM_SCALE_OUT);
    uint32_t *partial = static_cast<uint32_t *>(workspace);
    GemmEpilogue ep{};
    ep.out_dtype = NVFP4_OUT_BF16;
    ep.act = NVFP4_ACT_NONE;
    ep.Y = Y_bf16;
    ep.ldy = ldy;
    ep.stream_out = tiled && streams_out(M, N, NVFP4_OUT_BF16);
    ep.amax_partial = tiled ? partial : nullptr;        // the tiled kernels' epilogue leaves one maximum per workgroup
    int n_partial = 0;
    if (launch_gemm(A->codes, A->scales, A->global_scale, W->codes, W->scales, W->global_scale, M, N, A->K, ep,
                    &n_partial, s) != hipSuccess)
        return NVFP4_ERR_LAUNCH;
    if (n_partial == 0) {                               // odd shape: the fallback kernel has no such epilogue, one pass over Y
        if (launch_amax(static_cast<const uint16_t *>(Y_bf16), M, N, ldy, partial, &n_partial, s) != hipSuccess)
            return NVFP4_ERR_LAUNCH;
    }
    return launch_scale_from_partials(partial, n_partial, y_global_scale_out, s) == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

int nvfp4_lora_down(const void *x_bf16, int64_t M, int64_t K, int64_t ldx, const void *a_bf16,
                    void *t_bf16, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x_bf16 || !a_bf16 || !t_bf16) return NVFP4_ERR_NULL;
    if (M <= 0 || K <= 0 || (K & 15) != 0 || ldx < K) return NVFP4_ERR_SHAPE;
    if (!aligned16(x_bf16) || !aligned16(a_bf16) || !aligned16(t_bf16) || (ldx & 7) != 0) return NVFP4_ERR_ALIGN;
    if (!workspace || workspace_bytes < lora_down_workspace_bytes(M, K)) return NVFP4_ERR_WORKSPACE;
    if (!aligned16(workspace)) return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timed t(s, NVFP4_OP_LORA_DOWN);
    hipError_t e = launch_lora_down(static_cast<const uint16_t *>(x_bf16), M, K, ldx,
                                    static_cast<const uint16_t *>(a_bf16), static_cast<uint16_t *>(t_bf16),
                                    static_cast<float *>(workspace), s);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

int nvfp4_gemm_lora(const nvfp4_tensor *A, const nvfp4_tensor *W, const void *t_bf16, const void *b_bf16,
                    float lora_scale, void *Y, int64_t ldy, int out_dtype, void *stream)
{
    if (!Y || !t_bf16 || !b_bf16) return NVFP4_ERR_NULL;
    if (int rc = check_gemm(A, W)) return rc;
    if (out_dtype != NVFP4_OUT_F32 && out_dtype != NVFP4_OUT_BF16) return NVFP4_ERR_SHAPE;
    if (ldy < W->rows) return NVFP4_ERR_SHAPE;
    if (!gemm_is_tiled(A->rows, W->rows, A->K)) return NVFP4_ERR_SHAPE;   // K % 64 == 0 and N % 8 == 0 for the fused branch
    if (!aligned16(Y) || (ldy & (out_dtype == NVFP4_OUT_BF16 ? 7 : 3)) != 0 || !aligned16(t_bf16) || !aligned16(b_bf16))
        return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    Timed t(static_cast<hipStream_t>(stream), NVFP4_OP_GEMM_LORA);
    GemmEpilogue ep{};
    ep.out_dtype = out_dtype;
    ep.act = NVFP4_ACT_NONE;
    ep.Y = Y;
    ep.ldy = ldy;
    ep.stream_out = streams_out(A->rows, W->rows, out_dtype);
    LoraBranch lora;
    lora.t = static_cast<const uint16_t *>(t_bf16);
    lora.b = static_cast<const uint16_t *>(b_bf16);
    lora.scale = lora_scale;
    hipError_t e = launch_gemm(A->codes, A->scales, A->global_scale, W->codes, W->scales, W->global_scale,
                               A->rows, W->rows, A->K, ep, nullptr, static_cast<hipStream_t>(stream), lora);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

int nvfp4_gemm_act_quant(const nvfp4_tensor *A, const nvfp4_tensor *W, int act,
                         const float *global_scale_in, nvfp4_tensor *out, void *h_bf16_opt,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (int rc = check_gemm(A, W)) return rc;
    if (int rc = check_tensor(out)) return rc;
    if (act != NVFP4_ACT_NONE && act != NVFP4_ACT_GELU_TANH) return NVFP4_ERR_SHAPE;
    const int64_t M = A->rows, N = W->rows;
    if (out->rows != M || out->K != N) return NVFP4_ERR_SHAPE;
    if (h_bf16_opt && !aligned16(h_bf16_opt)) return NVFP4_ERR_ALIGN;
    const bool tiled = gemm_is_tiled(M, N, A->K);
    const bool single_pass = global_scale_in && tiled;          // the epilogue quantizes, H is not staged
    const size_t part_bytes = fused_partial_bytes(M, N);
    const size_t need = part_bytes + ((h_bf16_opt || single_pass) ? 0 : align_up((size_t)M * (size_t)N * 2, 256));
    if (!workspace || workspace_bytes < need) return NVFP4_ERR_WORKSPACE;
    if (!aligned16(workspace)) return NVFP4_ERR_ALIGN;
    if (tiled && (size_t)gemm_workgroups(M, N, A->K) * 4 > part_bytes) return NVFP4_ERR_WORKSPACE;   // (cannot happen: see fused_partial_bytes)

    std::lock_guard<std::mutex> lk(g_mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timed t(s, NVFP4_OP_GEMM_ACT_QUANT);
    // workspace: [partials][H if not supplied]
    uint32_t *partial = static_cast<uint32_t *>(workspace);
    uint16_t *H = h_bf16_opt ? static_cast<uint16_t *>(h_bf16_opt)
                             : reinterpret_cast<uint16_t *>(static_cast<uint8_t *>(workspace) + part_bytes);
    if (single_pass) {
        // single pass: the GEMM epilogue quantizes its own bf16 tile; H is written only on request
        GemmEpilogue ep{};
        ep.out_dtype = NVFP4_OUT_BF16;
        ep.act = act;
        ep.Y = h_bf16_opt;
        ep.ldy = N;
        ep.q_scale = global_scale_in;
        ep.q_scale_out = out->global_scale;
        ep.q_codes = out->codes;
        ep.q_scales = out->scales;
        Timed tg(s, NVFP4_OP_GEMM_ACT_QUANT_GEMM);
        hipError_t e = launch_gemm(A->codes, A->scales, A->global_scale, W->codes, W->scales,
                                   W->global_scale, M, N, A->K, ep, nullptr, s);
        return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
    }
    GemmEpilogue ep{};
    ep.out_dtype = NVFP4_OUT_BF16;
    ep.act = act;
    ep.Y = H;
    ep.ldy = N;
    ep.amax_partial = (global_scale_in || !tiled) ? nullptr : partial;
    int n_wg = 0;
    {
        Timed tg(s, NVFP4_OP_GEMM_ACT_QUANT_GEMM);
        if (launch_gemm(A->codes, A->scales, A->global_scale, W->codes, W->scales, W->global_scale, M, N,
                        A->K, ep, &n_wg, s) != hipSuccess)
            return NVFP4_ERR_LAUNCH;
    }
    int n_partial = n_wg;
    if (!global_scale_in && n_wg == 0) {   // shape went to the untiled kernel: ordinary amax pass over H
        if (launch_amax(H, M, N, N, partial, &n_partial, s) != hipSuccess) return NVFP4_ERR_LAUNCH;
    }
    hipError_t e = launch_quantize_rows(H, M, N, N, global_scale_in, partial, n_partial, out->codes,
                                        out->scales, out->global_scale, s);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

size_t nvfp4_workspace_bytes(int op, int64_t a, int64_t b, int64_t c)
{
    switch (op) {
    case NVFP4_OP_GEMM_SCALE_OUT: return fused_partial_bytes(a, b);
    case NVFP4_OP_QUANTIZE:
    case NVFP4_OP_KV_QUANT:
    case NVFP4_OP_QUANTIZE_4OVER6:
    case NVFP4_OP_KV_QUANT_4OVER6:
    case NVFP4_OP_KV_QUANT_K:
    case NVFP4_OP_QUANTIZE_2D:
    case NVFP4_OP_QUANTIZE_A2A:
        return kPartialBytes;
    case NVFP4_OP_QUANTIZE_RHT:       // a = R, b = C
        return kPartialBytes + ((a > 0 && b > 0) ? rht_inexact_bytes(a, b) : 0);
    case NVFP4_OP_LORA_DOWN:          // a = M, b = K
        if (a <= 0 || b <= 0) return 0;
        return lora_down_workspace_bytes(a, b);
    case NVFP4_OP_GEMM_ACT_QUANT: {   // a = M, b = N, c: bit 0 = caller supplies H, bit 1 = caller supplies the scale
        if (a <= 0 || b <= 0) return 0;
        // the GEMM tiles (hence the number of per-workgroup maxima) depend on K, which this query
        // does not know: reserve for the smallest tile everywhere
        size_t part = fused_partial_bytes(a, b);
        // with a given scale the fused epilogue needs no staging of H -- unless the shape falls back
        // to the untiled kernel (K % 64 != 0 or N % 8 != 0), which this query cannot see either:
        // only skip the H area when N is a multiple of 16 and leave K to the caller's contract
        const bool need_h = !(c & 1) && !((c & 2) && (b & 15) == 0);
        return part + (need_h ? align_up((size_t)a * (size_t)b * 2, 256) : 0);
    }
    default:
        return 0;
    }
}

const char *nvfp4_status_string(int status)
{
    switch (status) {
    case NVFP4_OK: return "ok";
    case NVFP4_ERR_NULL: return "a required pointer is NULL";
    case NVFP4_ERR_SHAPE: return "bad shape: sizes must be positive, K a multiple of 16, operands must agree";
    case NVFP4_ERR_ALIGN: return "bad alignment: pointers 16-byte aligned, row strides multiples of 8 elements (4 for fp32 outputs)";
    case NVFP4_ERR_WORKSPACE: return "workspace missing or too small (see nvfp4_workspace_bytes)";
    case NVFP4_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    default: return "unknown status";
    }
}

int nvfp4_gemm_plan(int64_t M, int64_t N, int64_t K, char *text, size_t text_bytes)
{
    if (!text) return NVFP4_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || (K & 15) != 0 || text_bytes == 0) return NVFP4_ERR_SHAPE;
    const int n = gemm_plan_text(M, N, K, text, text_bytes);
    return n < 0 ? NVFP4_ERR_WORKSPACE : n;
}

void nvfp4_set_timing(int enabled)
{
    nvfp4_set_timing_ops(enabled != 0 ? 0xffffffffu : 0u);
}

void nvfp4_set_timing_ops(uint32_t op_mask)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_timing = op_mask;
    g_used = 0;
}

int nvfp4_set_one_launch(int mode)
{
    if (mode < NVFP4_ONE_LAUNCH_AUTO || mode > NVFP4_ONE_LAUNCH_NEVER) return NVFP4_ERR_SHAPE;
    std::lock_guard<std::mutex> lk(g_mu);
    set_one_launch_mode(mode);
    return NVFP4_OK;
}

void nvfp4_set_sync_spin_limit(uint32_t ticks_10ns)
{
    std::lock_guard<std::mutex> lk(g_mu);
    set_resident_spin_limit(ticks_10ns == 0xFFFFFFFFu ? 200000u : ticks_10ns);
}

int nvfp4_timing_read_all(int op, float *ms_out, int max_records)
{
    if (!ms_out || max_records < 0) return NVFP4_ERR_NULL;
    std::lock_guard<std::mutex> lk(g_mu);
    int n = 0;
    for (int i = 0; i < g_used && n < max_records; ++i) {
        if (g_pool[i].op != op) continue;
        float ms = 0.0f;
        if (hipEventSynchronize(g_pool[i].e1) != hipSuccess) return NVFP4_ERR_LAUNCH;
        if (hipEventElapsedTime(&ms, g_pool[i].e0, g_pool[i].e1) != hipSuccess) return NVFP4_ERR_LAUNCH;
        ms_out[n++] = ms;
    }
    return n;
}

int nvfp4_probe(int kind, const void *a, void *b, size_t bytes, int iters, void *stream)
{
    if (kind < 0 || kind > 3) return NVFP4_ERR_SHAPE;
    if (!b || (kind != 1 && kind != 3 && !a)) return NVFP4_ERR_NULL;
    if (kind == 3 ? iters <= 0 : (bytes == 0 || (bytes & 15) != 0)) return NVFP4_ERR_SHAPE;
    if (!aligned16(a) || !aligned16(b)) return NVFP4_ERR_ALIGN;
    std::lock_guard<std::mutex> lk(g_mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Timed t(s, NVFP4_OP_PROBE);
    return launch_probe(kind, a, b, (int64_t)bytes, iters, s) == hipSuccess ? NVFP4_OK : NVFP4_ERR_LAUNCH;
}

int nvfp4_timing_read(int op, int *calls, float *total_ms)
{
    std::lock_guard<std::mutex> lk(g_mu);
    int n = 0;
    float sum = 0.0f;
    for (int i = 0; i < g_used; ++i) {
        if (g_pool[i].op != op) continue;
        float ms = 0.0f;
        if (hipEventSynchronize(g_pool[i].e1) != hipSuccess) return NVFP4_ERR_LAUNCH;
        if (hipEventElapsedTime(&ms, g_pool[i].e0, g_pool[i].e1) != hipSuccess) return NVFP4_ERR_LAUNCH;
        sum += ms;
        ++n;
    }
    if (calls) *calls = n;
    if (total_ms) *total_ms = sum;
    return NVFP4_OK;
}

}  // extern "C"
