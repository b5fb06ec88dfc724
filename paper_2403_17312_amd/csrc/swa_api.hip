// C-ABI entry points: argument validation on the host, then kernel launches on the
// caller's stream.  Nothing here allocates, synchronises (except
// swa_check_status) or reads device memory.  Process-wide state: the table of raised LDS
// limits, and the per-device address of the static scratch array below.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include <mutex>
#include <unordered_map>

#include "swa_kernels.hpp"

namespace swa {

int ensure_dynamic_lds(const void* kernel, size_t bytes)
{
    if (bytes <= 48 * 1024) return SWA_OK;
    static std::mutex mu;
    static std::unordered_map<const void*, size_t> granted;
    std::lock_guard<std::mutex> lock(mu);
    auto it = granted.find(kernel);
    if (it != granted.end() && it->second >= bytes) return SWA_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return SWA_ERR_CAPACITY;
    }
    granted[kernel] = bytes;
    return SWA_OK;
}

size_t shared_workspace_offset(const swa_params& p)
{
    const size_t head = kWsArriveOffset + sizeof(int32_t) * (size_t)p.b;
    return (head + 255) & ~(size_t)255;
}

int split_factor(int64_t pairs, int len_bound)
{
    // Four launches instead of one pay only when one workgroup per pair leaves most CUs idle for long:
    // measured break-even near 128 pairs of 4096 rows; below 2048 rows the extra launches cost more
    // than the slices gain.
    if (pairs > 128 || len_bound < 2048) return 1;
    // enough workgroups to put about four on every CU, every slice at least 128 rows long
    int64_t g = (1024 + pairs - 1) / pairs;
    const int by_rows = len_bound / 128;
    if (g > by_rows) g = by_rows;
    if (g > kMaxSplit) g = kMaxSplit;
    return g < 1 ? 1 : (int)g;
}

int decode_stash_rows(const swa_params& p)
{
    // window + a margin for evictions a little behind it; bounded so LDS keeps several
    // workgroups per CU; never more than the cache can hold
    int rows = p.w < 0 ? 48 : ((p.w + 16 + 15) / 16) * 16;
    if (rows > 96) rows = 96;
    const int bound = (p.len_bound > 0 && p.len_bound < p.cap) ? p.len_bound : p.cap;
    if (rows > bound) rows = ((bound + 15) / 16) * 16;
    // long caches (first step after a prompt) take the gather schedule, which has no use for it
    const int rowb = cache_row_bytes(p);
    if ((size_t)((bound + 63) & ~63) * 16 + (size_t)rows * rowb * 2 > 96 * 1024) rows = 0;
    return rows;
}

int decode_block_threads(int64_t pairs, int len_bound, bool kv_int8)
{
    // Measured on MI355X (all five workloads): caches of a thousand slots and more (the first
    // step after a prompt, low sparsity) want 512 threads per pair, shorter ones 256; the pair
    // count matters little.
    if (!kv_int8) return len_bound >= 1024 ? 512 : 256;
    // 8-bit rows are half as long, so a workgroup has half the lanes' worth of work per row and
    // the fixed phases weigh more: smaller workgroups, more of them in flight.
    return (pairs >= 1024 && len_bound < 1024) ? 128 : 256;
}

// Scratch of swa_decode_step_static, the entry point that allocates nothing and takes no
// workspace: status word, arrival counters and (head-shared step) the slabs between the launches.
// One copy per GPU, alive until the process ends, shared by every call on that GPU.  In host code
// this name is only a handle for hipGetSymbolAddress; kernels get the device address.
static __device__ __align__(256) unsigned char scratch[SWA_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];      // device address of `scratch`, per device
static std::mutex g_scratch_mu;

// Device address of this device's scratch array (looked up once per device, with it current).
static int static_scratch(void** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return SWA_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices) return SWA_ERR_BAD_SHAPE;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return SWA_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SWA_OK;
}

__global__ void swa_fill_zero_kernel(int32_t* p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

int launch_workspace_init(const swa_params& p, void* workspace, hipStream_t stream)
{
    const int64_t n = (int64_t)(shared_workspace_offset(p) / 4);   // status word and arrival counters
    hipLaunchKernelGGL(swa_fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                       static_cast<int32_t*>(workspace), n);
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

// Measurement aid: every workgroup streams its own contiguous piece of the buffer with 128-bit
// loads, eight in flight per lane, and folds what it read into one word that is (almost) never
// stored.  What this reaches is the streaming-read ceiling the decode kernel is compared with.
__global__ void __launch_bounds__(256) swa_stream_read_kernel(const Vec16* src, size_t vec_per_block, uint32_t* sink)
{
    const Vec16* base = src + (size_t)blockIdx.x * vec_per_block;
    uint32_t acc = 0;
    for (size_t i = threadIdx.x; i < vec_per_block; i += (size_t)256 * 8) {
        Vec16 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t j = i + (size_t)u * 256;
            v[u] = (j < vec_per_block) ? load16_stream(base + j) : Vec16{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;
}

static int validate(const swa_params* p)
{
    if (!p) return SWA_ERR_NULL;
    if (p->dtype != SWA_F32 && p->dtype != SWA_F16 && p->dtype != SWA_BF16) return SWA_ERR_UNSUPPORTED_DTYPE;
    if (p->d != 64 && p->d != 128) return SWA_ERR_UNSUPPORTED_D;
    if (p->b < 1 || p->h < 1 || p->cap < 1 || p->w < SWA_W_EVEN_SPLIT) return SWA_ERR_BAD_SHAPE;
    if ((int64_t)p->b * p->h > 0x7fffffffLL) return SWA_ERR_BAD_SHAPE;
    if (p->cap > SWA_MAX_CAP) return SWA_ERR_CAPACITY;
    if (p->sparsity_bp < 0 || p->sparsity_bp > 9999) return SWA_ERR_BAD_SPARSITY;
    if (!(p->scale >= 0.f) || isinf(p->scale)) return SWA_ERR_BAD_SHAPE;
    if (p->len_bound < 0) return SWA_ERR_BAD_SHAPE;
    if (p->flags & ~(SWA_FUSE_COMPACTION | SWA_UNORDERED | SWA_HEAD_SHARED | SWA_KV_INT8 | SWA_SPLIT_ROWS)) return SWA_ERR_BAD_SHAPE;
    if ((p->flags & SWA_SPLIT_ROWS) && p->flags != SWA_SPLIT_ROWS) return SWA_ERR_BAD_SHAPE;   // two-call form only
    if ((p->flags & SWA_KV_INT8) && p->dtype != SWA_F16) return SWA_ERR_UNSUPPORTED_DTYPE;
    if ((p->flags & SWA_UNORDERED) && !(p->flags & SWA_FUSE_COMPACTION)) return SWA_ERR_BAD_SHAPE;
    if ((p->flags & SWA_HEAD_SHARED) && !(p->flags & SWA_UNORDERED)) return SWA_ERR_BAD_SHAPE;
    if ((p->flags & SWA_HEAD_SHARED) && p->b > 65535) return SWA_ERR_BAD_SHAPE;   // one grid row per sequence
    return SWA_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static float effective_scale(const swa_params* p)
{
    return p->scale > 0.f ? p->scale : 1.0f / sqrtf((float)p->d);
}

}  // namespace swa

extern "C" {

const char* swa_strerror(int code)
{
    switch (code) {
        case SWA_OK: return "ok";
        case SWA_ERR_NULL: return "a required pointer is NULL";
        case SWA_ERR_BAD_SHAPE: return "b, h, cap, w, scale or R out of range";
        case SWA_ERR_UNSUPPORTED_D: return "head dimension must be 64 or 128";
        case SWA_ERR_UNSUPPORTED_DTYPE: return "dtype must be SWA_F32, SWA_F16 or SWA_BF16";
        case SWA_ERR_BAD_SPARSITY: return "sparsity_bp must be in 0..9999";
        case SWA_ERR_CAPACITY: return "cap exceeds SWA_MAX_CAP, or a sequence's cache was full";
        case SWA_ERR_HIP: return "a HIP runtime call failed";
        case SWA_ERR_ALIGNMENT: return "tensor pointers must be 16-byte aligned";
        case SWA_ERR_HOST_STORE_FULL: return "a host store had no room for the evicted tokens";
        case SWA_ERR_BAD_REQUEST: return "a reload named a token that the host store does not hold";
        default: return "unknown swa_status";
    }
}

size_t swa_workspace_bytes(const swa_params* params)
{
    if (swa::validate(params) != SWA_OK) return 0;
    size_t bytes = swa::shared_workspace_offset(*params);
    if (params->flags & SWA_HEAD_SHARED)
        bytes += sizeof(float) * ((size_t)params->b * params->h * params->cap * 2 + (size_t)params->b * params->h * params->d +
                                  (size_t)params->b * params->cap);
    if (params->flags & SWA_SPLIT_ROWS)
        bytes += sizeof(float) * ((size_t)params->b * params->h * params->cap * 2 +
                                  (size_t)params->b * params->h * swa::kMaxSplit * (params->d + 1) +
                                  (size_t)params->b * params->h);
    return (bytes + 255) & ~(size_t)255;
}

int swa_budget(int32_t n, int32_t m, int32_t w, int32_t sparsity_bp, int32_t* keep, int32_t* n_local,
               int32_t* n_global)
{
    if (!keep || !n_local || !n_global) return SWA_ERR_NULL;
    if (n < 0 || m < 0 || w < SWA_W_EVEN_SPLIT) return SWA_ERR_BAD_SHAPE;
    if (sparsity_bp < 0 || sparsity_bp > 9999) return SWA_ERR_BAD_SPARSITY;
    int32_t w_eff = 0;
    swa::budget(n, m, w, sparsity_bp, *keep, *n_local, *n_global, w_eff);
    return SWA_OK;
}

int swa_workspace_init(const swa_params* params, void* workspace, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (!workspace) return SWA_ERR_NULL;
    return swa::launch_workspace_init(*params, workspace, static_cast<hipStream_t>(stream));
}

int swa_prepare(void)
{
    void* ptr = nullptr;
    int rc = swa::static_scratch(&ptr);
    if (rc != SWA_OK) return rc;
    return swa::prepare_decode();
}

int swa_check_status(const swa_params* params, void* workspace, void* stream, int32_t* status_out)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (!status_out) return SWA_ERR_NULL;
    if (!workspace) {          // the status word of swa_decode_step_static on the current device
        rc = swa::static_scratch(&workspace);
        if (rc != SWA_OK) return rc;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t bits = 0;
    char* ws = static_cast<char*>(workspace) + swa::kWsStatusOffset;
    if (hipMemcpyAsync(&bits, ws, sizeof(bits), hipMemcpyDeviceToHost, st) != hipSuccess) return SWA_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return SWA_ERR_HIP;
    if (bits != 0) {
        hipLaunchKernelGGL(swa::swa_fill_zero_kernel, dim3(1), dim3(64), 0, st, reinterpret_cast<int32_t*>(ws),
                           (int64_t)1);
        if (hipGetLastError() != hipSuccess) return SWA_ERR_HIP;
    }
    *status_out = (bits & swa::kStatusCapacityBit)     ? SWA_ERR_CAPACITY
                  : (bits & swa::kStatusHostStoreBit) ? SWA_ERR_HOST_STORE_FULL
                  : (bits & swa::kStatusBadRequestBit) ? SWA_ERR_BAD_REQUEST
                                                       : SWA_OK;
    return SWA_OK;
}

int swa_prefill_scores(const swa_params* params, const void* q_tail, int32_t R, const void* k_cache,
                       const int32_t* cache_len, float* score, void* workspace, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    (void)workspace;
    if (!q_tail || !k_cache || !cache_len || !score) return SWA_ERR_NULL;
    if (R < 1 || R > SWA_MAX_PREFILL_ROWS) return SWA_ERR_BAD_SHAPE;
    if (!swa::aligned16(q_tail) || !swa::aligned16(k_cache)) return SWA_ERR_ALIGNMENT;
    return swa::launch_prefill(*params, swa::effective_scale(params), q_tail, R, k_cache, cache_len, score, nullptr, false,
                               static_cast<hipStream_t>(stream));
}

int swa_prefill_rows(const swa_params* params, const void* q_tail, int32_t R, const void* k_cache,
                     const int32_t* cache_len, float* ring, void* workspace, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    (void)workspace;
    if (params->flags & SWA_KV_INT8) return SWA_ERR_UNSUPPORTED_DTYPE;
    if (!q_tail || !k_cache || !cache_len || !ring) return SWA_ERR_NULL;
    if (R < 1 || R > SWA_MAX_WINDOW_ROWS) return SWA_ERR_BAD_SHAPE;
    if (!swa::aligned16(q_tail) || !swa::aligned16(k_cache)) return SWA_ERR_ALIGNMENT;
    return swa::launch_prefill(*params, swa::effective_scale(params), q_tail, R, k_cache, cache_len, nullptr, ring, false,
                               static_cast<hipStream_t>(stream));
}

static int decode_common(const swa_params* params, const void* q, const void* k_new, const void* v_new,
                         void* k_cache, void* v_cache, const float* qparams, float* score, int32_t* pos,
                         int32_t* cache_len, const int32_t* seq_len, int32_t* kept_idx, int32_t* kept_cnt,
                         void* out, float* probs_dbg, void* workspace, void* stream, float* ring = nullptr,
                         int32_t ring_rows = 0, int32_t ring_row = 0, bool zero_arrival_counters = false)
{
    const bool fuse = (params->flags & SWA_FUSE_COMPACTION) != 0;
    if (!q || !k_new || !v_new || !k_cache || !v_cache || !score || !pos || !cache_len || !seq_len ||
        (!kept_idx && !fuse) || !kept_cnt || !out || !workspace)
        return SWA_ERR_NULL;
    if (fuse) {
        const int bound = (params->len_bound > 0 && params->len_bound < params->cap) ? params->len_bound : params->cap;
        if (bound > ((params->flags & SWA_UNORDERED) ? SWA_MAX_UNORDERED_SLOTS : SWA_MAX_FUSED_SLOTS)) return SWA_ERR_CAPACITY;
        if (cache_len == kept_cnt) return SWA_ERR_BAD_SHAPE;
    }
    if (!swa::aligned16(q) || !swa::aligned16(k_new) || !swa::aligned16(v_new) || !swa::aligned16(k_cache) ||
        !swa::aligned16(v_cache) || !swa::aligned16(out))
        return SWA_ERR_ALIGNMENT;
    if (zero_arrival_counters) {
        // A fill kernel, not a memset node: callers may capture this call into a graph.
        hipLaunchKernelGGL(swa::swa_fill_zero_kernel, dim3((unsigned)((params->b + 255) / 256)), dim3(256), 0,
                           static_cast<hipStream_t>(stream),
                           reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + swa::kWsArriveOffset),
                           (int64_t)params->b);
        if (hipGetLastError() != hipSuccess) return SWA_ERR_HIP;
    }
    return swa::launch_decode(*params, swa::effective_scale(params), q, k_new, v_new, k_cache, v_cache, score,
                              pos, cache_len, seq_len, kept_idx, kept_cnt, out, probs_dbg, workspace, qparams, ring,
                              ring_rows, ring_row, static_cast<hipStream_t>(stream));
}

int swa_prefill_attention(const swa_params* params, const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* cache_len, void* out, int32_t R, float* score, void* workspace,
                          void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    (void)workspace;
    if (params->flags & SWA_KV_INT8) return SWA_ERR_UNSUPPORTED_DTYPE;
    if (!q || !k_cache || !v_cache || !cache_len || !out) return SWA_ERR_NULL;
    if (R < 0 || R > SWA_MAX_PREFILL_ROWS || (R > 0 && !score)) return R > 0 && !score ? SWA_ERR_NULL : SWA_ERR_BAD_SHAPE;
    if (!swa::aligned16(q) || !swa::aligned16(k_cache) || !swa::aligned16(v_cache) || !swa::aligned16(out))
        return SWA_ERR_ALIGNMENT;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = swa::launch_flash_prefill(*params, swa::effective_scale(params), q, k_cache, v_cache, cache_len, out, st);
    if (rc != SWA_OK || R == 0) return rc;
    return swa::launch_prefill(*params, swa::effective_scale(params), q, R, k_cache, cache_len, score, nullptr, true, st);
}

static int window_common(const swa_params* params, const void* q, const void* k_new, const void* v_new,
                         void* k_cache, void* v_cache, const float* qparams, float* ring, int32_t R,
                         int32_t ring_row, float* score, int32_t* pos, int32_t* cache_len, const int32_t* seq_len,
                         int32_t* kept_idx, int32_t* kept_cnt, void* out, float* probs_dbg, void* workspace,
                         void* stream)
{
    // the ring's columns follow their tokens through the hole-filling compaction only
    const int32_t form = params->flags & ~(SWA_HEAD_SHARED | SWA_KV_INT8);   // (SWA_SPLIT_ROWS is refused here)
    if (form != (SWA_FUSE_COMPACTION | SWA_UNORDERED)) return SWA_ERR_BAD_SHAPE;
    if (!ring) return SWA_ERR_NULL;
    if (R < 1 || R > SWA_MAX_WINDOW_ROWS || ring_row < 0 || ring_row >= R) return SWA_ERR_BAD_SHAPE;
    return decode_common(params, q, k_new, v_new, k_cache, v_cache, qparams, score, pos, cache_len, seq_len,
                         kept_idx, kept_cnt, out, probs_dbg, workspace, stream, ring, R, ring_row);
}

int swa_decode_step_window(const swa_params* params, const void* q, const void* k_new, const void* v_new,
                           void* k_cache, void* v_cache, float* ring, int32_t R, int32_t ring_row, float* score,
                           int32_t* pos, int32_t* cache_len, const int32_t* seq_len, int32_t* kept_idx,
                           int32_t* kept_cnt, void* out, float* probs_dbg, void* workspace, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (params->flags & SWA_KV_INT8) return SWA_ERR_UNSUPPORTED_DTYPE;   // codes need their parameters
    return window_common(params, q, k_new, v_new, k_cache, v_cache, nullptr, ring, R, ring_row, score, pos,
                         cache_len, seq_len, kept_idx, kept_cnt, out, probs_dbg, workspace, stream);
}

int swa_decode_step_window_q8(const swa_params* params, const void* q, const void* k_new, const void* v_new,
                              void* k_codes, void* v_codes, const float* qparams, float* ring, int32_t R,
                              int32_t ring_row, float* score, int32_t* pos, int32_t* cache_len,
                              const int32_t* seq_len, int32_t* kept_idx, int32_t* kept_cnt, void* out,
                              float* probs_dbg, void* workspace, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (!(params->flags & SWA_KV_INT8)) return SWA_ERR_UNSUPPORTED_DTYPE;
    if (!qparams) return SWA_ERR_NULL;
    return window_common(params, q, k_new, v_new, k_codes, v_codes, qparams, ring, R, ring_row, score, pos,
                         cache_len, seq_len, kept_idx, kept_cnt, out, probs_dbg, workspace, stream);
}

int swa_decode_step(const swa_params* params, const void* q, const void* k_new, const void* v_new,
                    void* k_cache, void* v_cache, float* score, int32_t* pos, int32_t* cache_len,
                    const int32_t* seq_len, int32_t* kept_idx, int32_t* kept_cnt, void* out,
                    float* probs_dbg, void* workspace, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (params->flags & SWA_KV_INT8) return SWA_ERR_UNSUPPORTED_DTYPE;   // codes need their parameters
    return decode_common(params, q, k_new, v_new, k_cache, v_cache, nullptr, score, pos, cache_len, seq_len,
                         kept_idx, kept_cnt, out, probs_dbg, workspace, stream);
}

int swa_decode_step_static(const swa_params* params, const void* q, const void* k_new, const void* v_new,
                           void* k_cache, void* v_cache, float* score, int32_t* pos, int32_t* cache_len,
                           const int32_t* seq_len, int32_t* kept_idx, int32_t* kept_cnt, void* out,
                           float* probs_dbg, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (params->flags & SWA_KV_INT8) return SWA_ERR_UNSUPPORTED_DTYPE;
    if (swa_workspace_bytes(params) > (size_t)SWA_STATIC_SCRATCH_BYTES) return SWA_ERR_CAPACITY;
    void* ptr = nullptr;
    rc = swa::static_scratch(&ptr);
    if (rc != SWA_OK) return rc;
    // The arrival counters of the two-call form must start at zero whatever an earlier call (of another
    // shape, or one that was abandoned) left in the shared array; the sticky status word is left alone.
    return decode_common(params, q, k_new, v_new, k_cache, v_cache, nullptr, score, pos, cache_len, seq_len,
                         kept_idx, kept_cnt, out, probs_dbg, ptr, stream, nullptr, 0, 0,
                         !(params->flags & SWA_FUSE_COMPACTION));
}

int swa_decode_step_q8(const swa_params* params, const void* q, const void* k_new, const void* v_new,
                       void* k_codes, void* v_codes, const float* qparams, float* score, int32_t* pos,
                       int32_t* cache_len, const int32_t* seq_len, int32_t* kept_idx, int32_t* kept_cnt,
                       void* out, float* probs_dbg, void* workspace, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (!(params->flags & SWA_KV_INT8)) return SWA_ERR_UNSUPPORTED_DTYPE;
    if (!qparams) return SWA_ERR_NULL;
    return decode_common(params, q, k_new, v_new, k_codes, v_codes, qparams, score, pos, cache_len, seq_len,
                         kept_idx, kept_cnt, out, probs_dbg, workspace, stream);
}

static int check_store(const swa_host_store* st)
{
    if (!st || !st->k || !st->v || !st->score || !st->pos || !st->len) return SWA_ERR_NULL;
    if (st->host_cap < 1) return SWA_ERR_BAD_SHAPE;
    if (!swa::aligned16(st->k) || !swa::aligned16(st->v)) return SWA_ERR_ALIGNMENT;
    return SWA_OK;
}

int swa_offload_evicted(const swa_params* params, const void* k_cache, const void* v_cache, const float* score,
                        const int32_t* pos, const int32_t* kept_idx, const int32_t* kept_cnt,
                        const int32_t* cache_len, const swa_host_store* store, void* workspace, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (!k_cache || !v_cache || !score || !pos || !kept_idx || !kept_cnt || !cache_len || !workspace) return SWA_ERR_NULL;
    rc = check_store(store);
    if (rc != SWA_OK) return rc;
    if (!swa::aligned16(k_cache) || !swa::aligned16(v_cache)) return SWA_ERR_ALIGNMENT;
    return swa::launch_offload(*params, k_cache, v_cache, score, pos, kept_idx, kept_cnt, cache_len, *store, workspace,
                               static_cast<hipStream_t>(stream));
}

int swa_reload_tokens(const swa_params* params, const swa_host_store* store, const int32_t* req_idx,
                      const int32_t* req_cnt, int32_t max_req, void* k_cache, void* v_cache, float* score,
                      int32_t* pos, const int32_t* cache_len, int32_t* new_len, void* workspace, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (!req_idx || !req_cnt || !k_cache || !v_cache || !score || !pos || !cache_len || !new_len || !workspace)
        return SWA_ERR_NULL;
    rc = check_store(store);
    if (rc != SWA_OK) return rc;
    if (max_req < 1 || max_req > params->cap || cache_len == new_len) return SWA_ERR_BAD_SHAPE;
    if (!swa::aligned16(k_cache) || !swa::aligned16(v_cache)) return SWA_ERR_ALIGNMENT;
    return swa::launch_reload(*params, *store, req_idx, req_cnt, max_req, k_cache, v_cache, score, pos, cache_len,
                              new_len, workspace, static_cast<hipStream_t>(stream));
}

int swa_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink) return SWA_ERR_NULL;
    if (!swa::aligned16(src)) return SWA_ERR_ALIGNMENT;
    const size_t piece = 104 * 1024;                    // bytes per workgroup
    const size_t blocks = bytes / piece;
    if (blocks == 0 || blocks > 0x7fffffffULL) return SWA_ERR_BAD_SHAPE;
    hipLaunchKernelGGL(swa::swa_stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const swa::Vec16*>(src), piece / 16,
                       static_cast<uint32_t*>(sink));
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

int swa_quantize_kv(const swa_params* params, const void* k_cache, const void* v_cache,
                    const int32_t* cache_len, void* k_codes, void* v_codes, float* qparams, void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    if (params->dtype != SWA_F16) return SWA_ERR_UNSUPPORTED_DTYPE;
    if (!k_cache || !v_cache || !cache_len || !k_codes || !v_codes || !qparams) return SWA_ERR_NULL;
    if (!swa::aligned16(k_cache) || !swa::aligned16(v_cache) || !swa::aligned16(k_codes) ||
        !swa::aligned16(v_codes))
        return SWA_ERR_ALIGNMENT;
    return swa::launch_quantize(*params, k_cache, v_cache, cache_len, k_codes, v_codes, qparams,
                                static_cast<hipStream_t>(stream));
}

int swa_compact_kv(const swa_params* params, void* k_cache, void* v_cache, float* score, int32_t* pos,
                   const int32_t* kept_idx, const int32_t* kept_cnt, int32_t* cache_len, void* workspace,
                   void* stream)
{
    int rc = swa::validate(params);
    if (rc != SWA_OK) return rc;
    (void)workspace;
    if (!k_cache || !v_cache || !score || !pos || !kept_idx || !kept_cnt || !cache_len) return SWA_ERR_NULL;
    if (!swa::aligned16(k_cache) || !swa::aligned16(v_cache)) return SWA_ERR_ALIGNMENT;
    return swa::launch_compact(*params, k_cache, v_cache, score, pos, kept_idx, kept_cnt, cache_len,
                               static_cast<hipStream_t>(stream));
}

}  // extern "C"
