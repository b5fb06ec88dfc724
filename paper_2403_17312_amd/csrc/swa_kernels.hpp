// Host-side launch interface between the C-ABI entry points and the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "swa.h"
#include "swa_device.hpp"

namespace swa {

// Raises the dynamic-LDS limit of a kernel when a launch needs more than the default.  The
// limits already granted are remembered per process (one mutex-guarded table): the only state
// the library keeps besides the address of the static scratch array.
int ensure_dynamic_lds(const void* kernel, size_t bytes);

// Raises that limit for every instantiation of the decode kernel on the current device.
int prepare_decode();

// Threads per workgroup of the decode kernel for this many (sequence, head) pairs, this bound on
// the cached length and this cache format.
int decode_block_threads(int64_t pairs, int len_bound, bool kv_int8);

// Byte offset, inside the caller's workspace, of the slabs the head-shared step passes from its
// first launch to its second (present only when SWA_HEAD_SHARED is set).
size_t shared_workspace_offset(const swa_params& p);

// Bytes of one cache row.
inline int cache_row_bytes(const swa_params& p)
{
    return (p.flags & SWA_KV_INT8) ? p.d : p.d * (p.dtype == SWA_F32 ? 4 : 2);
}

// Rows of K and V the fused-compaction decode parks in LDS (0 = none).
int decode_stash_rows(const swa_params& p);

int launch_workspace_init(const swa_params& p, void* workspace, hipStream_t stream);

int launch_decode(const swa_params& p, float scale, const void* q, const void* k_new, const void* v_new,
                  void* k_cache, void* v_cache, float* score, int32_t* pos, int32_t* cache_len,
                  const int32_t* seq_len, int32_t* kept_idx, int32_t* kept_cnt, void* out,
                  float* probs_dbg, void* workspace, const float* qparams, float* ring, int32_t ring_rows,
                  int32_t ring_row, hipStream_t stream);

// Channel-wise 8-bit compression of an fp16 cache (Section V-B): parameters from the cached rows,
// then the codes.  qparams: four fp32 arrays of b*h*d values (lambda_K, z_K, lambda_V, z_V).
int launch_quantize(const swa_params& p, const void* k_cache, const void* v_cache, const int32_t* cache_len,
                    void* k_codes, void* v_codes, float* qparams, hipStream_t stream);

int launch_compact(const swa_params& p, void* k_cache, void* v_cache, float* score, int32_t* pos,
                   const int32_t* kept_idx, const int32_t* kept_cnt, int32_t* cache_len,
                   hipStream_t stream);

int launch_prefill(const swa_params& p, float scale, const void* q_tail, int32_t R, const void* k_cache,
                   const int32_t* cache_len, float* score, float* rows, bool q_in_place, hipStream_t stream);

// SWA_SPLIT_ROWS: workgroups per pair for this many pairs and this bound on the cached length
// (1 = the one-workgroup kernel serves the call), and the launches around the selection launch
// (which = 1: logits of every cached key to ws_z; which = 2: output from ws_p and the kept list).
constexpr int kMaxSplit = 16;
int split_factor(int64_t pairs, int len_bound);
int launch_split(const swa_params& p, float scale, int which, int G, const void* q, const void* k_new,
                 const void* v_new, const void* k_cache, const void* v_cache, const int32_t* cache_len,
                 const int32_t* kept_idx, const int32_t* kept_cnt, float* ws_z, float* ws_p, float* ws_part,
                 int32_t* ws_ok, void* out, hipStream_t stream);

// Token-level offload tier (Section V-A, Algorithm 2): evicted rows to the host store, requested rows back.
int launch_offload(const swa_params& p, const void* k_cache, const void* v_cache, const float* score,
                   const int32_t* pos, const int32_t* kept_idx, const int32_t* kept_cnt, const int32_t* cache_len,
                   const swa_host_store& st, void* workspace, hipStream_t stream);
int launch_reload(const swa_params& p, const swa_host_store& st, const int32_t* req_idx, const int32_t* req_cnt,
                  int32_t max_req, void* k_cache, void* v_cache, float* score, int32_t* pos,
                  const int32_t* cache_len, int32_t* new_len, void* workspace, hipStream_t stream);

// Causal attention over the whole prompt (Eq. 1-2) on MFMA: out[t] for every prompt position.
int launch_flash_prefill(const swa_params& p, float scale, const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* cache_len, void* out, hipStream_t stream);

}  // namespace swa
