// Token-level offload tier: the store and load halves of the GPU-CPU caching phase of the
// paper's dynamic scheduling (Section V-A, Algorithm 2, Phase II: tokens that leave GPU memory are
// stored in CPU memory, tokens that are needed again are loaded back).  Tokens are moved one
// (sequence, head) row at a time, never whole heads: that is the point of token-level scheduling.
//
// The host store is pinned host memory that the device addresses directly; a workgroup copies its
// pair's rows with 16-byte vector accesses, so a row crosses the bus as whole 256-byte bursts.
// Which tokens to offload is decided by the decode step (everything it did not keep); which to load
// back is the caller's policy (the scheduler of Algorithm 2 is not part of this library).
#include "swa_kernels.hpp"

namespace swa {

struct OffloadArgs {
    const char* k_cache;
    const char* v_cache;
    const float* score;
    const int32_t* pos;
    const int32_t* kept_idx;
    const int32_t* kept_cnt;
    const int32_t* cache_len;
    char* hk;
    char* hv;
    float* hs;
    int32_t* hp;
    int32_t* hlen;
    int32_t* status;
    int32_t h, cap, host_cap, lds_slots;
};

// Every slot of [0, cache_len) that is not in the kept list goes to the end of the pair's host store,
// in ascending slot order.  cache_len is the length after swa_decode_step (the new token counted),
// the cache itself must not have been compacted yet.
template <int ROWB, int NT>
__global__ void __launch_bounds__(NT) swa_offload_kernel(OffloadArgs a)
{
    constexpr int LPR = ROWB / 16;
    constexpr int NG = NT / LPR;
    constexpr int NW = NT / kWave;
    constexpr int U = 4;
    extern __shared__ __align__(16) char smem[];
    uint16_t* s_list = reinterpret_cast<uint16_t*>(smem);                 // evicted slots, ascending
    unsigned char* s_kept = reinterpret_cast<unsigned char*>(s_list + a.lds_slots);
    __shared__ int32_t s_wcnt[16];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int sub = tid % LPR;
    const int grp = tid / LPR;
    const int64_t pair = blockIdx.x;
    const int s = (int)(pair / a.h);
    const int cap = a.cap;
    int m = a.cache_len[s];
    if (m > cap || m > a.lds_slots) {               // longer than the call was sized for: skipped, reported
        if (tid == 0) atomicOr(a.status, kStatusCapacityBit);
        return;
    }
    m = m < 0 ? 0 : m;
    int cnt = a.kept_cnt[s];
    cnt = cnt < 0 ? 0 : (cnt > m ? m : cnt);

    const int32_t* idx = a.kept_idx + pair * (int64_t)cap;
    for (int i = tid; i < m; i += NT) s_kept[i] = 0;
    __syncthreads();
    for (int j = tid; j < cnt; j += NT) {
        const int i = idx[j];
        if (i >= 0 && i < m) s_kept[i] = 1;
    }
    __syncthreads();

    // ordered compaction of the slots that were not kept
    int run = 0;
    const uint64_t lt = (1ull << lane) - 1ull;
    for (int base = 0; base < m; base += NT) {
        const int i = base + tid;
        const bool ev = i < m && s_kept[i] == 0;
        const uint64_t em = __ballot(ev);
        if (lane == 0) s_wcnt[wave] = __popcll(em);
        __syncthreads();
        int r = run + __popcll(em & lt);
        int all = 0;
#pragma unroll
        for (int v = 0; v < NW; ++v) {
            const int c = s_wcnt[v];
            if (v < wave) r += c;
            all += c;
        }
        if (ev) s_list[r] = (uint16_t)i;
        run += all;
        __syncthreads();
    }
    const int E = run;
    const int hl = a.hlen[pair];
    if (E == 0) return;
    if (hl < 0 || hl + E > a.host_cap) {            // no room: nothing of this pair is written
        if (tid == 0) atomicOr(a.status, kStatusHostStoreBit);
        return;
    }

    const char* Kp = a.k_cache + pair * (int64_t)cap * ROWB;
    const char* Vp = a.v_cache + pair * (int64_t)cap * ROWB;
    char* HK = a.hk + (pair * (int64_t)a.host_cap + hl) * ROWB;
    char* HV = a.hv + (pair * (int64_t)a.host_cap + hl) * ROWB;
    for (int k0 = 0; k0 < E; k0 += NG * U) {
        Vec16 kk[U], vv[U];
        int dst[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = k0 + u * NG + grp;
            dst[u] = -1;
            if (k < E) {
                const int src = s_list[k];
                kk[u] = load16_stream(Kp + (int64_t)src * ROWB + sub * 16);
                vv[u] = load16_stream(Vp + (int64_t)src * ROWB + sub * 16);
                dst[u] = k;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (dst[u] >= 0) {
                store16(HK + (int64_t)dst[u] * ROWB + sub * 16, kk[u]);
                store16(HV + (int64_t)dst[u] * ROWB + sub * 16, vv[u]);
            }
        }
    }
    const float* Sp = a.score + pair * (int64_t)cap;
    const int32_t* Pp = a.pos + pair * (int64_t)cap;
    float* HS = a.hs + pair * (int64_t)a.host_cap + hl;
    int32_t* HP = a.hp + pair * (int64_t)a.host_cap + hl;
    for (int k = tid; k < E; k += NT) {
        const int src = s_list[k];
        HS[k] = Sp[src];
        HP[k] = Pp[src];
    }
    if (tid == 0) a.hlen[pair] = hl + E;
}

struct ReloadArgs {
    const char* hk;
    const char* hv;
    const float* hs;
    const int32_t* hp;
    const int32_t* hlen;
    const int32_t* req_idx;
    const int32_t* req_cnt;
    char* k_cache;
    char* v_cache;
    float* score;
    int32_t* pos;
    const int32_t* cache_len;
    int32_t* new_len;
    int32_t* status;
    int32_t h, cap, host_cap, max_req;
};

// Tokens req_idx[0 .. req_cnt) of the pair's host store are appended to its cache.
template <int ROWB, int NT>
__global__ void __launch_bounds__(NT) swa_reload_kernel(ReloadArgs a)
{
    constexpr int LPR = ROWB / 16;
    constexpr int NG = NT / LPR;
    constexpr int U = 4;
    const int tid = threadIdx.x;
    const int sub = tid % LPR;
    const int grp = tid / LPR;
    const int64_t pair = blockIdx.x;
    const int s = (int)(pair / a.h);
    const int cap = a.cap;
    const int len = a.cache_len[s];
    int r = a.req_cnt[s];
    r = r < 0 ? 0 : (r > a.max_req ? a.max_req : r);
    const bool head0 = pair - (int64_t)s * a.h == 0;
    if (len < 0 || len + r > cap) {                 // no room in the cache: the sequence is skipped
        if (tid == 0) {
            atomicOr(a.status, kStatusCapacityBit);
            if (head0) a.new_len[s] = len;
        }
        return;
    }
    const int hl = a.hlen[pair];
    const int32_t* req = a.req_idx + pair * (int64_t)a.max_req;
    const char* HK = a.hk + pair * (int64_t)a.host_cap * ROWB;
    const char* HV = a.hv + pair * (int64_t)a.host_cap * ROWB;
    char* Kp = a.k_cache + (pair * (int64_t)cap + len) * ROWB;
    char* Vp = a.v_cache + (pair * (int64_t)cap + len) * ROWB;
    bool bad = false;
    for (int k0 = 0; k0 < r; k0 += NG * U) {
        Vec16 kk[U], vv[U];
        int dst[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = k0 + u * NG + grp;
            dst[u] = -1;
            if (k < r) {
                int src = req[k];
                if (src < 0 || src >= hl) {         // not a token of the store: slot 0 stands in, reported
                    bad = true;
                    src = 0;
                }
                if (hl > 0) {
                    kk[u] = load16(HK + (int64_t)src * ROWB + sub * 16);
                    vv[u] = load16(HV + (int64_t)src * ROWB + sub * 16);
                } else {
                    kk[u] = Vec16{0u, 0u, 0u, 0u};
                    vv[u] = Vec16{0u, 0u, 0u, 0u};
                }
                dst[u] = k;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (dst[u] >= 0) {
                store16(Kp + (int64_t)dst[u] * ROWB + sub * 16, kk[u]);
                store16(Vp + (int64_t)dst[u] * ROWB + sub * 16, vv[u]);
            }
        }
    }
    float* Sp = a.score + pair * (int64_t)cap + len;
    int32_t* Pp = a.pos + pair * (int64_t)cap + len;
    const float* HS = a.hs + pair * (int64_t)a.host_cap;
    const int32_t* HP = a.hp + pair * (int64_t)a.host_cap;
    for (int k = tid; k < r; k += NT) {
        int src = req[k];
        if (src < 0 || src >= hl) {
            bad = true;
            src = 0;
        }
        Sp[k] = hl > 0 ? HS[src] : 0.f;
        Pp[k] = hl > 0 ? HP[src] : -1;
    }
    if (bad) atomicOr(a.status, kStatusBadRequestBit);
    if (tid == 0 && head0) a.new_len[s] = len + r;
}

int launch_offload(const swa_params& p, const void* k_cache, const void* v_cache, const float* score,
                   const int32_t* pos, const int32_t* kept_idx, const int32_t* kept_cnt, const int32_t* cache_len,
                   const swa_host_store& st, void* workspace, hipStream_t stream)
{
    OffloadArgs a;
    a.k_cache = static_cast<const char*>(k_cache);
    a.v_cache = static_cast<const char*>(v_cache);
    a.score = score;
    a.pos = pos;
    a.kept_idx = kept_idx;
    a.kept_cnt = kept_cnt;
    a.cache_len = cache_len;
    a.hk = static_cast<char*>(st.k);
    a.hv = static_cast<char*>(st.v);
    a.hs = st.score;
    a.hp = st.pos;
    a.hlen = st.len;
    a.status = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + kWsStatusOffset);
    a.h = p.h;
    a.cap = p.cap;
    a.host_cap = st.host_cap;
    const int bound = (p.len_bound > 0 && p.len_bound < p.cap) ? p.len_bound : p.cap;
    a.lds_slots = (bound + 63) & ~63;
    const size_t lds = (size_t)a.lds_slots * 3;
    const int64_t pairs = (int64_t)p.b * p.h;
    const int rowb = cache_row_bytes(p);
    constexpr int NT = 256;
    const dim3 grid((unsigned)pairs), block(NT);
    switch (rowb) {
        case 64: hipLaunchKernelGGL((swa_offload_kernel<64, NT>), grid, block, lds, stream, a); break;
        case 128: hipLaunchKernelGGL((swa_offload_kernel<128, NT>), grid, block, lds, stream, a); break;
        case 256: hipLaunchKernelGGL((swa_offload_kernel<256, NT>), grid, block, lds, stream, a); break;
        case 512: hipLaunchKernelGGL((swa_offload_kernel<512, NT>), grid, block, lds, stream, a); break;
        default: return SWA_ERR_UNSUPPORTED_D;
    }
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

int launch_reload(const swa_params& p, const swa_host_store& st, const int32_t* req_idx, const int32_t* req_cnt,
                  int32_t max_req, void* k_cache, void* v_cache, float* score, int32_t* pos,
                  const int32_t* cache_len, int32_t* new_len, void* workspace, hipStream_t stream)
{
    ReloadArgs a;
    a.hk = static_cast<const char*>(st.k);
    a.hv = static_cast<const char*>(st.v);
    a.hs = st.score;
    a.hp = st.pos;
    a.hlen = st.len;
    a.req_idx = req_idx;
    a.req_cnt = req_cnt;
    a.k_cache = static_cast<char*>(k_cache);
    a.v_cache = static_cast<char*>(v_cache);
    a.score = score;
    a.pos = pos;
    a.cache_len = cache_len;
    a.new_len = new_len;
    a.status = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + kWsStatusOffset);
    a.h = p.h;
    a.cap = p.cap;
    a.host_cap = st.host_cap;
    a.max_req = max_req;
    const int64_t pairs = (int64_t)p.b * p.h;
    const int rowb = cache_row_bytes(p);
    constexpr int NT = 256;
    const dim3 grid((unsigned)pairs), block(NT);
    switch (rowb) {
        case 64: hipLaunchKernelGGL((swa_reload_kernel<64, NT>), grid, block, 0, stream, a); break;
        case 128: hipLaunchKernelGGL((swa_reload_kernel<128, NT>), grid, block, 0, stream, a); break;
        case 256: hipLaunchKernelGGL((swa_reload_kernel<256, NT>), grid, block, 0, stream, a); break;
        case 512: hipLaunchKernelGGL((swa_reload_kernel<512, NT>), grid, block, 0, stream, a); break;
        default: return SWA_ERR_UNSUPPORTED_D;
    }
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

}  // namespace swa
