// In-place compaction of the KV cache to the kept set: row kept_idx[j] of K, V,
// score and pos moves to slot j (the gather of Algorithm 1 line 6 applied to the
// cache itself).  One workgroup per (sequence, head) pair.
//
// The kept list is ascending, so kept_idx[j] >= j: a row never moves to a
// higher slot.  Rows are handled in ascending chunks; within a chunk every
// source is read into registers before any destination is written (one barrier),
// and a later chunk's sources all lie above an earlier chunk's destinations, so
// no unread row is ever overwritten.  The prefix with kept_idx[j] == j is
// skipped: only the rows behind the first hole move.
#include "swa_kernels.hpp"

namespace swa {

struct CompactArgs {
    char* k_cache;
    char* v_cache;
    float* score;
    int32_t* pos;
    const int32_t* kept_idx;
    const int32_t* kept_cnt;
    int32_t* cache_len;
    int32_t h, cap;
};

template <int ROWB, int NT>
__global__ void __launch_bounds__(NT) swa_compact_kernel(CompactArgs a)
{
    constexpr int LPR = ROWB / 16;   // lanes per row
    constexpr int NG = NT / LPR;     // rows per workgroup per load
    constexpr int U = 4;
    constexpr int CH = NG * U;       // rows per chunk
    static_assert(CH <= NT, "score/pos of a chunk are moved by the first CH threads");

    const int tid = threadIdx.x;
    const int sub = tid % LPR;
    const int grp = tid / LPR;
    const int64_t pair = blockIdx.x;
    const int s = (int)(pair / a.h);
    const int cap = a.cap;
    int cnt = a.kept_cnt[s];
    cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);

    const int32_t* idx = a.kept_idx + pair * (int64_t)cap;
    char* Kp = a.k_cache + pair * (int64_t)cap * ROWB;
    char* Vp = a.v_cache + pair * (int64_t)cap * ROWB;
    float* Sp = a.score + pair * (int64_t)cap;
    int32_t* Pp = a.pos + pair * (int64_t)cap;

    // first j with kept_idx[j] != j (the predicate is monotone for an ascending list)
    int lo = 0, hi = cnt;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (idx[mid] == mid) lo = mid + 1; else hi = mid;
    }

    for (int c0 = lo; c0 < cnt; c0 += CH) {
        Vec16 kk[U], vv[U];
        int dst[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = c0 + u * NG + grp;
            dst[u] = -1;
            if (j < cnt) {
                int src = idx[j];
                src = src < 0 ? 0 : (src >= cap ? cap - 1 : src);
                kk[u] = load16_stream(Kp + (int64_t)src * ROWB + sub * 16);
                vv[u] = load16_stream(Vp + (int64_t)src * ROWB + sub * 16);
                dst[u] = j;
            }
        }
        float sc = 0.f;
        int32_t ps = 0;
        const int jj = c0 + tid;
        const bool mv = tid < CH && jj < cnt;
        if (mv) {
            int src = idx[jj];
            src = src < 0 ? 0 : (src >= cap ? cap - 1 : src);
            sc = Sp[src];
            ps = Pp[src];
        }
        // every source of the chunk is in registers before any destination is written
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (dst[u] >= 0) {
                store16(Kp + (int64_t)dst[u] * ROWB + sub * 16, kk[u]);
                store16(Vp + (int64_t)dst[u] * ROWB + sub * 16, vv[u]);
            }
        }
        if (mv) {
            Sp[jj] = sc;
            Pp[jj] = ps;
        }
    }
    if (tid == 0 && pair % a.h == 0) a.cache_len[s] = cnt;
}

int launch_compact(const swa_params& p, void* k_cache, void* v_cache, float* score, int32_t* pos,
                   const int32_t* kept_idx, const int32_t* kept_cnt, int32_t* cache_len,
                   hipStream_t stream)
{
    CompactArgs a;
    a.k_cache = static_cast<char*>(k_cache);
    a.v_cache = static_cast<char*>(v_cache);
    a.score = score;
    a.pos = pos;
    a.kept_idx = kept_idx;
    a.kept_cnt = kept_cnt;
    a.cache_len = cache_len;
    a.h = p.h;
    a.cap = p.cap;
    const int64_t pairs = (int64_t)p.b * p.h;
    const int rowb = cache_row_bytes(p);
    constexpr int NT = 256;
    switch (rowb) {
        case 64: hipLaunchKernelGGL((swa_compact_kernel<64, NT>), dim3((unsigned)pairs), dim3(NT), 0, stream, a); break;
        case 128: hipLaunchKernelGGL((swa_compact_kernel<128, NT>), dim3((unsigned)pairs), dim3(NT), 0, stream, a); break;
        case 256: hipLaunchKernelGGL((swa_compact_kernel<256, NT>), dim3((unsigned)pairs), dim3(NT), 0, stream, a); break;
        case 512: hipLaunchKernelGGL((swa_compact_kernel<512, NT>), dim3((unsigned)pairs), dim3(NT), 0, stream, a); break;
        default: return SWA_ERR_UNSUPPORTED_D;
    }
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

}  // namespace swa
