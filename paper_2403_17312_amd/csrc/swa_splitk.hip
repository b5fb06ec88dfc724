// Decode step with one pair's rows split over several workgroups (SWA_SPLIT_ROWS): for few
// (sequence, head) pairs with long caches - small batches, long contexts, caches that are compacted
// rarely or never - one workgroup per pair cannot keep the memory system busy.  The step then runs
// as four launches:
//   1. swa_split_logits_kernel   G workgroups per pair: logits q . k_i * scale of a slice of the
//                                cached keys (Eq. 1 numerator), written to the workspace;
//   2. swa_decode_kernel, phase 3 one workgroup per pair: append, softmax over the stored logits,
//                                importance accumulation, budget and selection (Alg. 1 lines 1-5),
//                                kept list and attention weights to memory;
//   3. swa_split_gather_kernel   G workgroups per pair: partial sums  sum p_i v_i  and  sum p_i
//                                over a slice of the kept list (Alg. 1 lines 6-8);
//   4. swa_split_merge_kernel    one workgroup per pair: partials added in slice order, divided,
//                                rounded once to the output type.
// The logits are formed exactly as the one-workgroup kernel forms them (same products, same
// reduction order), so weights, importance and the kept set are bit-identical to that form; only
// the order in which the output's partial sums are added differs.
#include "swa_kernels.hpp"

namespace swa {

struct SplitArgs {
    const char* q;
    const char* k_new;
    const char* v_new;
    const char* k_cache;
    const char* v_cache;
    const int32_t* cache_len;
    const int32_t* kept_idx;
    const int32_t* kept_cnt;
    float* ws_z;        // [pairs, cap] logits
    const float* ws_p;  // [pairs, cap] attention weights of launch 2
    float* ws_part;     // [pairs, G, D + 1] partial outputs and their weight sums
    int32_t* ws_ok;     // [pairs] 1 once launch 2 has finished the pair's step (0: skipped, cache full)
    char* out;
    int32_t h, cap, G;
    float scale;
};

// Launch 1.  cache_len is the length BEFORE the step's append; slot `len` is the new token, whose
// key comes from k_new (launch 2 writes it to the cache).
template <typename T, int D, int NT>
__global__ void __launch_bounds__(NT) swa_split_logits_kernel(SplitArgs a)
{
    constexpr int EPV = Elem<T>::kPerVec;
    constexpr int LPR = D / EPV;
    constexpr int NG = NT / LPR;
    constexpr int ROWB = D * Elem<T>::kBytes;
    constexpr int UK = 8;
    const int tid = threadIdx.x;
    const int sub = tid % LPR;
    const int grp = tid / LPR;
    const int64_t pair = blockIdx.x / a.G;
    const int g = blockIdx.x % a.G;
    const int s = (int)(pair / a.h);
    const int len = a.cache_len[s];
    const int m = len + 1;
    if (g == 0 && tid == 0) a.ws_ok[pair] = 0;         // launch 2 sets it when it completes the pair
    if (len < 0 || m > a.cap) return;                  // launch 2 reports the full cache
    const int per = (m + a.G - 1) / a.G;
    const int lo = g * per;
    const int hi = lo + per < m ? lo + per : m;
    const char* Kp = a.k_cache + pair * (int64_t)a.cap * ROWB;
    float* Zp = a.ws_z + pair * (int64_t)a.cap;
    QFrag<T> qf;
    qf.load(load16(a.q + pair * ROWB + sub * 16));
    const Vec16 nk = load16(a.k_new + pair * ROWB + sub * 16);
    for (int base = lo; base < hi; base += NG * UK) {
        Vec16 kv[UK];
#pragma unroll
        for (int u = 0; u < UK; ++u) {
            const int row = base + u * NG + grp;
            kv[u] = (row < len && row < hi) ? load16_stream(Kp + (int64_t)row * ROWB + sub * 16) : nk;
        }
#pragma unroll
        for (int u = 0; u < UK; ++u) {
            const int row = base + u * NG + grp;
            const float d = group_sum<LPR>(qf.dot(kv[u], 0.f)) * a.scale;
            if (sub == 0 && row < hi) Zp[row] = d;
        }
    }
}

// Launch 3.  Slice g of the kept list of the pair: weighted value rows and their weights.
template <typename T, int D, int NT>
__global__ void __launch_bounds__(NT) swa_split_gather_kernel(SplitArgs a)
{
    constexpr int EPV = Elem<T>::kPerVec;
    constexpr int LPR = D / EPV;
    constexpr int NG = NT / LPR;
    constexpr int NW = NT / kWave;
    constexpr int ROWB = D * Elem<T>::kBytes;
    constexpr int UV = 8;
    __shared__ float s_acc[NW * D];
    __shared__ float s_ps[NW];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int sub = tid % LPR;
    const int grp = tid / LPR;
    const int64_t pair = blockIdx.x / a.G;
    const int g = blockIdx.x % a.G;
    const int s = (int)(pair / a.h);
    if (a.ws_ok[pair] == 0) return;                    // a skipped pair: nothing is written for it
    int keep = a.kept_cnt[s];
    keep = keep < 0 ? 0 : (keep > a.cap ? a.cap : keep);
    const int per = (keep + a.G - 1) / a.G;
    const int lo = g * per;
    const int hi = lo + per < keep ? lo + per : keep;
    const char* Vp = a.v_cache + pair * (int64_t)a.cap * ROWB;
    const float* Pp = a.ws_p + pair * (int64_t)a.cap;
    const int32_t* idx = a.kept_idx + pair * (int64_t)a.cap;
    float acc[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) acc[e] = 0.f;
    float ps = 0.f;
    for (int j0 = lo; j0 < hi; j0 += NG * UV) {
        Vec16 vv[UV];
        float pw[UV];
#pragma unroll
        for (int u = 0; u < UV; ++u) {
            const int j = j0 + u * NG + grp;
            pw[u] = 0.f;
            vv[u] = Vec16{0u, 0u, 0u, 0u};
            if (j < hi) {
                int i = idx[j];
                i = i < 0 ? 0 : (i >= a.cap ? a.cap - 1 : i);
                pw[u] = Pp[i];
                vv[u] = load16_stream(Vp + (int64_t)i * ROWB + sub * 16);
            }
        }
#pragma unroll
        for (int u = 0; u < UV; ++u) {
            float f[EPV];
            unpack<T>(vv[u], f);
#pragma unroll
            for (int e = 0; e < EPV; ++e) acc[e] = __builtin_fmaf(pw[u], f[e], acc[e]);
            ps += pw[u];
        }
    }
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
        ps += __shfl_xor(ps, o, kWave);
    }
    if (lane < LPR) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) s_acc[wave * D + sub * EPV + e] = acc[e];
        if (lane == 0) s_ps[wave] = ps;
    }
    __syncthreads();
    float* part = a.ws_part + (pair * a.G + g) * (int64_t)(D + 1);
    for (int e = tid; e < D; e += NT) {
        float t = 0.f;
#pragma unroll
        for (int v = 0; v < NW; ++v) t += s_acc[v * D + e];
        part[e] = t;
    }
    if (tid == 0) {
        float t = 0.f;
#pragma unroll
        for (int v = 0; v < NW; ++v) t += s_ps[v];
        part[D] = t;
    }
}

// Launch 4.  out = (sum over the slices of the partial sums) / (sum of their weights), slice 0 first.
template <typename T, int D>
__global__ void __launch_bounds__(D) swa_split_merge_kernel(SplitArgs a)
{
    constexpr int ROWB = D * Elem<T>::kBytes;
    const int e = threadIdx.x;
    const int64_t pair = blockIdx.x;
    const int s = (int)(pair / a.h);
    const int keep = a.kept_cnt[s];
    if (a.ws_ok[pair] == 0) return;                    // a skipped (full) sequence: nothing is written
    if (keep <= 0) {                                   // a budget that keeps no token: an empty sum
        store_elem<T>(a.out + pair * ROWB, e, 0.f);
        return;
    }
    const float* part = a.ws_part + pair * a.G * (int64_t)(D + 1);
    float t = 0.f, ps = 0.f;
    for (int g = 0; g < a.G; ++g) {
        t += part[g * (D + 1) + e];
        ps += part[g * (D + 1) + D];
    }
    store_elem<T>(a.out + pair * ROWB, e, t / ps);
}

template <typename T, int D>
static int launch_split_t(const SplitArgs& a, int64_t pairs, int which, hipStream_t stream)
{
    constexpr int NT = 256;
    const dim3 grid((unsigned)(pairs * a.G));
    if (which == 1) {
        hipLaunchKernelGGL((swa_split_logits_kernel<T, D, NT>), grid, dim3(NT), 0, stream, a);
    } else {
        hipLaunchKernelGGL((swa_split_gather_kernel<T, D, NT>), grid, dim3(NT), 0, stream, a);
        if (hipGetLastError() != hipSuccess) return SWA_ERR_HIP;
        hipLaunchKernelGGL((swa_split_merge_kernel<T, D>), dim3((unsigned)pairs), dim3(D), 0, stream, a);
    }
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

// which = 1: the logits launch (before the selection launch); which = 2: gather and merge (after it).
int launch_split(const swa_params& p, float scale, int which, int G, const void* q, const void* k_new,
                 const void* v_new, const void* k_cache, const void* v_cache, const int32_t* cache_len,
                 const int32_t* kept_idx, const int32_t* kept_cnt, float* ws_z, float* ws_p, float* ws_part,
                 int32_t* ws_ok, void* out, hipStream_t stream)
{
    SplitArgs a;
    a.ws_ok = ws_ok;
    a.q = static_cast<const char*>(q);
    a.k_new = static_cast<const char*>(k_new);
    a.v_new = static_cast<const char*>(v_new);
    a.k_cache = static_cast<const char*>(k_cache);
    a.v_cache = static_cast<const char*>(v_cache);
    a.cache_len = cache_len;
    a.kept_idx = kept_idx;
    a.kept_cnt = kept_cnt;
    a.ws_z = ws_z;
    a.ws_p = ws_p;
    a.ws_part = ws_part;
    a.out = static_cast<char*>(out);
    a.h = p.h;
    a.cap = p.cap;
    a.G = G;
    a.scale = scale;
    const int64_t pairs = (int64_t)p.b * p.h;
    if (p.dtype == SWA_F32) {
        return p.d == 64 ? launch_split_t<F32, 64>(a, pairs, which, stream) : launch_split_t<F32, 128>(a, pairs, which, stream);
    } else if (p.dtype == SWA_F16) {
        return p.d == 64 ? launch_split_t<F16, 64>(a, pairs, which, stream) : launch_split_t<F16, 128>(a, pairs, which, stream);
    }
    return p.d == 64 ? launch_split_t<BF16, 64>(a, pairs, which, stream) : launch_split_t<BF16, 128>(a, pairs, which, stream);
}

}  // namespace swa
