// Decode-step Sparse Window Attention: one workgroup per (sequence, head) pair.
//
// A workgroup walks the whole step for its pair without leaving the CU:
//   append -> logits GEMV over the cached keys (Eq. 1) -> softmax -> importance
//   accumulation (running local attention sum, Alg. 1 line 2) -> budget and
//   radix-select of the globally dynamic tokens (Alg. 1 lines 1, 3-5) -> gathered
//   weighted sum of the kept values, renormalised over the kept set (lines 6-8).
// Logits, probabilities, selection keys and the kept list live in LDS, so the
// only HBM traffic is one read of the key rows, one read of the kept value rows,
// one read+write of the importance vector and the index list.
#include "swa_kernels.hpp"

namespace swa {

struct DecodeArgs {
    const char* q;
    const char* k_new;
    const char* v_new;
    char* k_cache;
    char* v_cache;
    float* score;
    int32_t* pos;
    int32_t* cache_len;
    const int32_t* seq_len;
    int32_t* kept_idx;
    int32_t* kept_cnt;
    char* out;
    float* probs_dbg;
    int32_t* status;
    int32_t* arrive;
    int32_t h, cap, cap_pad, w, sparsity_bp;
    float scale;
};

// Monotone map fp32 -> uint32 (larger float <=> larger key).
__device__ __forceinline__ uint32_t order_key(float f)
{
    uint32_t u = f2u(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <typename T, int D, int NT>
__global__ void __launch_bounds__(NT) swa_decode_kernel(DecodeArgs a)
{
    constexpr int EPV = Elem<T>::kPerVec;   // elements per 16-byte vector
    constexpr int LPR = D / EPV;            // lanes per row
    constexpr int NW = NT / kWave;
    constexpr int NG = NT / LPR;            // row groups per workgroup
    constexpr int ROWB = D * Elem<T>::kBytes;
    constexpr int U = 4;                    // independent 16-byte loads in flight per lane

    extern __shared__ __align__(16) char smem[];
    float* s_p = reinterpret_cast<float*>(smem);                       // logits -> probabilities
    uint32_t* s_key = reinterpret_cast<uint32_t*>(s_p + a.cap_pad);    // selection keys
    int32_t* s_kept = reinterpret_cast<int32_t*>(s_key + a.cap_pad);   // ascending kept list
    __shared__ float s_red[16];
    __shared__ int32_t s_hist[256];
    __shared__ int32_t s_wcnt[2][16];
    __shared__ int32_t s_sel[2];
    __shared__ float s_acc[NW * D];
    __shared__ float s_ps[16];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int sub = lane % LPR;
    const int grp = tid / LPR;
    const int64_t pair = blockIdx.x;
    const int s = (int)(pair / a.h);

    const int len = a.cache_len[s];
    const int n = a.seq_len[s];
    const int m = len + 1;
    const bool overflow = (m > a.cap) || (len < 0);

    int keep = 0, n_local = 0, n_global = 0;

    if (!overflow) {
        const int cap = a.cap;
        char* Kp = a.k_cache + pair * (int64_t)cap * ROWB;
        char* Vp = a.v_cache + pair * (int64_t)cap * ROWB;
        float* Sp = a.score + pair * (int64_t)cap;
        const char* knew = a.k_new + pair * ROWB;
        const char* vnew = a.v_new + pair * ROWB;

        // ---- append ---------------------------------------------------------------
        if (tid < LPR) {
            store16(Kp + (int64_t)len * ROWB + tid * 16, load16(knew + tid * 16));
        } else if (tid < 2 * LPR) {
            const int t2 = tid - LPR;
            store16(Vp + (int64_t)len * ROWB + t2 * 16, load16(vnew + t2 * 16));
        } else if (tid == 2 * LPR) {
            a.pos[pair * (int64_t)cap + len] = n - 1;
        }

        // ---- logits: z_i = scale * q . k_i ------------------------------------------
        QFrag<T> qf;
        qf.load(load16(a.q + pair * ROWB + sub * 16));
        for (int base = 0; base < m; base += NG * U) {
            Vec16 kv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = base + u * NG + grp;
                if (row < m) {
                    const char* src = (row == len) ? knew : Kp + (int64_t)row * ROWB;
                    kv[u] = load16(src + sub * 16);
                } else {
                    kv[u] = Vec16{0u, 0u, 0u, 0u};
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = base + u * NG + grp;
                float z = qf.dot(kv[u], 0.f);
#pragma unroll
                for (int o = LPR / 2; o > 0; o >>= 1) z += __shfl_xor(z, o, kWave);
                if (sub == 0 && row < m) s_p[row] = z * a.scale;
            }
        }
        __syncthreads();

        // ---- softmax over the m cached slots ----------------------------------------
        float mx = -INFINITY;
        for (int i = tid; i < m; i += NT) mx = fmaxf(mx, s_p[i]);
        mx = block_max<NT>(mx, s_red);
        float sum = 0.f;
        for (int i = tid; i < m; i += NT) {
            const float e = expf(s_p[i] - mx);
            s_p[i] = e;
            sum += e;
        }
        sum = block_sum<NT>(sum, s_red);

        // ---- importance accumulation --------------------------------------------------
        for (int i = tid; i < m; i += NT) {
            const float p = s_p[i] / sum;
            s_p[i] = p;
            const float old = (i == len) ? 0.f : Sp[i];
            const float sc = old + p;
            Sp[i] = sc;
            s_key[i] = order_key(sc);
        }
        if (a.probs_dbg) {
            float* dbg = a.probs_dbg + pair * (int64_t)cap;
            for (int i = tid; i < cap; i += NT) dbg[i] = (i < m) ? s_p[i] : 0.f;
        }

        // ---- budget + selection -------------------------------------------------------
        budget(n, m, a.w, a.sparsity_bp, keep, n_local, n_global);
        const int ncand = m - n_local;
        __syncthreads();
        if (n_global >= ncand) {
            for (int i = tid; i < m; i += NT) s_kept[i] = i;   // nothing evicted
        } else {
            // radix select: the n_global-th largest key among candidates 0..ncand-1
            uint32_t prefix = 0u, mask = 0u;
            int rem = n_global;
            if (n_global > 0) {
                for (int shift = 24; shift >= 0; shift -= 8) {
                    if (tid < 256) s_hist[tid] = 0;
                    __syncthreads();
                    for (int i = tid; i < ncand; i += NT) {
                        const uint32_t key = s_key[i];
                        if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255u], 1);
                    }
                    __syncthreads();
                    if (wave == 0) {
                        const int c0 = s_hist[4 * lane + 0], c1 = s_hist[4 * lane + 1];
                        const int c2 = s_hist[4 * lane + 2], c3 = s_hist[4 * lane + 3];
                        const int tot = c0 + c1 + c2 + c3;
                        int suf = tot;   // inclusive suffix sum over lanes
#pragma unroll
                        for (int o = 1; o < 64; o <<= 1) {
                            const int t = __shfl_down(suf, o, kWave);
                            if (lane + o < 64) suf += t;
                        }
                        int above = suf - tot;   // keys with a larger digit, in higher lanes
                        const int cs[4] = {c3, c2, c1, c0};
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            if (above < rem && rem <= above + cs[k]) {
                                s_sel[0] = 4 * lane + 3 - k;
                                s_sel[1] = rem - above;
                            }
                            above += cs[k];
                        }
                    }
                    __syncthreads();
                    prefix |= ((uint32_t)s_sel[0]) << shift;
                    mask |= 255u << shift;
                    rem = s_sel[1];
                }
            }
            // Ordered compaction of the kept flags.  A candidate is kept if its key
            // exceeds the threshold, or equals it and is among the first `rem` equals.
            int run_out = 0, run_eq = 0;
            const uint64_t lt = (1ull << lane) - 1ull;
            for (int base = 0; base < m; base += NT) {
                const int i = base + tid;
                const bool is_cand = i < ncand;
                const uint32_t key = is_cand ? s_key[i] : 0u;
                const bool is_eq = is_cand && n_global > 0 && key == prefix;
                const uint64_t eqm = __ballot(is_eq);
                if (lane == 0) s_wcnt[0][wave] = __popcll(eqm);
                __syncthreads();
                int eq_rank = run_eq + __popcll(eqm & lt);
                int eq_all = 0;
#pragma unroll
                for (int v = 0; v < NW; ++v) {
                    const int c = s_wcnt[0][v];
                    if (v < wave) eq_rank += c;
                    eq_all += c;
                }
                const bool kept = (i < m) && (!is_cand || (n_global > 0 && key > prefix) ||
                                              (is_eq && eq_rank < rem));
                const uint64_t km = __ballot(kept);
                if (lane == 0) s_wcnt[1][wave] = __popcll(km);
                __syncthreads();
                int out_pos = run_out + __popcll(km & lt);
                int k_all = 0;
#pragma unroll
                for (int v = 0; v < NW; ++v) {
                    const int c = s_wcnt[1][v];
                    if (v < wave) out_pos += c;
                    k_all += c;
                }
                if (kept) s_kept[out_pos] = i;
                run_eq += eq_all;
                run_out += k_all;
                __syncthreads();
            }
        }
        __syncthreads();

        // ---- kept list to HBM -----------------------------------------------------------
        {
            int32_t* kout = a.kept_idx + pair * (int64_t)cap;
            for (int j = tid; j < keep; j += NT) kout[j] = s_kept[j];
        }

        // ---- sparse attention output: sum_kept p_i v_i / sum_kept p_i ---------------------
        float acc[EPV];
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[e] = 0.f;
        float ps = 0.f;
        for (int j0 = 0; j0 < keep; j0 += NG * U) {
            Vec16 vv[U];
            float pw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = j0 + u * NG + grp;
                if (j < keep) {
                    int idx = s_kept[j];
                    idx = idx < 0 ? 0 : (idx > len ? len : idx);
                    pw[u] = s_p[idx];
                    const char* src = (idx == len) ? vnew : Vp + (int64_t)idx * ROWB;
                    vv[u] = load16(src + sub * 16);
                } else {
                    pw[u] = 0.f;
                    vv[u] = Vec16{0u, 0u, 0u, 0u};
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
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
        if (tid < LPR) {
            float pst = 0.f;
#pragma unroll
            for (int v = 0; v < NW; ++v) pst += s_ps[v];
            float f[EPV];
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                float t = 0.f;
#pragma unroll
                for (int v = 0; v < NW; ++v) t += s_acc[v * D + tid * EPV + e];
                f[e] = t / pst;
            }
            store16(a.out + pair * ROWB + tid * 16, pack<T>(f));
        }
    }

    // ---- per-sequence arrival: the last head to finish publishes the new length --------
    if (tid == 0) {
        if (overflow) {
            atomicOr(a.status, kStatusCapacityBit);
        } else {
            a.kept_cnt[s] = keep;
        }
        __threadfence();
        const int old = atomicAdd(&a.arrive[s], 1);
        if (old == a.h - 1) {
            atomicExch(&a.arrive[s], 0);
            if (!overflow) a.cache_len[s] = m;
        }
    }
}

template <typename T, int D, int NT>
static int launch_decode_nt(const DecodeArgs& a, int64_t pairs, size_t lds_bytes, hipStream_t stream)
{
    auto kern = swa_decode_kernel<T, D, NT>;
    int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes);
    if (rc != SWA_OK) return rc;
    hipLaunchKernelGGL(kern, dim3((unsigned)pairs), dim3(NT), lds_bytes, stream, a);
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

template <typename T, int D>
static int launch_decode_t(const DecodeArgs& a, int64_t pairs, size_t lds_bytes, int nt, hipStream_t stream)
{
    switch (nt) {
        case 256: return launch_decode_nt<T, D, 256>(a, pairs, lds_bytes, stream);
        case 512: return launch_decode_nt<T, D, 512>(a, pairs, lds_bytes, stream);
        default: return launch_decode_nt<T, D, 1024>(a, pairs, lds_bytes, stream);
    }
}

int launch_decode(const swa_params& p, float scale, const void* q, const void* k_new, const void* v_new,
                  void* k_cache, void* v_cache, float* score, int32_t* pos, int32_t* cache_len,
                  const int32_t* seq_len, int32_t* kept_idx, int32_t* kept_cnt, void* out,
                  float* probs_dbg, void* workspace, hipStream_t stream)
{
    DecodeArgs a;
    a.q = static_cast<const char*>(q);
    a.k_new = static_cast<const char*>(k_new);
    a.v_new = static_cast<const char*>(v_new);
    a.k_cache = static_cast<char*>(k_cache);
    a.v_cache = static_cast<char*>(v_cache);
    a.score = score;
    a.pos = pos;
    a.cache_len = cache_len;
    a.seq_len = seq_len;
    a.kept_idx = kept_idx;
    a.kept_cnt = kept_cnt;
    a.out = static_cast<char*>(out);
    a.probs_dbg = probs_dbg;
    a.status = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + kWsStatusOffset);
    a.arrive = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + kWsArriveOffset);
    a.h = p.h;
    a.cap = p.cap;
    a.cap_pad = (p.cap + 63) & ~63;
    a.w = p.w;
    a.sparsity_bp = p.sparsity_bp;
    a.scale = scale;

    const int64_t pairs = (int64_t)p.b * p.h;
    const size_t lds_bytes = (size_t)a.cap_pad * 12;
    // Few pairs per CU: larger workgroups keep more loads in flight per CU.
    const int nt = decode_block_threads(pairs);

    if (p.dtype == SWA_F32) {
        return p.d == 64 ? launch_decode_t<F32, 64>(a, pairs, lds_bytes, nt, stream)
                         : launch_decode_t<F32, 128>(a, pairs, lds_bytes, nt, stream);
    } else if (p.dtype == SWA_F16) {
        return p.d == 64 ? launch_decode_t<F16, 64>(a, pairs, lds_bytes, nt, stream)
                         : launch_decode_t<F16, 128>(a, pairs, lds_bytes, nt, stream);
    } else {
        return p.d == 64 ? launch_decode_t<BF16, 64>(a, pairs, lds_bytes, nt, stream)
                         : launch_decode_t<BF16, 128>(a, pairs, lds_bytes, nt, stream);
    }
}

}  // namespace swa
