// Prefill importance seed on MFMA: the local attention sum of Algorithm 1 line 2
// evaluated at the end of the prompt,
//   score[j] = sum_{r<R} softmax_causal(Q_tail K^T * scale)[r, j].
// One workgroup (4 waves) per (sequence, head) pair.  The R x s logit tile is
// never stored: pass 1 computes every query row's max and normaliser, pass 2
// recomputes the logits and reduces exp(z - max_r) / sum_r over the rows.
//
// MFMA operand layout used here (32x32 tiles, wave64): lane l supplies row
// (l % 32) of its operand and the contiguous half-row (l / 32) of the head
// dimension; successive MFMA issues walk along that half-row.  Both operands
// use the same walk, so the contraction is over the whole head dimension
// whatever order the hardware sums in.  The 32x32 fp32 result gives lane l
// column (l % 32) and rows 8*(i/4) + 4*(l/32) + (i%4), i = 0..15.
//   pass 1: A = key tile,   B = query tile -> lane owns ONE query, 16 keys
//           (row statistics reduce inside the lane);
//   pass 2: A = query tile, B = key tile   -> lane owns ONE key, 16 queries
//           (column sums reduce inside the lane).
#include "swa_kernels.hpp"

namespace swa {

struct PrefillArgs {
    const char* q_tail;
    const char* k_cache;
    const int32_t* cache_len;
    float* score;   // column sums over the R rows, or NULL
    float* rows;    // [b,h,R,cap] the R rows themselves, or NULL
    int32_t h, cap, R;
    int32_t q_in_place;   // 0: q_tail is [b,h,R,d]; 1: it is the whole prompt's [b,h,cap,d] and the
                          //    R rows are the ones at positions cache_len-R .. cache_len-1
    float scale_log2e;
};

// Merge two (max, sum-of-exp2) pairs of disjoint key sets.
__device__ __forceinline__ void merge_stats(float& M, float& L, float M2, float L2)
{
    const float Mn = fmaxf(M, M2);
    if (Mn == -INFINITY) return;   // both empty
    const float a = (M == -INFINITY) ? 0.f : L * exp2f(M - Mn);
    const float b = (M2 == -INFINITY) ? 0.f : L2 * exp2f(M2 - Mn);
    M = Mn;
    L = a + b;
}

// WR: also write the R rows themselves (the ring of the strict local attention sum).
template <typename T, int D, int RT, bool WR>
__global__ void __launch_bounds__(256) swa_prefill_kernel(PrefillArgs a)
{
    constexpr int NT = 256;
    constexpr int NW = NT / kWave;
    constexpr int ROWB = D * Elem<T>::kBytes;
    constexpr int NV = (ROWB / 2) / 16;   // 16-byte vectors per lane and tile row
    constexpr int RP = RT * 32;           // padded query rows

    __shared__ float s_m[NW][RP];
    __shared__ float s_l[NW][RP];
    __shared__ __align__(16) float s_M[RP];
    __shared__ __align__(16) float s_invL[RP];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int hb = lane >> 5;
    const int64_t pair = blockIdx.x;
    const int cap = a.cap;
    const int R = a.R;
    int s = a.cache_len[pair / a.h];
    s = s > cap ? cap : s;
    float* Sp = a.score ? a.score + pair * (int64_t)cap : nullptr;
    float* Rp = WR ? a.rows + pair * (int64_t)R * cap : nullptr;

    if (s <= 0) {
        if (Sp)
            for (int j = tid; j < cap; j += NT) Sp[j] = 0.f;
        if (Rp)
            for (int j = tid; j < R * cap; j += NT) Rp[j] = 0.f;
        return;
    }

    const char* Kp = a.k_cache + pair * (int64_t)cap * ROWB;
    const int qbase = a.q_in_place ? s - R : 0;   // row index of query 0 (negative: rows before the prompt)
    const char* Qp = a.q_tail + pair * (int64_t)(a.q_in_place ? cap : R) * ROWB;

    // Lane (row, hb) supplies the 16-byte chunks 2v + hb, v = 0..NV-1, of its row: the two
    // half-wave lanes of a row read adjacent chunks, and query and key fragments use the same
    // walk, so every MFMA issue contracts matching slices of the head dimension.
    const int lane_off = hb * 16;

    // Query fragments stay in registers for both passes.  Rows >= R are zero.
    Vec16 qv[RT][NV];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int r = rt * 32 + l32;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int qrow = qbase + r > 0 ? qbase + r : 0;          // rows before the prompt are masked below
            qv[rt][v] = (r < R) ? load16(Qp + (int64_t)qrow * ROWB + v * 32 + lane_off)
                                : Vec16{0u, 0u, 0u, 0u};
        }
    }

    const int ntiles = (s + 31) / 32;
    const int t_off = s - R;   // query r sits at position t_off + r and sees keys 0..t_off+r

    // Unconditional tile load (rows past the end re-read the last row and are masked later), so
    // that the loads of the next tile can stay in flight while the current one is reduced.
    // Plain loads, not streaming ones: a lane takes 32 bytes of a line per instruction, so the line
    // has to survive in the cache between the instructions that consume it.
    auto load_tile = [&](int tile, Vec16(&kv)[NV]) {
        int krow = tile * 32 + l32;
        krow = krow < s ? krow : s - 1;
        krow = krow < 0 ? 0 : krow;
        const char* src = Kp + (int64_t)krow * ROWB + lane_off;
#pragma unroll
        for (int v = 0; v < NV; ++v) kv[v] = load16(src + v * 32);
    };

    // ------------------------------ pass 1: row statistics ------------------------------
    float M[RT], L[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        M[rt] = -INFINITY;
        L[rt] = 0.f;
    }
    auto stats_tile = [&](int tile, const Vec16(&kv)[NV]) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            float16_t c;
#pragma unroll
            for (int i = 0; i < 16; ++i) c[i] = 0.f;
#pragma unroll
            for (int v = 0; v < NV; ++v) c = Mfma<T>::run(kv[v], qv[rt][v], c);   // C[key][query]
            const int r = rt * 32 + l32;
            const int tmax = (r < R) ? t_off + r : -1;   // last visible key of this lane's query
            float z[16];
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = tile * 32 + 8 * (i / 4) + 4 * hb + (i % 4);
                z[i] = (key <= tmax) ? c[i] * a.scale_log2e : -INFINITY;
                mx = fmaxf(mx, z[i]);
            }
            if (mx > -INFINITY) {
                const float Mn = fmaxf(M[rt], mx);
                float acc = L[rt] * __builtin_amdgcn_exp2f(M[rt] - Mn);   // 0 while M is -inf
#pragma unroll
                for (int i = 0; i < 16; ++i) acc += __builtin_amdgcn_exp2f(z[i] - Mn);
                M[rt] = Mn;
                L[rt] = acc;
            }
        }
    };
    {
        Vec16 kA[NV], kB[NV];
        load_tile(wave, kA);
        for (int tile = wave; tile < ntiles; tile += 2 * NW) {
            load_tile(tile + NW, kB);
            stats_tile(tile, kA);
            load_tile(tile + 2 * NW, kA);
            if (tile + NW < ntiles) stats_tile(tile + NW, kB);
        }
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const float M2 = __shfl_xor(M[rt], 32, kWave);
        const float L2 = __shfl_xor(L[rt], 32, kWave);
        merge_stats(M[rt], L[rt], M2, L2);
        if (hb == 0) {
            s_m[wave][rt * 32 + l32] = M[rt];
            s_l[wave][rt * 32 + l32] = L[rt];
        }
    }
    __syncthreads();
    if (tid < RP) {
        float Mt = s_m[0][tid], Lt = s_l[0][tid];
#pragma unroll
        for (int v = 1; v < NW; ++v) merge_stats(Mt, Lt, s_m[v][tid], s_l[v][tid]);
        const bool ok = Mt > -INFINITY && Lt > 0.f;
        s_M[tid] = ok ? Mt : 0.f;
        s_invL[tid] = ok ? 1.f / Lt : 0.f;
    }
    __syncthreads();

    // ------------------------------ pass 2: column sums ---------------------------------
    auto colsum_tile = [&](int tile, const Vec16(&kv)[NV]) {
        const int key = tile * 32 + l32;
        float colsum = 0.f;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            float16_t c;
#pragma unroll
            for (int i = 0; i < 16; ++i) c[i] = 0.f;
#pragma unroll
            for (int v = 0; v < NV; ++v) c = Mfma<T>::run(qv[rt][v], kv[v], c);   // C[query][key]
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                // the lane's rows 8g + 4hb .. +3 of this query tile: one 16-byte LDS read each
                const int r0 = rt * 32 + 8 * g + 4 * hb;
                const float4_t Mr = *reinterpret_cast<const float4_t*>(&s_M[r0]);
                const float4_t Ir = *reinterpret_cast<const float4_t*>(&s_invL[r0]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = r0 + j;
                    const bool vis = (r < R) && (key <= t_off + r);
                    const float p = __builtin_amdgcn_exp2f(c[4 * g + j] * a.scale_log2e - Mr[j]) * Ir[j];
                    colsum += vis ? p : 0.f;
                    if constexpr (WR) {
                        if (r < R && key < s) Rp[(int64_t)r * cap + key] = vis ? p : 0.f;
                    }
                }
            }
        }
        colsum += __shfl_xor(colsum, 32, kWave);
        if (Sp && hb == 0 && key < s) Sp[key] = colsum;
    };
    {
        Vec16 kA[NV], kB[NV];
        // the keys read last by pass 1 are read first here
        const int last = ntiles - 1 - wave;
        load_tile(last, kA);
        for (int tile = last; tile >= 0; tile -= 2 * NW) {
            load_tile(tile - NW, kB);
            colsum_tile(tile, kA);
            load_tile(tile - 2 * NW, kA);
            if (tile - NW >= 0) colsum_tile(tile - NW, kB);
        }
    }
    if (Sp)
        for (int j = s + tid; j < cap; j += NT) Sp[j] = 0.f;
    if (Rp)
        for (int r = 0; r < R; ++r)
            for (int j = s + tid; j < cap; j += NT) Rp[(int64_t)r * cap + j] = 0.f;
}

template <typename T, int D>
static int launch_prefill_t(const PrefillArgs& a, int64_t pairs, hipStream_t stream)
{
    const int rt = (a.R + 31) / 32;
    const dim3 grid((unsigned)pairs), block(256);
    if (a.rows) {
        switch (rt) {
            case 1: hipLaunchKernelGGL((swa_prefill_kernel<T, D, 1, true>), grid, block, 0, stream, a); break;
            case 2: hipLaunchKernelGGL((swa_prefill_kernel<T, D, 2, true>), grid, block, 0, stream, a); break;
            default: return SWA_ERR_BAD_SHAPE;
        }
    } else {
        switch (rt) {
            case 1: hipLaunchKernelGGL((swa_prefill_kernel<T, D, 1, false>), grid, block, 0, stream, a); break;
            case 2: hipLaunchKernelGGL((swa_prefill_kernel<T, D, 2, false>), grid, block, 0, stream, a); break;
            case 3: hipLaunchKernelGGL((swa_prefill_kernel<T, D, 3, false>), grid, block, 0, stream, a); break;
            case 4: hipLaunchKernelGGL((swa_prefill_kernel<T, D, 4, false>), grid, block, 0, stream, a); break;
            default: return SWA_ERR_BAD_SHAPE;
        }
    }
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

int launch_prefill(const swa_params& p, float scale, const void* q_tail, int32_t R, const void* k_cache,
                   const int32_t* cache_len, float* score, float* rows, bool q_in_place, hipStream_t stream)
{
    PrefillArgs a;
    a.q_in_place = q_in_place ? 1 : 0;
    a.rows = rows;
    a.q_tail = static_cast<const char*>(q_tail);
    a.k_cache = static_cast<const char*>(k_cache);
    a.cache_len = cache_len;
    a.score = score;
    a.h = p.h;
    a.cap = p.cap;
    a.R = R;
    a.scale_log2e = scale * 1.44269504088896340736f;
    const int64_t pairs = (int64_t)p.b * p.h;
    if (p.dtype == SWA_F32) {
        return p.d == 64 ? launch_prefill_t<F32, 64>(a, pairs, stream) : launch_prefill_t<F32, 128>(a, pairs, stream);
    } else if (p.dtype == SWA_F16) {
        return p.d == 64 ? launch_prefill_t<F16, 64>(a, pairs, stream) : launch_prefill_t<F16, 128>(a, pairs, stream);
    } else {
        return p.d == 64 ? launch_prefill_t<BF16, 64>(a, pairs, stream) : launch_prefill_t<BF16, 128>(a, pairs, stream);
    }
}

}  // namespace swa
