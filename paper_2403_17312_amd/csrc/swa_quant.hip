// Channel-wise 8-bit compression of an fp16 KV cache (Section V-B): for every (sequence, head)
// pair and every channel, lambda = (max - min) / 255 over the cached tokens and the zero point
// z = nint(-min / lambda); then code = round(x / lambda + z) for every cached element.
// One workgroup per (pair, tensor): a first pass over the rows finds the channel extrema
// (registers, then one LDS reduction over the row groups), a second pass re-reads the rows
// (mostly from L2) and writes the codes.  Runs once, when the prompt's cache is handed over.
#include "swa_kernels.hpp"

namespace swa {

struct QuantArgs {
    const char* src[2];   // fp16 K and V caches
    char* dst[2];         // code caches
    const int32_t* cache_len;
    float* qparams;       // lambda_K, z_K, lambda_V, z_V, each qstride values
    int64_t qstride;
    int32_t h, cap;
};

constexpr float kMinRange = 0.0078125f;   // 2^-7: a flat channel still gets a non-zero scale

template <int D, int NT>
__global__ void __launch_bounds__(NT) swa_quantize_kernel(QuantArgs a)
{
    constexpr int LPR = D / 8;        // lanes per fp16 row, 8 channels each
    constexpr int NG = NT / LPR;      // row groups
    constexpr int ROWB = D * 2;
    __shared__ float s_lo[NG][D];
    __shared__ float s_hi[NG][D];
    __shared__ float s_lam[D];
    __shared__ float s_zero[D];

    const int tid = threadIdx.x;
    const int sub = tid % LPR;
    const int grp = tid / LPR;
    const int64_t pair = blockIdx.x;
    const int which = blockIdx.y;
    const int s = (int)(pair / a.h);
    int len = a.cache_len[s];
    len = len < 0 ? 0 : (len > a.cap ? a.cap : len);
    const char* src = a.src[which] + pair * (int64_t)a.cap * ROWB;
    char* dst = a.dst[which] + pair * (int64_t)a.cap * D;

    float lo[8], hi[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        lo[e] = INFINITY;
        hi[e] = -INFINITY;
    }
    for (int row = grp; row < len; row += NG) {
        float f[8];
        unpack<F16>(load16(src + (int64_t)row * ROWB + sub * 16), f);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            lo[e] = fminf(lo[e], f[e]);
            hi[e] = fmaxf(hi[e], f[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        s_lo[grp][sub * 8 + e] = lo[e];
        s_hi[grp][sub * 8 + e] = hi[e];
    }
    __syncthreads();
    if (tid < D) {
        float l = INFINITY, u = -INFINITY;
        for (int g = 0; g < NG; ++g) {
            l = fminf(l, s_lo[g][tid]);
            u = fmaxf(u, s_hi[g][tid]);
        }
        if (len == 0) l = u = 0.f;
        float range = __fsub_rn(u, l);
        range = range < kMinRange ? kMinRange : range;
        const float lam = __fdiv_rn(range, 255.f);
        const float z = rintf(__fdiv_rn(-l, lam));
        s_lam[tid] = lam;
        s_zero[tid] = z;
        a.qparams[(2 * which) * a.qstride + pair * D + tid] = lam;
        a.qparams[(2 * which + 1) * a.qstride + pair * D + tid] = z;
    }
    __syncthreads();
    float lam[8], zero[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        lam[e] = s_lam[sub * 8 + e];
        zero[e] = s_zero[sub * 8 + e];
    }
    for (int row = grp; row < len; row += NG) {
        float f[8];
        unpack<F16>(load16(src + (int64_t)row * ROWB + sub * 16), f);
        uint32_t w0 = 0u, w1 = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            w0 |= quantise_one(f[e], lam[e], zero[e]) << (8 * e);
            w1 |= quantise_one(f[4 + e], lam[4 + e], zero[4 + e]) << (8 * e);
        }
        *reinterpret_cast<uint2*>(dst + (int64_t)row * D + sub * 8) = make_uint2(w0, w1);
    }
}

int launch_quantize(const swa_params& p, const void* k_cache, const void* v_cache, const int32_t* cache_len,
                    void* k_codes, void* v_codes, float* qparams, hipStream_t stream)
{
    QuantArgs a;
    a.src[0] = static_cast<const char*>(k_cache);
    a.src[1] = static_cast<const char*>(v_cache);
    a.dst[0] = static_cast<char*>(k_codes);
    a.dst[1] = static_cast<char*>(v_codes);
    a.cache_len = cache_len;
    a.qparams = qparams;
    a.qstride = (int64_t)p.b * p.h * p.d;
    a.h = p.h;
    a.cap = p.cap;
    const dim3 grid((unsigned)((int64_t)p.b * p.h), 2);
    constexpr int NT = 256;
    if (p.d == 64) {
        hipLaunchKernelGGL((swa_quantize_kernel<64, NT>), grid, dim3(NT), 0, stream, a);
    } else {
        hipLaunchKernelGGL((swa_quantize_kernel<128, NT>), grid, dim3(NT), 0, stream, a);
    }
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

}  // namespace swa
