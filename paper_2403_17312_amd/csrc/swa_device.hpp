// Device-side helpers shared by the SWA kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "swa.h"

namespace swa {

constexpr int kWave = 64;

// Workspace layout (device memory supplied by the caller):
//   int32 status                     sticky error bits
//   int32 arrive[b]  (at +64 bytes)  per-sequence arrival counters of decode steps
constexpr size_t kWsStatusOffset = 0;
constexpr size_t kWsArriveOffset = 64;
constexpr int32_t kStatusCapacityBit = 1;      // a cache was full (or longer than len_bound)
constexpr int32_t kStatusHostStoreBit = 2;     // a pair's host store had no room for its evicted tokens
constexpr int32_t kStatusBadRequestBit = 4;    // a reload asked for a token the host store does not hold

struct F32 {};
struct F16 {};
struct BF16 {};
struct Q8 {};   // cache rows hold 8-bit codes (Section V-B); queries, new rows and outputs are fp16

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

// One 16-byte vector of cache elements, as loaded by one lane.
struct alignas(16) Vec16 {
    uint32_t x, y, z, w;
};

template <typename T>
struct Elem;
template <>
struct Elem<F32> {
    static constexpr int kBytes = 4;
    static constexpr int kPerVec = 4;
};
template <>
struct Elem<F16> {
    static constexpr int kBytes = 2;
    static constexpr int kPerVec = 8;
};
template <>
struct Elem<BF16> {
    static constexpr int kBytes = 2;
    static constexpr int kPerVec = 8;
};

template <>
struct Elem<Q8> {
    static constexpr int kBytes = 1;
    static constexpr int kPerVec = 16;
};

// Type of the per-step rows (q, k_new, v_new, out) that go with a cache element type.
template <typename T>
struct Act {
    typedef T type;
};
template <>
struct Act<Q8> {
    typedef F16 type;
};

__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }

__device__ __forceinline__ float bf16_lo(uint32_t u) { return u2f(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return u2f(u & 0xffff0000u); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

// Two fp32 values rounded to bf16 (nearest even) in one dword: v_cvt_pk_bf16_f32 on gfx950.
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_bits(float lo, float hi)
{
    const float2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    return f32x2_to_bf16x2_bits(f, 0.f) & 0xffffu;
}

__device__ __forceinline__ uint32_t f32_to_f16_bits(float f)
{
    _Float16 h = (_Float16)f;
    return (uint32_t) __builtin_bit_cast(uint16_t, h);
}

// Widen the elements of one 16-byte vector to fp32.
template <typename T>
__device__ __forceinline__ void unpack(const Vec16& v, float* f);
template <>
__device__ __forceinline__ void unpack<F32>(const Vec16& v, float* f)
{
    f[0] = u2f(v.x); f[1] = u2f(v.y); f[2] = u2f(v.z); f[3] = u2f(v.w);
}
template <>
__device__ __forceinline__ void unpack<F16>(const Vec16& v, float* f)
{
    half8_t h = __builtin_bit_cast(half8_t, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = (float)h[i];
}
template <>
__device__ __forceinline__ void unpack<BF16>(const Vec16& v, float* f)
{
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}

template <>
__device__ __forceinline__ void unpack<Q8>(const Vec16& v, float* f)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[4 * i + 0] = (float)(w[i] & 0xffu);
        f[4 * i + 1] = (float)((w[i] >> 8) & 0xffu);
        f[4 * i + 2] = (float)((w[i] >> 16) & 0xffu);
        f[4 * i + 3] = (float)(w[i] >> 24);
    }
}

// Section V-B: code = round(x / lambda + z), saturated to 8 bits.  One IEEE rounding per
// operation (no reciprocal, no contraction), ties to even: the code is an integer decision and
// has to come out the same wherever it is taken.
__device__ __forceinline__ uint32_t quantise_one(float x, float lam, float z)
{
    float t = __fdiv_rn(x, lam);
    t = __fadd_rn(t, z);
    t = rintf(t);
    t = t < 0.f ? 0.f : (t > 255.f ? 255.f : t);
    return (uint32_t)t;
}

// Partial dot product of one 16-byte key vector with the matching query vector,
// fp32 accumulation.  Query operand: the raw vector for F16 (packed dot), the
// widened fp32 values otherwise.
template <typename T>
struct QFrag;
template <>
struct QFrag<F32> {
    float f[4];
    __device__ __forceinline__ void load(const Vec16& v) { unpack<F32>(v, f); }
    __device__ __forceinline__ float dot(const Vec16& k, float acc) const
    {
        acc = __builtin_fmaf(u2f(k.x), f[0], acc);
        acc = __builtin_fmaf(u2f(k.y), f[1], acc);
        acc = __builtin_fmaf(u2f(k.z), f[2], acc);
        acc = __builtin_fmaf(u2f(k.w), f[3], acc);
        return acc;
    }
};
template <>
struct QFrag<F16> {
    Vec16 raw;
    __device__ __forceinline__ void load(const Vec16& v) { raw = v; }
    __device__ __forceinline__ float dot(const Vec16& k, float acc) const
    {
        // v_dot2_f32_f16: exact fp16 products, fp32 accumulation
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.x), __builtin_bit_cast(half2_t, raw.x), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.y), __builtin_bit_cast(half2_t, raw.y), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.z), __builtin_bit_cast(half2_t, raw.z), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.w), __builtin_bit_cast(half2_t, raw.w), acc, false);
        return acc;
    }
};
template <>
struct QFrag<BF16> {
    Vec16 raw;
    __device__ __forceinline__ void load(const Vec16& v) { raw = v; }
    __device__ __forceinline__ float dot(const Vec16& k, float acc) const
    {
        // v_dot2c_f32_bf16 (gfx950): bf16 products are exact in fp32, accumulation in fp32
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.x), __builtin_bit_cast(bf16x2_t, raw.x), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.y), __builtin_bit_cast(bf16x2_t, raw.y), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.z), __builtin_bit_cast(bf16x2_t, raw.z), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.w), __builtin_bit_cast(bf16x2_t, raw.w), acc, false);
        return acc;
    }
};

// Compressed keys: q . k = sum_c q_c lambda_c (code_c - z_c), so the query is scaled by the
// channel's lambda once and the zero-point term becomes a per-lane constant; the inner loop is
// one convert and one FMA per code.
template <>
struct QFrag<Q8> {
    float f[16];
    float c0;
    // qs[c] = q_c lambda_c and qz[c] = q_c lambda_c z_c for this lane's 16 channels
    __device__ __forceinline__ void load(const float* qs, const float* qz)
    {
        c0 = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            f[i] = qs[i];
            c0 -= qz[i];
        }
    }
    __device__ __forceinline__ float dot(const Vec16& k, float acc) const
    {
        float c[16];
        unpack<Q8>(k, c);
        acc += c0;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc = __builtin_fmaf(c[i], f[i], acc);
        return acc;
    }
};

// One 32x32 MFMA step over a 16-byte operand vector per lane: lane l supplies row (l % 32) of its
// operand and the k-slice (l / 32); the fp32 result gives lane l column (l % 32) and rows
// 8*(i/4) + 4*(l/32) + (i%4), i = 0..15.
template <typename T>
struct Mfma;
template <>
struct Mfma<F16> {
    static constexpr int kElemsPerIssue = 8;
    // one issue consumes a whole 16-byte vector
    static __device__ __forceinline__ float16_t run(const Vec16& a, const Vec16& b, float16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a),
                                                      __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
    }
};
template <>
struct Mfma<BF16> {
    static constexpr int kElemsPerIssue = 8;
    static __device__ __forceinline__ float16_t run(const Vec16& a, const Vec16& b, float16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <>
struct Mfma<F32> {
    static constexpr int kElemsPerIssue = 1;
    // four issues per 16-byte vector, one fp32 element each
    static __device__ __forceinline__ float16_t run(const Vec16& a, const Vec16& b, float16_t c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(u2f(a.x), u2f(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(u2f(a.y), u2f(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(u2f(a.z), u2f(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(u2f(a.w), u2f(b.w), c, 0, 0, 0);
        return c;
    }
};

// Round fp32 values to the cache dtype and pack them into one 16-byte vector.
template <typename T>
__device__ __forceinline__ Vec16 pack(const float* f);
template <>
__device__ __forceinline__ Vec16 pack<F32>(const float* f)
{
    return Vec16{f2u(f[0]), f2u(f[1]), f2u(f[2]), f2u(f[3])};
}
template <>
__device__ __forceinline__ Vec16 pack<F16>(const float* f)
{
    Vec16 v;
    v.x = f32_to_f16_bits(f[0]) | (f32_to_f16_bits(f[1]) << 16);
    v.y = f32_to_f16_bits(f[2]) | (f32_to_f16_bits(f[3]) << 16);
    v.z = f32_to_f16_bits(f[4]) | (f32_to_f16_bits(f[5]) << 16);
    v.w = f32_to_f16_bits(f[6]) | (f32_to_f16_bits(f[7]) << 16);
    return v;
}
template <>
__device__ __forceinline__ Vec16 pack<BF16>(const float* f)
{
    Vec16 v;
    v.x = f32x2_to_bf16x2_bits(f[0], f[1]);
    v.y = f32x2_to_bf16x2_bits(f[2], f[3]);
    v.z = f32x2_to_bf16x2_bits(f[4], f[5]);
    v.w = f32x2_to_bf16x2_bits(f[6], f[7]);
    return v;
}

// Round one fp32 value to the cache dtype and store it as element e of a row.
template <typename T>
__device__ __forceinline__ void store_elem(char* row, int e, float v);
template <>
__device__ __forceinline__ void store_elem<F32>(char* row, int e, float v)
{
    reinterpret_cast<float*>(row)[e] = v;
}
template <>
__device__ __forceinline__ void store_elem<F16>(char* row, int e, float v)
{
    reinterpret_cast<uint16_t*>(row)[e] = (uint16_t)f32_to_f16_bits(v);
}
template <>
__device__ __forceinline__ void store_elem<BF16>(char* row, int e, float v)
{
    reinterpret_cast<uint16_t*>(row)[e] = (uint16_t)f32_to_bf16_bits(v);
}

__device__ __forceinline__ Vec16 load16(const void* p) { return *reinterpret_cast<const Vec16*>(p); }
// Streaming load of cache rows that are read once per launch: marked non-temporal, so the rows
// neither displace the small read-modify-write state (importance, positions) from the caches nor
// linger there themselves.  Measured on MI355X: a row stream of the decode step's shape runs at
// 6.8 TB/s this way against 5.9 TB/s with plain loads.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ Vec16 load16_stream(const void* p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return Vec16{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ void store16(void* p, const Vec16& v) { *reinterpret_cast<Vec16*>(p) = v; }

// ---- wave / block reductions -------------------------------------------------

// Cross-lane move on the VALU data-parallel-primitive path (no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over aligned groups of LANES consecutive lanes (4, 8, 16 or 32); every lane of the
// group gets the total.  quad_perm swaps (xor 1, xor 2), then mirrors within 8 and
// within 16 lanes; only the 32-lane case needs one LDS-routed exchange.
template <int LANES>
__device__ __forceinline__ float group_sum(float v)
{
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    if (LANES >= 8) v += dpp_move<0x141>(v);   // row_half_mirror
    if (LANES >= 16) v += dpp_move<0x140>(v);   // row_mirror
    if (LANES >= 32) v += __shfl_xor(v, 16, 64);
    return v;
}

// Whole-wave reductions: four DPP steps inside each row of 16 lanes, then two LDS-routed
// exchanges across the four rows.  Every lane gets the result.
__device__ __forceinline__ float wave_sum(float v)
{
    v = group_sum<16>(v);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_move<0xB1>(v));
    v = fmaxf(v, dpp_move<0x4E>(v));
    v = fmaxf(v, dpp_move<0x141>(v));
    v = fmaxf(v, dpp_move<0x140>(v));
    v = fmaxf(v, __shfl_xor(v, 16, kWave));
    v = fmaxf(v, __shfl_xor(v, 32, kWave));
    return v;
}
// Lexicographic minimum of a 64-bit key held as (hi, lo), carrying a payload along with the winner.
template <int CTRL>
__device__ __forceinline__ void min64p_dpp(uint32_t& hi, uint32_t& lo, int& pl)
{
    const uint32_t h2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)hi, CTRL, 0xf, 0xf, true);
    const uint32_t l2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lo, CTRL, 0xf, 0xf, true);
    const int p2 = __builtin_amdgcn_update_dpp(0, pl, CTRL, 0xf, 0xf, true);
    const bool take = (h2 < hi) || (h2 == hi && l2 < lo);
    hi = take ? h2 : hi;
    lo = take ? l2 : lo;
    pl = take ? p2 : pl;
}
__device__ __forceinline__ void wave_min64p(unsigned long long& v, int& payload)
{
    uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
    min64p_dpp<0xB1>(hi, lo, payload);
    min64p_dpp<0x4E>(hi, lo, payload);
    min64p_dpp<0x141>(hi, lo, payload);
    min64p_dpp<0x140>(hi, lo, payload);
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
        const uint32_t h2 = (uint32_t)__shfl_xor((int)hi, o, kWave);
        const uint32_t l2 = (uint32_t)__shfl_xor((int)lo, o, kWave);
        const int p2 = __shfl_xor(payload, o, kWave);
        const bool take = (h2 < hi) || (h2 == hi && l2 < lo);
        hi = take ? h2 : hi;
        lo = take ? l2 : lo;
        payload = take ? p2 : payload;
    }
    v = ((unsigned long long)hi << 32) | lo;
}
// Budget of Algorithm 1 line 1 with an independent window (integer arithmetic on
// basis points so that host and device agree exactly).
// w < 0: Algorithm 1's even split, k = nint(n*r/2) local and k global tokens.  w_eff returns the
// window actually used.
__host__ __device__ __forceinline__ void budget(int32_t n, int32_t m, int32_t w, int32_t sparsity_bp,
                                                int32_t& keep, int32_t& n_local, int32_t& n_global,
                                                int32_t& w_eff)
{
    long long keep_raw = ((long long)n * (long long)(10000 - sparsity_bp) + 5000) / 10000;
    if (w < 0) {
        const long long k = ((long long)n * (long long)(10000 - sparsity_bp) + 10000) / 20000;
        w = (int32_t)k;
        keep_raw = 2 * k;
    }
    w_eff = w;
    long long wl = w < m ? w : m;
    long long k = keep_raw > wl ? keep_raw : wl;
    if (k > m) k = m;
    keep = (int32_t)k;
    n_local = (int32_t)wl;
    n_global = (int32_t)(k - wl);
}

}  // namespace swa
