// Prefill attention on MFMA: Eq. 1-2 over the whole prompt with the causal mask,
//   out[t] = sum_{j<=t} softmax_{j<=t}(q_t . k_j * scale) v_j      for every prompt position t.
// One workgroup (4 waves) per (pair, block of 128 queries); a wave owns 32 queries.  The
// attention-weight matrix is never stored: key tiles of 32 stream through LDS (double-buffered,
// loaded to registers one tile ahead), and every wave keeps flash-style running (max, sum,
// output) state for its queries.
//
// Both contractions are arranged so that a lane owns ONE query throughout:
//   S^T = K Q^T     A = key tile (LDS, row-major), B = query fragments (registers)
//                   -> lane l holds, for query l%32, the logits of 16 of the tile's keys;
//   O^T = V^T P^T   A = value tile transposed in LDS, B = the lane's own 16 weights, packed
//                   -> lane l holds, for query l%32, 16 channels of every 32-channel tile.
// So the row statistics, the rescaling of the running output and the weights that feed the
// second product never leave the lane (one exchange with the other half-wave for the maximum).
// The 16 keys a lane holds are keys 8*(i/4) + 4*(l/32) + (i%4) of the tile; the value tile is
// written to LDS transposed AND with its keys in that order, so a value fragment is one 16-byte
// LDS read and the contraction pairs every weight with its own key.
#include "swa_kernels.hpp"

namespace swa {

struct FlashArgs {
    const char* q;
    const char* k;
    const char* v;
    char* out;
    const int32_t* cache_len;
    int32_t h, cap;
    int32_t pairs, nqb;    // (sequence, head) pairs and query blocks per pair in the grid
    float scale_log2e;
};

constexpr int kXcds = 8;   // workgroups are dealt round-robin to the 8 XCDs, each with its own L2

// Half-precision element e (0..7) of a 16-byte vector, in the low 16 bits.
__device__ __forceinline__ uint32_t half_of(const Vec16& v, int e)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    return (w[e >> 1] >> ((e & 1) * 16)) & 0xffffu;
}

// x of lane (l % 32) and x of lane (l % 32) + 32, in every lane: v_permlane32_swap exchanges the
// upper half of one register with the lower half of another, so two copies of x come back as
// (the lower half's x, the upper half's x) - no trip through LDS.
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi)
{
    const uint32_t u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    lo = __uint_as_float(r[0]);
    hi = __uint_as_float(r[1]);
}

// Two fp32 values rounded to T, packed into one dword.
template <typename T>
__device__ __forceinline__ uint32_t pack2(float f0, float f1);
template <>
__device__ __forceinline__ uint32_t pack2<F16>(float f0, float f1)
{
    return f32_to_f16_bits(f0) | (f32_to_f16_bits(f1) << 16);
}
template <>
__device__ __forceinline__ uint32_t pack2<BF16>(float f0, float f1)
{
    return f32x2_to_bf16x2_bits(f0, f1);
}

// 16-bit formats: three workgroups per CU (one wave of each per SIMD), 168 registers per lane,
// 38 KB of LDS each.  fp32 (32x32x2 MFMA, four issues per 16-byte fragment) is there for
// completeness, not speed: two waves per SIMD, and at d = 128 a single LDS buffer.
template <typename T, int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(Elem<T>::kBytes == 2 ? 3 : 2)))
swa_flash_prefill_kernel(FlashArgs a)
{
    constexpr int NT = 256;
    constexpr int EB = Elem<T>::kBytes;     // 2 or 4
    constexpr int EPV = Elem<T>::kPerVec;   // elements per 16-byte fragment: 8 or 4
    constexpr int NP = 16 / EPV;            // fragments that hold a lane's 16 weights
    constexpr int ROWB = D * EB;
    constexpr int NV = ROWB / 32;       // 16-byte vectors a lane supplies for a 32-row operand
    constexpr int CT = D / 32;          // 32-channel tiles of the output
    constexpr int BK = 32;              // keys per tile
    constexpr int BQ = 128;             // queries per workgroup
    constexpr int KSTR = ROWB + 16;     // LDS row of the key tile, padded against bank conflicts
    constexpr int VSTR = BK * EB + 16;  // LDS row (one channel, 32 keys) of the transposed value tile
    constexpr int CPR = ROWB / 16;      // 16-byte chunks per cache row
    constexpr int LD = BK * CPR / NT;   // chunks per thread, per tensor and tile
    constexpr bool kPaired = EB == 2 && LD == 2;
    constexpr float kSlack = 8.f;       // how far (powers of two) a tile maximum may exceed the reference maximum
    constexpr int PF = 3;               // LDS fragment reads in flight ahead of the product that uses them
    constexpr int NBUF = (EB == 4 && D == 128) ? 1 : 2;   // LDS buffers (64 KB of static LDS at most)
    static_assert(LD >= 1 && BK * CPR % NT == 0, "tile must split evenly over the workgroup");

    __shared__ __align__(16) char s_k[NBUF][BK * KSTR];
    // Channel c's row of the transposed value tile starts at vt_row(c): 80 bytes per row keep the
    // 16-byte fragment reads of 16 consecutive channels on disjoint banks, and every group of 16
    // channels is skewed by another 16 bytes so that the transposing stores (16 lanes, channels 8
    // apart) spread over the banks as well.
    constexpr int VT_BYTES = D * VSTR + (D / 16) * 16;
    __shared__ __align__(16) char s_vt[NBUF][VT_BYTES];
    auto vt_row = [](int c) { return c * VSTR + (c >> 4) * 16; };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int hb = lane >> 5;
    // XCD-aware placement: the query blocks of one pair all read the same K and V, so they go to
    // the same XCD, next to each other in launch order, and share the pair's rows through that
    // XCD's L2; the XCDs work on different pairs.  Longest blocks of a pair first.
    const int xcd = blockIdx.x % kXcds;
    const int idx = blockIdx.x / kXcds;
    const int64_t pair = xcd + (int64_t)kXcds * (idx / a.nqb);
    if (pair >= a.pairs) return;
    int s = a.cache_len[pair / a.h];
    s = s > a.cap ? a.cap : s;
    const int qb = a.nqb - 1 - idx % a.nqb;
    const int q0 = qb * BQ;
    if (q0 >= s) return;

    const char* Qp = a.q + pair * (int64_t)a.cap * ROWB;
    const char* Kp = a.k + pair * (int64_t)a.cap * ROWB;
    const char* Vp = a.v + pair * (int64_t)a.cap * ROWB;
    char* Op = a.out + pair * (int64_t)a.cap * ROWB;

    const int t = q0 + wave * 32 + l32;          // this lane's query position
    const int tq = t < s ? t : s - 1;            // lanes past the prompt shadow the last query
    Vec16 qv[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) qv[v] = load16(Qp + (int64_t)tq * ROWB + v * 32 + hb * 16);

    const int q_hi = (q0 + BQ < s ? q0 + BQ : s) - 1;    // last query of the workgroup
    const int nkt = q_hi / BK + 1;                        // key tiles 0..nkt-1 cover keys 0..q_hi
    const int w_lo = q0 + wave * 32;
    const int w_hi = (w_lo + 31 < s - 1) ? w_lo + 31 : s - 1;
    const int my_last = (w_lo < s) ? w_hi / BK : -1;      // last tile with a visible key for this wave

    // Which tile rows a thread stages.  With two chunks per thread (d = 128) they are an even key
    // and its successor, which sit next to each other in a lane's key order, so their values are
    // stored to the transposed tile as one dword; the four (even key) slots of a wave are chosen
    // so that, with the 16 channel groups, its 64 stores hit 64 different banks.
    auto tile_key = [&](int x) {
        if constexpr (kPaired) {
            const int q = tid / CPR;                 // 0..15
            const int pr = (q & 1) + 4 * ((q >> 1) & 1) + 2 * ((q >> 2) & 1) + 8 * (q >> 3);
            return 2 * pr + x;
        } else {
            return (tid + x * NT) / CPR;
        }
    };
    Vec16 gk[LD], gv[LD];
    auto gload = [&](int kt) {
#pragma unroll
        for (int x = 0; x < LD; ++x) {
            const int j = tile_key(x), cc = tid % CPR;
            int row = kt * BK + j;
            row = row < s ? row : s - 1;          // rows past the prompt are masked; keep them finite
            // uniform base + 32-bit offset (cap <= SWA_MAX_CAP keeps a pair's rows within 8 MiB)
            const uint32_t off = (uint32_t)row * ROWB + cc * 16;
            gk[x] = load16(Kp + off);
            gv[x] = load16(Vp + off);
        }
    };
    // key j is element i16 of half-wave hbk's 16 keys: its place (in elements) in a channel's
    // row.  16-bit: fragment v of half-wave hbk holds i16 = 8v..8v+7; fp32 fragments hold four
    // consecutive keys, so there the natural order is already the lanes' order.
    auto key_slot = [](int j) {
        if constexpr (EB == 4) return j;
        const int i16 = 4 * (j / 8) + (j % 4);
        const int hbk = (j / 4) % 2;
        return ((i16 / 8) * 2 + hbk) * 8 + (i16 % 8);
    };
    auto lstore = [&](int buf) {
        const int cc = tid % CPR;
#pragma unroll
        for (int x = 0; x < LD; ++x) store16(s_k[buf] + tile_key(x) * KSTR + cc * 16, gk[x]);
        if constexpr (kPaired) {
            const int posk = key_slot(tile_key(0));      // even, and key_slot(tile_key(1)) == posk + 1
            const uint32_t w0[4] = {gv[0].x, gv[0].y, gv[0].z, gv[0].w}, w1[4] = {gv[1].x, gv[1].y, gv[1].z, gv[1].w};
#pragma unroll
            for (int e = 0; e < 8; ++e)      // channel e of the even key below, of its successor above: one byte permute
                *reinterpret_cast<uint32_t*>(s_vt[buf] + vt_row(cc * 8 + e) + posk * 2) =
                    __builtin_amdgcn_perm(w1[e >> 1], w0[e >> 1], (e & 1) ? 0x07060302u : 0x05040100u);
        } else if constexpr (EB == 2) {
#pragma unroll
            for (int x = 0; x < LD; ++x) {
                const int posk = key_slot(tile_key(x));
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    *reinterpret_cast<uint16_t*>(s_vt[buf] + vt_row(cc * 8 + e) + posk * 2) = (uint16_t)half_of(gv[x], e);
            }
        } else {
#pragma unroll
            for (int x = 0; x < LD; ++x) {
                const int posk = key_slot(tile_key(x));
                const uint32_t w[4] = {gv[x].x, gv[x].y, gv[x].z, gv[x].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    *reinterpret_cast<uint32_t*>(s_vt[buf] + vt_row(cc * 4 + e) + posk * 4) = w[e];
            }
        }
    };

    float16_t o[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[ct][i] = 0.f;
    float m = -INFINITY, l = 0.f;

    gload(0);
    lstore(0);
    // Every load issued so far (the query fragments among them) is waited for HERE, once: the
    // memory counter is in-order, so a query fragment still in flight at the loop's entry would
    // make the compiler wait, inside every iteration's first product, for counts that on all
    // later iterations mean "the tile just requested has arrived" - the prefetch would be lost.
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
    __syncthreads();
    for (int kt = 0; kt < nkt; ++kt) {
        const int buf = kt % NBUF;
        if (kt + 1 < nkt) gload(kt + 1);
        if (kt <= my_last) {
            float16_t c;
#pragma unroll
            for (int i = 0; i < 16; ++i) c[i] = 0.f;
            const char* kb = s_k[buf] + l32 * KSTR + hb * 16;
            // key fragments are read from LDS PF products ahead of their use, in this order
            Vec16 kf[NV];
#pragma unroll
            for (int v = 0; v < PF && v < NV; ++v) kf[v] = load16(kb + v * 32);
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                if (v + PF < NV) kf[v + PF] = load16(kb + (v + PF) * 32);
                __builtin_amdgcn_sched_barrier(0);
                c = Mfma<T>::run(kf[v], qv[v], c);   // C[key][query]
                __builtin_amdgcn_sched_barrier(0);
            }
            // only the tiles that reach the wave's diagonal need the causal mask
            if (kt * BK + BK - 1 > w_lo) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = kt * BK + 8 * (i / 4) + 4 * hb + (i % 4);
                    c[i] = (key <= tq) ? c[i] : -INFINITY;
                }
            }
            float mx = c[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, c[i]);
            float mx_lo, mx_hi;
            both_halves(mx, mx_lo, mx_hi);
            mx = fmaxf(mx_lo, mx_hi) * a.scale_log2e;     // scale > 0: max commutes
            // tile 0 holds key 0, visible to every query, so the reference maximum is finite from
            // the first tile on.  The reference only has to bound the exponents, not equal the true
            // maximum (out = o / l whatever it is): it follows the tile maximum only when that
            // exceeds it by more than kSlack powers of two, so the weights stay below 2^kSlack and
            // the running output is rescaled a few times per query instead of at every new maximum.
            const float m_new = (mx > m + kSlack) ? mx : m;
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);     // 0 on the first tile, else mostly 1
            float p[16];
            float ps = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(c[i], a.scale_log2e, -m_new));   // 0 for masked keys
                ps += p[i];
            }
            l = l * alpha + ps;
            m = m_new;
            // the running maximum settles after a few tiles: rescale only when some query's moved
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[ct][i] *= alpha;
            }
            Vec16 pv[NP];
#pragma unroll
            for (int v = 0; v < NP; ++v) pv[v] = pack<T>(p + v * EPV);
            // value fragments likewise: fragment f = ct * NP + v, read PF products ahead
            Vec16 vf[CT * NP];
            // vt_row(32 ct + l32) = vt_row(l32) + ct (32 VSTR + 32): one lane address, constant offsets
            const char* vb0 = s_vt[buf] + vt_row(l32) + hb * 16;
            // product f works on channel tile f % CT with weight fragment f / CT: consecutive products
            // accumulate into different tiles, so none waits for the one before it
            auto vfrag = [&](int f) { return load16(vb0 + (f % CT) * (32 * VSTR + 32) + (f / CT) * 32); };
#pragma unroll
            for (int f = 0; f < PF && f < CT * NP; ++f) vf[f] = vfrag(f);
#pragma unroll
            for (int f = 0; f < CT * NP; ++f) {
                if (f + PF < CT * NP) vf[f + PF] = vfrag(f + PF);
                __builtin_amdgcn_sched_barrier(0);
                o[f % CT] = Mfma<T>::run(vf[f], pv[f / CT], o[f % CT]);   // C[channel][query]
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if constexpr (NBUF == 1) __syncthreads();      // every wave is done with the only buffer
        if (kt + 1 < nkt) lstore((kt + 1) % NBUF);
        __syncthreads();
    }

    float l_lo, l_hi;
    both_halves(l, l_lo, l_hi);
    l = l_lo + l_hi;
    if (t < s) {
        const float inv = 1.f / l;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                // channels 32 ct + 8 g + 4 hb + 0..3 of query t
                char* dst = Op + (int64_t)t * ROWB + (32 * ct + 8 * g + 4 * hb) * EB;
                if constexpr (EB == 4) {
                    float f[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) f[r] = o[ct][4 * g + r] * inv;
                    store16(dst, pack<F32>(f));
                } else {
                    uint32_t w[2];
#pragma unroll
                    for (int r = 0; r < 2; ++r)
                        w[r] = pack2<T>(o[ct][4 * g + 2 * r] * inv, o[ct][4 * g + 2 * r + 1] * inv);
                    *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
                }
            }
        }
    }
}

int launch_flash_prefill(const swa_params& p, float scale, const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* cache_len, void* out, hipStream_t stream)
{
    FlashArgs a;
    a.q = static_cast<const char*>(q);
    a.k = static_cast<const char*>(k_cache);
    a.v = static_cast<const char*>(v_cache);
    a.out = static_cast<char*>(out);
    a.cache_len = cache_len;
    a.h = p.h;
    a.cap = p.cap;
    a.scale_log2e = scale * 1.44269504088896340736f;
    const int bound = (p.len_bound > 0 && p.len_bound < p.cap) ? p.len_bound : p.cap;
    a.pairs = p.b * p.h;
    a.nqb = (bound + 127) / 128;
    const int64_t per_xcd = ((int64_t)a.pairs + kXcds - 1) / kXcds;
    const int64_t wgs = per_xcd * kXcds * a.nqb;
    if (wgs > 0x7fffffffLL) return SWA_ERR_BAD_SHAPE;
    const dim3 grid((unsigned)wgs);
    if (p.dtype == SWA_F16) {
        if (p.d == 64) hipLaunchKernelGGL((swa_flash_prefill_kernel<F16, 64>), grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((swa_flash_prefill_kernel<F16, 128>), grid, dim3(256), 0, stream, a);
    } else if (p.dtype == SWA_BF16) {
        if (p.d == 64) hipLaunchKernelGGL((swa_flash_prefill_kernel<BF16, 64>), grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((swa_flash_prefill_kernel<BF16, 128>), grid, dim3(256), 0, stream, a);
    } else {
        if (p.d == 64) hipLaunchKernelGGL((swa_flash_prefill_kernel<F32, 64>), grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((swa_flash_prefill_kernel<F32, 128>), grid, dim3(256), 0, stream, a);
    }
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

}  // namespace swa
