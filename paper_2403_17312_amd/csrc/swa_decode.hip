// Decode-step Sparse Window Attention: one workgroup per (sequence, head) pair.
//
// A workgroup walks the whole step for its pair without leaving the CU:
//   append -> logits GEMV over the cached keys (Eq. 1) -> softmax -> importance
//   accumulation (running local attention sum, Alg. 1 line 2) -> budget and
//   selection of the globally dynamic tokens (Alg. 1 lines 1, 3-5) -> weighted sum
//   of the kept values, renormalised over the kept set (lines 6-8).
// Logits, probabilities, selection keys and the kept list live in LDS, so the
// only HBM traffic is one read of the key rows, one read of the value rows that
// are needed, one read+write of the importance vector and the index list.
//
// Two schedules, chosen per sequence from the number of evictions E = m - keep
// (known before any data is read):
//   * few evictions (the steady state under per-step compaction, E <= 1): ONE
//     streaming pass loads key and value rows together and keeps flash-style
//     running (max, sum, weighted-value) accumulators over ALL slots; after the
//     selection, the evicted rows' contribution is subtracted:
//         out = (dense - sum_E p_j v_j) / (1 - sum_E p_j).
//     If the kept mass 1 - sum_E p_j is small the subtraction would cancel, and
//     the kernel falls back to the gathered pass below.
//   * many evictions (first step after a prompt, lazy compaction): the key pass
//     runs alone, then only the kept value rows are gathered.
// Selection: E == 0 keeps everything; E == 1 is a workgroup arg-min; otherwise an
// LDS radix select (4 x 8 bits, most significant first) finds the n_global-th
// largest key, and an ordered ballot/popcount compaction writes the ascending
// kept list with ties resolved towards the lowest slot.
//
// The same kernel also carries, selected by its arguments:
//   * fused compaction (the kept rows move to slots 0..keep-1 inside the step), either in token
//     order (rows behind a hole shift down, newest rows parked in LDS) or unordered (holes are
//     filled by kept rows from above `keep`; window and tie rule then go by token position);
//   * the head-reduced token set of Algorithm 1's header (phase 1 publishes every pair's new
//     importance, weights and dense output; after a sum over the heads, phase 2 selects and
//     finishes);
//   * the 8-bit compressed cache of Section V-B (the Q8 instantiation: codes are converted and
//     multiplied in registers, scale and zero point are folded into the query and the output);
//   * the strict local attention sum (importance = sum of a ring of the last R attention rows,
//     whose columns follow their tokens through the compaction).
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
    int32_t h, cap, lds_slots, w, sparsity_bp;
    float scale;
    int32_t fuse_compaction;
    int32_t unordered;    // fused compaction fills holes instead of shifting rows (order by pos only)
    // Head-shared selection runs as three launches: phase 1 streams the cache and publishes the
    // new importance, the attention weights and the dense output of every pair; a small kernel
    // sums the new importance over the heads of every sequence; phase 2 selects from that sum
    // (every head of a sequence reaches the same decision) and finishes output and compaction.
    int32_t phase;        // 0 = whole step in one launch; 1, 2 = the two halves of the head-shared
                          // step; 3 = rows split over workgroups: the logits come from ws_z, and the
                          // weights go to ws_p for the launches that form the output
    const float* ws_z;    // [b,h,cap] logits of the split step
    int32_t* ws_ok;       // [b,h]     split step: set to 1 when the pair's step has run (not skipped)
    float* ws_p;          // [b,h,cap] attention weights of phase 1
    float* ws_snew;       // [b,h,cap] new importance of phase 1
    float* ws_abar;       // [b,h,d]   dense attention output of phase 1
    float* ws_tot;        // [b,cap]   new importance summed over the heads
    int32_t stash_rows;   // fused compaction: newest rows kept in LDS during the streaming pass
    // Compressed cache (Section V-B): per (pair, channel) scale and zero point of keys and values,
    // four fp32 arrays of qstride = b*h*d values each (lambda_K, z_K, lambda_V, z_V).
    const float* qparams;
    int64_t qstride;
    // Strict local attention sum (Algorithm 1 line 2): the last ring_rows attention rows per pair,
    // [b,h,ring_rows,cap]; this step overwrites row ring_row and the importance is the sum of
    // the rows.  NULL: running sum in `score`.
    float* ring;
    int32_t ring_rows, ring_row;
};

constexpr int kMaxFix = 8;           // evicted rows the subtractive schedule handles
constexpr float kMinKeptMass = 0.05f;
constexpr float kLog2e = 1.44269504088896340736f;

// Monotone map fp32 -> uint32 (larger float <=> larger key).
__device__ __forceinline__ uint32_t order_key(float f)
{
    uint32_t u = f2u(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Merge the flash accumulators (M, S, acc) of two disjoint row sets.
template <int EPV>
__device__ __forceinline__ void merge_acc(float& M, float& S, float* acc, float M2, float S2, const float* acc2)
{
    const float Mn = fmaxf(M, M2);
    const float r1 = (M == -INFINITY) ? 0.f : fast_exp2((M - Mn) * kLog2e);
    const float r2 = (M2 == -INFINITY) ? 0.f : fast_exp2((M2 - Mn) * kLog2e);
    S = S * r1 + S2 * r2;
#pragma unroll
    for (int e = 0; e < EPV; ++e) acc[e] = acc[e] * r1 + acc2[e] * r2;
    M = Mn;
}

// Register budget: five waves per SIMD (96 VGPRs) for the 16- and 32-bit caches, four (128) for
// the 8-bit one, whose lanes carry 16 channels each, and for the 512-thread workgroups that serve
// long caches (two of them fill a CU's wave slots either way); none of the bounds spills.  RING: the strict
// local attention sum, a separate instantiation so that the other forms carry none of its code.
template <typename T, int D, int NT, bool RING>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu((Elem<T>::kBytes == 1 || NT >= 512) ? 4 : 5)))
swa_decode_kernel(DecodeArgs a)
{
    // a.ring is non-NULL exactly when RING (the launcher picks the instantiation)
    const bool has_ring = RING;
    constexpr int EPV = Elem<T>::kPerVec;   // elements per 16-byte vector
    constexpr int LPR = D / EPV;            // lanes per row
    constexpr int NW = NT / kWave;
    constexpr int NG = NT / LPR;            // row groups per workgroup
    constexpr int ROWB = D * Elem<T>::kBytes;          // one cache row
    typedef typename Act<T>::type AT;
    constexpr int XROWB = D * Elem<AT>::kBytes;        // one row of q, k_new, v_new, out
    constexpr bool kQ8 = Elem<T>::kBytes == 1;
    constexpr int UK = 8;                   // key rows in flight per group (key-only pass)
    constexpr int UF = 2;                   // key+value row pairs per group and pipeline stage (fused pass)
    // The 512-thread instantiation (long caches: the step after a prompt) has 128 registers per
    // lane and keeps twice as many rows in flight in the gathered pass and in the row moves.
    constexpr bool kWide = NT >= 512;
    constexpr int UV = kWide ? 6 : 4;       // value rows in flight per group (gathered pass)
    constexpr int SPF = 4;                  // importance values prefetched per thread

    extern __shared__ __align__(16) char smem[];
    float* s_p = reinterpret_cast<float*>(smem);                       // logits -> probabilities
    uint32_t* s_key = reinterpret_cast<uint32_t*>(s_p + a.lds_slots);  // selection keys
    // The ascending kept list (16-bit slots) overlays the key array: entry j is written
    // only after key j' >= j of the same or a later tile has been read (see the ordered
    // compaction below), and the keys are dead once the list is complete.
    uint16_t* s_kept = reinterpret_cast<uint16_t*>(s_key);
    // Fused compaction only: the new importance values and the old positions wait in LDS
    // until the selection is known, then go straight to their compacted slots.
    float* s_sc = reinterpret_cast<float*>(s_key + a.lds_slots);
    int32_t* s_pos = reinterpret_cast<int32_t*>(s_sc + a.lds_slots);
    // ... and the newest stash_rows key/value rows are parked in LDS while they stream by: the
    // token evicted in the steady state sits just behind the window, so the rows that have to
    // move down (and the evicted row itself) are then served from LDS instead of being re-read.
    const bool fc = a.fuse_compaction != 0;
    const bool bag = a.unordered != 0;
    // Unordered compaction only: source slot of every final slot, the holes below `keep` and the
    // kept rows above it that fill them (at most half of the slots each).
    uint16_t* s_src = reinterpret_cast<uint16_t*>(s_pos + a.lds_slots);
    uint16_t* s_holes = s_src + a.lds_slots;
    uint16_t* s_movers = s_holes + a.lds_slots / 2;
    char* s_stK = reinterpret_cast<char*>(s_pos + a.lds_slots) + (bag ? (size_t)a.lds_slots * 4 : 0);
    char* s_stV = s_stK + (size_t)a.stash_rows * ROWB;
    __shared__ float s_redA[16];
    __shared__ float s_redB[16];
    __shared__ unsigned long long s_red64[16];
    __shared__ int32_t s_hist[256];
    __shared__ int32_t s_wcnt[2][16];
    __shared__ int32_t s_sel[3];
    __shared__ float s_acc[NW * D];
    __shared__ float s_wS[16];
    __shared__ float s_fix[kMaxFix * D];
    __shared__ int32_t s_evict[kMaxFix];
    __shared__ int32_t s_ecnt;
    __shared__ __align__(16) unsigned char s_newc[kQ8 ? 2 * D : 16];   // codes of the new K and V rows
    __shared__ __align__(16) float s_qs[kQ8 ? D : 4];
    __shared__ __align__(16) float s_qz[kQ8 ? D : 4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int sub = lane % LPR;
    const int grp = tid / LPR;
    const int64_t pair = blockIdx.x;
    const int s = (int)(pair / a.h);

    // The first stage of the streaming pass is requested before the lengths are known (they are a
    // dependent round trip of their own): its rows exist whatever the length is (clamped to the
    // last slot), and whatever lies at or beyond `len` is replaced by the new row when the stage
    // is reduced.  They are waited for at their first use.
    // (Not for the 8-bit cache: its lanes have no registers to spare, and it measured slower.)
    constexpr bool kEarlyStage = !kQ8;
    Vec16 k0[UF], v0[UF];
    if (kEarlyStage && a.phase != 2 && a.phase != 3) {
        const char* Kq = a.k_cache + pair * (int64_t)a.cap * ROWB;
        const char* Vq = a.v_cache + pair * (int64_t)a.cap * ROWB;
#pragma unroll
        for (int u = 0; u < UF; ++u) {
            int row = u * NG + grp;
            row = row < a.cap ? row : a.cap - 1;
            k0[u] = load16_stream(Kq + (int64_t)row * ROWB + sub * 16);
            v0[u] = load16_stream(Vq + (int64_t)row * ROWB + sub * 16);
        }
    }

    const int len = a.cache_len[s];
    const int n = a.seq_len[s];
    const int m = len + 1;
    const bool overflow = (m > a.cap) || (m > a.lds_slots) || (len < 0);

    int keep = 0, n_local = 0, n_global = 0;

    if (!overflow) {
        const int cap = a.cap;
        char* Kp = a.k_cache + pair * (int64_t)cap * ROWB;
        char* Vp = a.v_cache + pair * (int64_t)cap * ROWB;
        float* Sp = a.score + pair * (int64_t)cap;
        int32_t* Pp = a.pos + pair * (int64_t)cap;
        const float* lamK = kQ8 ? a.qparams + pair * D : nullptr;
        const float* zK = kQ8 ? lamK + a.qstride : nullptr;
        const float* lamV = kQ8 ? lamK + 2 * a.qstride : nullptr;
        const float* zV = kQ8 ? lamK + 3 * a.qstride : nullptr;
        // This lane's 16 bytes of the new token's key and value rows, in the cache's format, and
        // its query operand.  Wherever a loop meets slot `len` it takes nk/nv instead of what it
        // loaded.  With a compressed cache the new row is quantised on arrival (the step reads
        // what memory will hold): one thread per channel loads the parameters, quantises and
        // pre-scales the query (q_c lambda_c, and its zero-point product) into LDS, and the
        // lanes pick their 16-channel pieces up from there in new_row_ready(), which every
        // path calls once, after its first cache loads are in flight.
        Vec16 nk, nv;
        QFrag<T> qf;
        float pq = 0.f, pl = 0.f, pz = 0.f, pkn = 0.f, pvn = 0.f, plv = 0.f, pzv = 0.f;
        if constexpr (kQ8) {
            if (tid < D) {
                pl = lamK[tid];
                pz = zK[tid];
                plv = lamV[tid];
                pzv = zV[tid];
                pq = (float)reinterpret_cast<const _Float16*>(a.q + pair * XROWB)[tid];
                pkn = (float)reinterpret_cast<const _Float16*>(a.k_new + pair * XROWB)[tid];
                pvn = (float)reinterpret_cast<const _Float16*>(a.v_new + pair * XROWB)[tid];
            }
        } else {
            nk = load16(a.k_new + pair * XROWB + sub * 16);
            nv = load16(a.v_new + pair * XROWB + sub * 16);
            qf.load(load16(a.q + pair * XROWB + sub * 16));
        }
        auto new_row_ready = [&]() {
            if constexpr (kQ8) {
                if (tid < D) {
                    s_newc[tid] = (unsigned char)quantise_one(pkn, pl, pz);
                    s_newc[D + tid] = (unsigned char)quantise_one(pvn, plv, pzv);
                    const float qs = pq * pl;
                    s_qs[tid] = qs;
                    s_qz[tid] = qs * pz;
                }
                __syncthreads();
                nk = *reinterpret_cast<const Vec16*>(s_newc + sub * 16);
                nv = *reinterpret_cast<const Vec16*>(s_newc + D + sub * 16);
                qf.load(s_qs + sub * 16, s_qz + sub * 16);
            }
        };
        auto write_out = [&](int e, float v) {
            if constexpr (kQ8) v = lamV[e] * (v - zV[e]);      // accumulated in code space
            store_elem<AT>(a.out + pair * XROWB, e, v);
        };

        int w_eff = 0;
        budget(n, m, a.w, a.sparsity_bp, keep, n_local, n_global, w_eff);
        const int ncand = m - n_local;
        const int wlo = n - w_eff;                    // unordered layout: the window is pos >= wlo
        const int E = m - keep;                       // evictions of this step
        const bool fused = (E <= kMaxFix) && (8 * E <= m) && a.phase != 3;
        // first stashed slot (m = nothing stashed: only the streaming schedule fills the stash)
        const int stash_lo = (fc && fused) ? (m > a.stash_rows ? m - a.stash_rows : 0) : m;

        float acc[EPV];           // fused pass: running sum of exp(z - Mg) * v
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[e] = 0.f;
        float mx = 0.f;           // global max of the logits (reference of the wave partials)
        // (key << 32 | ~t): min = lowest score, then highest t; t is the slot, or the token
        // position when slots are unordered.  The slot rides along as payload.
        unsigned long long best = ~0ull;
        int bslot = m;

        if (a.phase != 2) {
        // ---- importance prefetch: the old values are needed only after the softmax ----
        float sold[SPF];
#pragma unroll
        for (int k = 0; k < SPF; ++k) {
            const int i = tid + k * NT;
            sold[k] = (i < len && !has_ring) ? Sp[i] : 0.f;
        }
        int32_t pold[SPF];
#pragma unroll
        for (int k = 0; k < SPF; ++k) {
            const int i = tid + k * NT;
            pold[k] = (fc && i < len) ? Pp[i] : (n - 1);
        }

        // ---- append (with fused compaction the new row goes straight to its final slot) ----
        if (!fc) {
            new_row_ready();
            if (tid < LPR) {
                store16(Kp + (int64_t)len * ROWB + sub * 16, nk);
            } else if (tid < 2 * LPR) {
                store16(Vp + (int64_t)len * ROWB + sub * 16, nv);
            }
            if (tid == 0) Pp[len] = n - 1;
        }
        if (tid == 0) s_ecnt = 0;


        float Mg = -INFINITY;     // running max of this group's logits
        float Sg = 0.f;           // fused pass: running sum of exp(z - Mg)

        if (fused) {
            // ---- one pass over key AND value rows, flash-style accumulators ---------
            // Software-pipelined: the loads of stage i+1 are in flight while stage i is
            // reduced, so the memory system never idles inside a wave.  Loads are
            // unconditional (out-of-range rows re-read the newest row and get weight 0)
            // so that the outstanding-load count is exact and stage i's wait does not
            // also drain stage i+1.
            constexpr int STEP = NG * UF;
            auto load_stage = [&](int base, Vec16(&kv)[UF], Vec16(&vv)[UF]) {
#pragma unroll
                for (int u = 0; u < UF; ++u) {
                    int row = base + u * NG + grp;
                    row = row < m ? row : len;
                    kv[u] = load16_stream(Kp + (int64_t)row * ROWB + sub * 16);
                    vv[u] = load16_stream(Vp + (int64_t)row * ROWB + sub * 16);
                }
            };
            auto reduce_stage = [&](int base, Vec16(&kv)[UF], Vec16(&vv)[UF]) {
                float z[UF];
#pragma unroll
                for (int u = 0; u < UF; ++u) {
                    if (base + u * NG + grp >= len) {      // slot len and the padding behind it
                        kv[u] = nk;
                        vv[u] = nv;
                    }
                    z[u] = qf.dot(kv[u], 0.f);
                }
#pragma unroll
                for (int u = 0; u < UF; ++u) z[u] = group_sum<LPR>(z[u]) * a.scale;
                float mc = -INFINITY;
#pragma unroll
                for (int u = 0; u < UF; ++u) {
                    const int row = base + u * NG + grp;
                    if (row >= stash_lo && row < m) {
                        store16(s_stK + (row - stash_lo) * ROWB + sub * 16, kv[u]);
                        store16(s_stV + (row - stash_lo) * ROWB + sub * 16, vv[u]);
                    }
                    if (sub == 0 && row < m) s_p[row] = z[u];
                    z[u] = (row < m) ? z[u] : -INFINITY;
                    mc = fmaxf(mc, z[u]);
                }
                if (mc > -INFINITY) {
                    const float Mn = fmaxf(Mg, mc);
                    const float r = fast_exp2((Mg - Mn) * kLog2e);   // 0 when Mg is -inf
                    Sg *= r;
#pragma unroll
                    for (int e = 0; e < EPV; ++e) acc[e] *= r;
#pragma unroll
                    for (int u = 0; u < UF; ++u) {
                        const float ew = fast_exp2((z[u] - Mn) * kLog2e);   // 0 for padding rows
                        float f[EPV];
                        unpack<T>(vv[u], f);
                        Sg += ew;
#pragma unroll
                        for (int e = 0; e < EPV; ++e) acc[e] = __builtin_fmaf(ew, f[e], acc[e]);
                    }
                    Mg = Mn;
                }
            };
            Vec16 kA[UF], vA[UF], kB[UF], vB[UF];
            if constexpr (kEarlyStage) {
#pragma unroll
                for (int u = 0; u < UF; ++u) {
                    kA[u] = k0[u];
                    vA[u] = v0[u];
                }
            } else {
                load_stage(0, kA, vA);
            }
            if (fc) new_row_ready();
            for (int base = 0; base < m; base += 2 * STEP) {
                load_stage(base + STEP, kB, vB);
                reduce_stage(base, kA, vA);
                load_stage(base + 2 * STEP, kA, vA);
                reduce_stage(base + STEP, kB, vB);
            }
            // combine the row groups of a wave, then park the wave partials in LDS
#pragma unroll
            for (int o = LPR; o < kWave; o <<= 1) {
                const float M2 = __shfl_xor(Mg, o, kWave);
                const float S2 = __shfl_xor(Sg, o, kWave);
                float acc2[EPV];
#pragma unroll
                for (int e = 0; e < EPV; ++e) acc2[e] = __shfl_xor(acc[e], o, kWave);
                merge_acc<EPV>(Mg, Sg, acc, M2, S2, acc2);
            }
            if (lane < LPR) {
#pragma unroll
                for (int e = 0; e < EPV; ++e) s_acc[wave * D + sub * EPV + e] = acc[e];
            }
            if (lane == 0) {
                s_redA[wave] = Mg;
                s_wS[wave] = Sg;
            }
        } else if (a.phase == 3) {
            // ---- rows split over workgroups: the logits were formed by the launch before ----
            const float* Zp = a.ws_z + pair * (int64_t)cap;
            for (int i = tid; i < m; i += NT) {
                const float d = Zp[i];
                s_p[i] = d;
                Mg = fmaxf(Mg, d);
            }
            Mg = wave_max(Mg);
            if (lane == 0) s_redA[wave] = Mg;
        } else {
            // ---- key-only pass -------------------------------------------------------
            if (fc) new_row_ready();
            for (int base = 0; base < m; base += NG * UK) {
                Vec16 kv[UK];
#pragma unroll
                for (int u = 0; u < UK; ++u) {
                    const int row = base + u * NG + grp;
                    if (row < len) {
                        // with fused compaction the key rows that change slot are read again soon:
                        // plain loads leave them where the second read can find them
                        kv[u] = fc ? load16(Kp + (int64_t)row * ROWB + sub * 16)
                                   : load16_stream(Kp + (int64_t)row * ROWB + sub * 16);
                    } else {
                        kv[u] = nk;
                    }
                }
#pragma unroll
                for (int u = 0; u < UK; ++u) {
                    const int row = base + u * NG + grp;
                    const float d = group_sum<LPR>(qf.dot(kv[u], 0.f)) * a.scale;
                    if (row < m) {
                        if (sub == 0) s_p[row] = d;
                        Mg = fmaxf(Mg, d);
                    }
                }
            }
            Mg = wave_max(Mg);
            if (lane == 0) s_redA[wave] = Mg;
        }
        __syncthreads();

        // Strict window: request the ring entries of this thread's first slot now, so that they
        // travel while the softmax runs (rings of up to kRingAhead rows; longer ones, and the
        // further slots of long caches, are read in the accumulation loop itself).
        constexpr int kRingAhead = 32;
        float* Rg = has_ring ? a.ring + pair * (int64_t)a.ring_rows * cap : nullptr;
        // (not on the 8-bit cache, whose lanes have no registers to spare for it)
        const bool ring_ahead = has_ring && !kQ8 && a.ring_rows <= kRingAhead;
        float rpre[kRingAhead];
        if (ring_ahead) {
            const bool old = tid < len;
#pragma unroll
            for (int j = 0; j < kRingAhead; ++j)
                rpre[j] = (old && j < a.ring_rows && j != a.ring_row) ? Rg[(int64_t)j * cap + tid] : 0.f;
        }

        // ---- softmax over the m cached slots ------------------------------------------
        mx = s_redA[0];
#pragma unroll
        for (int v = 1; v < NW; ++v) mx = fmaxf(mx, s_redA[v]);
        float sum = 0.f;
        for (int i = tid; i < m; i += NT) {
            const float e = expf(s_p[i] - mx);
            s_p[i] = e;
            sum += e;
        }
        sum = wave_sum(sum);
        if (lane == 0) s_redB[wave] = sum;
        __syncthreads();
        sum = 0.f;
#pragma unroll
        for (int v = 0; v < NW; ++v) sum += s_redB[v];

        // Strict window: the rows of the ring in index order, the current weight standing in for
        // the row this step replaces; a token appended in this step has no earlier rows.
        auto window_sum = [&](int i, float p) -> float {
            float t = 0.f;
            const bool old = i < len;
            int j = 0;
            for (; j + 8 <= a.ring_rows; j += 8) {
                float v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] = (old && j + k != a.ring_row) ? Rg[(int64_t)(j + k) * cap + i] : 0.f;
#pragma unroll
                for (int k = 0; k < 8; ++k) t += (j + k == a.ring_row) ? p : v[k];
            }
            for (; j < a.ring_rows; ++j) {
                const float v = (old && j != a.ring_row) ? Rg[(int64_t)j * cap + i] : 0.f;
                t += (j == a.ring_row) ? p : v;
            }
            return t;
        };

        // ---- importance accumulation; arg-min bookkeeping for the E == 1 case ------------
#pragma unroll
        for (int k = 0; k < SPF; ++k) {
            const int i = tid + k * NT;
            if (i < m) {
                const float p = s_p[i] / sum;
                s_p[i] = p;
                float sc;
                if (ring_ahead && k == 0) {
                    sc = 0.f;                         // same order of additions as window_sum
#pragma unroll
                    for (int j = 0; j < kRingAhead; ++j)
                        if (j < a.ring_rows) sc += (j == a.ring_row) ? p : rpre[j];
                } else {
                    sc = has_ring ? window_sum(i, p) : sold[k] + p;
                }
                if (fc) {
                    s_sc[i] = sc;
                    s_pos[i] = pold[k];
                } else {
                    Sp[i] = sc;
                }
                if (a.phase == 1) a.ws_snew[pair * (int64_t)cap + i] = sc;
                if (a.phase == 1 || a.phase == 3) a.ws_p[pair * (int64_t)cap + i] = p;
                const uint32_t key = order_key(sc);
                s_key[i] = key;
                if (bag ? (pold[k] < wlo) : (i < ncand)) {
                    const uint32_t t = bag ? (uint32_t)pold[k] : (uint32_t)i;
                    const unsigned long long c = ((unsigned long long)key << 32) | (uint32_t)(~t);
                    if (c < best) {
                        best = c;
                        bslot = i;
                    }
                }
            }
        }
        for (int i = tid + SPF * NT; i < m; i += NT) {
            const float p = s_p[i] / sum;
            s_p[i] = p;
            const float sc = has_ring ? window_sum(i, p) : ((i == len) ? 0.f : Sp[i]) + p;
            const int posi = (fc && i < len) ? Pp[i] : (n - 1);
            if (fc) {
                s_sc[i] = sc;
                s_pos[i] = posi;
            } else {
                Sp[i] = sc;
            }
            if (a.phase == 1) a.ws_snew[pair * (int64_t)cap + i] = sc;
            if (a.phase == 1 || a.phase == 3) a.ws_p[pair * (int64_t)cap + i] = p;
            const uint32_t key = order_key(sc);
            s_key[i] = key;
            if (bag ? (posi < wlo) : (i < ncand)) {
                const uint32_t t = bag ? (uint32_t)posi : (uint32_t)i;
                const unsigned long long c = ((unsigned long long)key << 32) | (uint32_t)(~t);
                if (c < best) {
                    best = c;
                    bslot = i;
                }
            }
        }
        if (a.probs_dbg) {
            __syncthreads();
            float* dbg = a.probs_dbg + pair * (int64_t)cap;
            for (int i = tid; i < cap; i += NT) dbg[i] = (i < m) ? s_p[i] : 0.f;
        }

        if (a.phase == 1) {
            // publish the dense output; phase 2 subtracts the evicted rows from it
            if (fused) {
                for (int e = tid; e < D; e += NT) {
                    float St = 0.f, At = 0.f;
#pragma unroll
                    for (int v = 0; v < NW; ++v) {
                        const float r = fast_exp2((s_redA[v] - mx) * kLog2e);
                        St = __builtin_fmaf(s_wS[v], r, St);
                        At = __builtin_fmaf(s_acc[v * D + e], r, At);
                    }
                    a.ws_abar[pair * D + e] = At / St;
                }
            }
            return;
        }
        } else {
            // ---- phase 2 of the head-shared step: reload what phase 1 published --------------
            new_row_ready();
            if (tid == 0) s_ecnt = 0;
            const float* Pw = a.ws_p + pair * (int64_t)cap;
            const float* Sn = a.ws_snew + pair * (int64_t)cap;
            const float* Tot = a.ws_tot + (int64_t)s * cap;
            for (int i = tid; i < m; i += NT) {
                s_p[i] = Pw[i];
                s_sc[i] = Sn[i];
                const int posi = (i < len) ? Pp[i] : (n - 1);
                s_pos[i] = posi;
                const uint32_t key = order_key(Tot[i]);
                s_key[i] = key;
                if (posi < wlo) {
                    const unsigned long long c = ((unsigned long long)key << 32) | (uint32_t)(~(uint32_t)posi);
                    if (c < best) {
                        best = c;
                        bslot = i;
                    }
                }
            }
            // the dense output stands in for wave 0's partial of the streaming pass; the other
            // waves' partials are empty (weight 0, so their sums must be finite: zero)
            for (int e = tid; e < NW * D; e += NT) s_acc[e] = (fused && e < D) ? a.ws_abar[pair * D + e] : 0.f;
            if (tid < 16) {
                s_redA[tid] = (tid == 0) ? 0.f : -INFINITY;
                s_wS[tid] = (tid == 0) ? 1.f : 0.f;
            }
            mx = 0.f;
        }

        // ---- selection ---------------------------------------------------------------------
        int32_t* kout = a.kept_idx ? a.kept_idx + pair * (int64_t)cap : nullptr;
        bool have_list = false;           // s_kept holds the kept list
        int jstar = m;                    // E <= 1: the evicted slot (m = none)
        int n_moves = 0;                  // unordered layout: rows that change slot
        if (E == 0) {
            if (kout)
                for (int i = tid; i < m; i += NT) kout[i] = i;
            __syncthreads();
        } else if (E == 1 && n_global > 0) {
            // evict the single candidate that loses: lowest score, ties -> the latest token
            wave_min64p(best, bslot);
            if (lane == 0) {
                s_red64[wave] = best;
                s_wcnt[0][wave] = bslot;
            }
            __syncthreads();
            best = s_red64[0];
            jstar = s_wcnt[0][0];
#pragma unroll
            for (int v = 1; v < NW; ++v) {
                if (s_red64[v] < best) {
                    best = s_red64[v];
                    jstar = s_wcnt[0][v];
                }
            }
            jstar = jstar < 0 ? 0 : (jstar > len ? len : jstar);
            if (kout) {
                // ordered: the rows behind the hole shift down; unordered: the new row fills it
                for (int j = tid; j < keep; j += NT)
                    kout[j] = bag ? (j == jstar ? len : j) : j + (j >= jstar ? 1 : 0);
            }
            if (tid == 0) {
                s_evict[0] = jstar;
                s_ecnt = 1;
            }
            __syncthreads();
        } else {
            have_list = true;
            __syncthreads();   // keys of every thread are in LDS
            if (bag) {
                // The window is found by position.  If the caller widened it since the last call,
                // some of its positions were evicted earlier: what is missing is made up by global
                // tokens, so that exactly `keep` tokens are kept and every hole finds its mover.
                int present = 0;
                for (int base = 0; base < m; base += NT) {
                    const int i = base + tid;
                    present += (int)__popcll(__ballot(i < m && s_pos[i] >= wlo));
                }
                if (lane == 0) s_wcnt[0][wave] = present;
                __syncthreads();
                present = 0;
#pragma unroll
                for (int v = 0; v < NW; ++v) present += s_wcnt[0][v];
                __syncthreads();
                n_global = keep - present;
                n_global = n_global < 0 ? 0 : n_global;
            }
            // radix select: the n_global-th largest key among candidates 0..ncand-1
            uint32_t prefix = 0u, mask = 0u;
            int rem = n_global;
            if (n_global > 0) {
                for (int shift = 24; shift >= 0; shift -= 8) {
                    for (int i = tid; i < 256; i += NT) s_hist[i] = 0;
                    __syncthreads();
                    for (int i = tid; i < m; i += NT) {
                        const uint32_t key = s_key[i];
                        const bool c_i = bag ? (s_pos[i] < wlo) : (i < ncand);
                        if (c_i && (key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255u], 1);
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
                                s_sel[2] = cs[k];      // keys sharing the whole prefix so far
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
            // Both compactions below give every thread a contiguous run of `per` slots (at most 64:
            // a cache has at most 16384 slots and long caches get 256 threads or more), so a
            // thread's decisions fit one 64-bit mask and their order needs two block-wide prefix
            // sums instead of a ballot and two barriers per 64 slots.
            const int per = (m + NT - 1) / NT;
            const int lo = tid * per;
            const int hi = lo + per < m ? lo + per : m;
            // exclusive prefix sum over the threads of the workgroup, and the total
            auto block_scan = [&](int v, int& before, int& total) {
                int inc = v;
#pragma unroll
                for (int o = 1; o < kWave; o <<= 1) {
                    const int t = __shfl_up(inc, o, kWave);
                    if (lane >= o) inc += t;
                }
                if (lane == kWave - 1) s_wcnt[0][wave] = inc;
                __syncthreads();
                int wb = 0, tot = 0;
#pragma unroll
                for (int v2 = 0; v2 < NW; ++v2) {
                    const int c = s_wcnt[0][v2];
                    if (v2 < wave) wb += c;
                    tot += c;
                }
                before = wb + inc - v;
                total = tot;
                __syncthreads();
            };
            if (bag) {
                // ---- unordered layout: holes below `keep` are filled by kept rows above it ----
                // A candidate is kept if its key exceeds the threshold, or equals it and is one of
                // the `rem` earliest tokens among the equals (rank by position, found by a scan
                // of the candidates only when some equal key has to lose).
                const int n_eq = (n_global > 0) ? s_sel[2] : 0;
                uint64_t keptm = 0ull;
                for (int k = 0; k < per; ++k) {
                    const int i = lo + k;
                    if (i >= hi) break;
                    bool kept = false;
                    const int posi = s_pos[i];
                    if (posi >= wlo) {
                        kept = true;
                    } else if (n_global > 0) {
                        const uint32_t key = s_key[i];
                        if (key > prefix) {
                            kept = true;
                        } else if (key == prefix) {
                            if (n_eq == rem) {
                                kept = true;
                            } else {
                                int rank = 0;
                                for (int j = 0; j < m; ++j)
                                    rank += (s_key[j] == prefix && s_pos[j] < posi) ? 1 : 0;
                                kept = rank < rem;
                            }
                        }
                    }
                    if (kept) keptm |= 1ull << k;
                }
                // holes (low half) and movers (high half) of this thread's run, counted together
                int nh = 0, nm = 0;
                for (int k = 0; k < per; ++k) {
                    const int i = lo + k;
                    if (i >= hi) break;
                    const bool kept = (keptm >> k) & 1ull;
                    nh += (i < keep && !kept) ? 1 : 0;
                    nm += (i >= keep && kept) ? 1 : 0;
                }
                int before = 0, total = 0;
                block_scan(nh | (nm << 16), before, total);
                int hr = before & 0xffff, mr = before >> 16;
                const int run_h = total & 0xffff, run_m = total >> 16;
                for (int k = 0; k < per; ++k) {
                    const int i = lo + k;
                    if (i >= hi) break;
                    const bool kept = (keptm >> k) & 1ull;
                    // the evicted slots are listed in ascending order (a fixed order: the subtractive
                    // output adds them up in list order, and the result must not depend on timing)
                    if (i < keep) {
                        if (kept) {
                            s_src[i] = (uint16_t)i;
                        } else {
                            if (hr < a.lds_slots / 2) s_holes[hr] = (uint16_t)i;
                            if (fused && hr < kMaxFix) s_evict[hr] = i;
                            ++hr;
                        }
                    } else if (kept) {
                        if (mr < a.lds_slots / 2) s_movers[mr] = (uint16_t)i;
                        ++mr;
                    } else if (fused) {
                        const int e = run_h + (i - keep) - mr;
                        if (e >= 0 && e < kMaxFix) s_evict[e] = i;
                    }
                }
                if (fused && tid == 0) {
                    const int ne = run_h + (m - keep) - run_m;
                    s_ecnt = ne < 0 ? 0 : (ne > kMaxFix ? kMaxFix : ne);
                }
                __syncthreads();
                n_moves = run_h < run_m ? run_h : run_m;
                n_moves = n_moves < a.lds_slots / 2 ? n_moves : a.lds_slots / 2;
                for (int k = tid; k < run_h; k += NT) {
                    if (k < a.lds_slots / 2) s_src[s_holes[k]] = (k < n_moves) ? s_movers[k] : s_holes[k];
                }
                __syncthreads();
                if (kout)
                    for (int j = tid; j < keep; j += NT) kout[j] = s_src[j];
            } else {
            // Ordered compaction of the kept flags.  A candidate is kept if its key
            // exceeds the threshold, or equals it and is among the first `rem` equals.  Every key
            // is read before the first barrier of the prefix sums, the list (which lies over the
            // key array) is written after them.
            uint64_t surem = 0ull, eqm = 0ull;      // kept for sure / equal to the threshold
            for (int k = 0; k < per; ++k) {
                const int i = lo + k;
                if (i >= hi) break;
                if (i >= ncand) {
                    surem |= 1ull << k;
                } else if (n_global > 0) {
                    const uint32_t key = s_key[i];
                    if (key > prefix) surem |= 1ull << k;
                    else if (key == prefix) eqm |= 1ull << k;
                }
            }
            int eq_before = 0, eq_total = 0;
            block_scan((int)__popcll(eqm), eq_before, eq_total);
            // the first (rem - eq_before) equals of this run are kept
            uint64_t keptm = surem;
            {
                int take = rem - eq_before;
                uint64_t e = eqm;
                while (take > 0 && e != 0ull) {
                    const uint64_t low = e & (~e + 1ull);
                    keptm |= low;
                    e ^= low;
                    --take;
                }
            }
            int out_pos = 0, out_total = 0;
            block_scan((int)__popcll(keptm), out_pos, out_total);
            for (int k = 0; k < per; ++k) {
                const int i = lo + k;
                if (i >= hi) break;
                if ((keptm >> k) & 1ull) {
                    s_kept[out_pos++] = (uint16_t)i;
                } else if (fused) {
                    const int e = i - out_pos;             // evicted slots before this one: ascending list
                    if (e < kMaxFix) s_evict[e] = i;
                }
            }
            if (fused && tid == 0) {
                const int ne = m - out_total;
                s_ecnt = ne < 0 ? 0 : (ne > kMaxFix ? kMaxFix : ne);
            }
            __syncthreads();
            if (kout)
                for (int j = tid; j < keep; j += NT) kout[j] = s_kept[j];
            }
        }

        // pre-compaction slot of the token that ends up in final slot j
        auto src_of = [&](int j) -> int {
            if (bag) return have_list ? (int)s_src[j] : (j == jstar ? len : j);
            return have_list ? (int)s_kept[j] : j + (j >= jstar ? 1 : 0);
        };

        // ---- output ---------------------------------------------------------------------------
        // kept mass 1 - sum_E p_j decides whether the subtractive form is safe
        bool subtract = fused;
        bool rows_moved = false;          // the output pass moved the value rows and the first key rows
        constexpr int UM = kWide ? 8 : 4; // rows per group and batch when rows change slot
        float pe = 0.f;
        int ec = 0;
        if (fused) {
            ec = s_ecnt;
            ec = ec > kMaxFix ? kMaxFix : ec;
#pragma unroll
            for (int k = 0; k < kMaxFix; ++k)
                if (k < ec) pe += s_p[s_evict[k]];
            subtract = (1.f - pe) >= kMinKeptMass;
        }

        if (subtract) {
            // out = (dense - sum_E p_j v_j) / (1 - sum_E p_j)
            for (int k = grp; k < ec; k += NG) {
                int idx = s_evict[k];
                idx = idx < 0 ? 0 : (idx > len ? len : idx);
                const float pw = s_p[idx];
                const char* vs = (idx >= stash_lo) ? s_stV + (idx - stash_lo) * ROWB : Vp + (int64_t)idx * ROWB;
                Vec16 vr = load16(vs + sub * 16);
                if (idx == len) vr = nv;
                float f[EPV];
                unpack<T>(vr, f);
#pragma unroll
                for (int e = 0; e < EPV; ++e) s_fix[k * D + sub * EPV + e] = pw * f[e];
            }
            __syncthreads();
            // one thread per output element: merge the wave partials relative to the global max
            for (int e = tid; e < D; e += NT) {
                float St = 0.f, At = 0.f;
#pragma unroll
                for (int v = 0; v < NW; ++v) {
                    const float r = fast_exp2((s_redA[v] - mx) * kLog2e);   // 0 for an empty wave (-inf)
                    St = __builtin_fmaf(s_wS[v], r, St);
                    At = __builtin_fmaf(s_acc[v * D + e], r, At);
                }
                float t = At / St;
                for (int k = 0; k < ec; ++k) t -= s_fix[k * D + e];
                write_out(e, t / (1.f - pe));
            }
        } else if (a.phase != 3) {       // (phase 3: the output is formed by the launches that follow)
            // gathered pass over the kept value rows: sum_kept p_i v_i / sum_kept p_i.
            // Unordered layout with many evictions (the step after a prompt): the rows that change
            // slot are moved inside this pass, so that the whole step needs one more memory round
            // trip instead of four.  A value row that moves is stored to its final slot as soon as
            // it has been accumulated (its destination is an evicted slot, which nobody reads), and
            // the key rows of the first NG*UM movers are requested before the value rows and stored
            // after the pass (sources lie at or above `keep`, destinations below: disjoint).
            __syncthreads();
            rows_moved = kWide && fc && bag && have_list;
            Vec16 kmv[UM];
            int kdst[UM];
            if (rows_moved) {
#pragma unroll
                for (int u = 0; u < UM; ++u) {
                    const int k = u * NG + grp;
                    kdst[u] = -1;
                    if (k < n_moves) {
                        int src = s_movers[k], dst = s_holes[k];
                        src = src > len ? len : src;
                        dst = dst >= keep ? keep - 1 : dst;
                        kmv[u] = load16(Kp + (int64_t)src * ROWB + sub * 16);
                        if (src == len) kmv[u] = nk;
                        kdst[u] = dst;
                    }
                }
            }
#pragma unroll
            for (int e = 0; e < EPV; ++e) acc[e] = 0.f;
            float ps = 0.f;
            for (int j0 = 0; j0 < keep; j0 += NG * UV) {
                Vec16 vv[UV];
                float pw[UV];
                int vdst[UV];
#pragma unroll
                for (int u = 0; u < UV; ++u) {
                    const int j = j0 + u * NG + grp;
                    vdst[u] = -1;
                    if (j < keep) {
                        int idx = src_of(j);
                        idx = idx < 0 ? 0 : (idx > len ? len : idx);
                        pw[u] = s_p[idx];
                        // (plain loads under fused compaction: the rows that move are read again)
                        vv[u] = fc ? load16(Vp + (int64_t)idx * ROWB + sub * 16)
                                   : load16_stream(Vp + (int64_t)idx * ROWB + sub * 16);
                        if (idx == len) vv[u] = nv;
                        if (rows_moved && idx != j) vdst[u] = j;
                    } else {
                        pw[u] = 0.f;
                        vv[u] = Vec16{0u, 0u, 0u, 0u};
                    }
                }
#pragma unroll
                for (int u = 0; u < UV; ++u) {
                    float f[EPV];
                    unpack<T>(vv[u], f);
#pragma unroll
                    for (int e = 0; e < EPV; ++e) acc[e] = __builtin_fmaf(pw[u], f[e], acc[e]);
                    ps += pw[u];
                    if (vdst[u] >= 0) store16(Vp + (int64_t)vdst[u] * ROWB + sub * 16, vv[u]);
                }
            }
            if (rows_moved) {
#pragma unroll
                for (int u = 0; u < UM; ++u)
                    if (kdst[u] >= 0) store16(Kp + (int64_t)kdst[u] * ROWB + sub * 16, kmv[u]);
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
                if (lane == 0) s_wS[wave] = ps;
            }
            __syncthreads();
            for (int e = tid; e < D; e += NT) {
                float pst = 0.f, t = 0.f;
#pragma unroll
                for (int v = 0; v < NW; ++v) {
                    pst += s_wS[v];
                    t += s_acc[v * D + e];
                }
                // (a budget that keeps no token - no local window and n r below one half - leaves an
                // empty sum: the output is zero)
                if (keep > 0) write_out(e, t / pst);
                else store_elem<AT>(a.out + pair * XROWB, e, 0.f);
            }
        }

        // ---- fused compaction: kept rows of K, V, score, pos go to slots 0..keep-1 -----------
        if (fc) {
            __syncthreads();   // s_sc, s_pos and the kept list of every thread are in LDS
            // final slot j holds the token of pre-compaction slot src(j)
            for (int j = tid; j < keep; j += NT) {
                int src = src_of(j);
                src = src < 0 ? 0 : (src > len ? len : src);
                Sp[j] = s_sc[src];
                if (src != j || src == len) Pp[j] = s_pos[src];
                if (has_ring) a.ring[(pair * a.ring_rows + a.ring_row) * (int64_t)cap + j] = s_p[src];
            }
            if (has_ring) {
                // The other rows of the ring follow the tokens that change slot (sources at or above
                // `keep`, destinations below it: disjoint); the new token's column is zero there.
                float* Rn = a.ring + pair * (int64_t)a.ring_rows * cap;
                const int Rr = a.ring_rows;
                if (!have_list) {
                    const int dst = (jstar < len) ? jstar : len;
                    if (dst < keep)
                        for (int j = tid; j < Rr; j += NT)
                            if (j != a.ring_row) Rn[(int64_t)j * cap + dst] = 0.f;
                } else {
                    for (int e = tid; e < n_moves * Rr; e += NT) {
                        const int k = e / Rr, j = e - k * Rr;
                        int src = s_movers[k], dst = s_holes[k];
                        src = src > len ? len : src;
                        dst = dst >= keep ? keep - 1 : dst;
                        if (j != a.ring_row) Rn[(int64_t)j * cap + dst] = (src == len) ? 0.f : Rn[(int64_t)j * cap + src];
                    }
                    if (len < keep)       // the new token stays in slot len: clear what the slot held before
                        for (int j = tid; j < Rr; j += NT)
                            if (j != a.ring_row) Rn[(int64_t)j * cap + len] = 0.f;
                }
            }
            if (bag) {
                // Sources (slots >= keep, or the new row) and destinations (holes < keep) are
                // disjoint, so the rows can move without any ordering.
                if (!have_list) {
                    // E <= 1: the only row written is the new one, into the hole or at the end
                    const int dst = (jstar < len) ? jstar : len;
                    if (dst < keep) {
                        if (tid < LPR) {
                            store16(Kp + (int64_t)dst * ROWB + sub * 16, nk);
                        } else if (tid < 2 * LPR) {
                            store16(Vp + (int64_t)dst * ROWB + sub * 16, nv);
                        }
                    }
                } else {
                    // UM rows per group in flight at a time, key rows and value rows in turn: a
                    // batch's loads are all issued before its first store.  After a gathered output
                    // pass only the key rows beyond its first batch are left.
                    for (int k0 = rows_moved ? NG * UM : 0; k0 < n_moves; k0 += NG * UM) {
#pragma unroll
                        for (int t = 0; t < (rows_moved ? 1 : 2); ++t) {
                            char* base = t == 0 ? Kp : Vp;
                            Vec16 rr[UM];
                            int dd[UM];
#pragma unroll
                            for (int u = 0; u < UM; ++u) {
                                const int k = k0 + u * NG + grp;
                                dd[u] = -1;
                                if (k < n_moves) {
                                    int src = s_movers[k], dst = s_holes[k];
                                    src = src > len ? len : src;
                                    dst = dst >= keep ? keep - 1 : dst;
                                    rr[u] = load16(base + (int64_t)src * ROWB + sub * 16);
                                    if (src == len) rr[u] = t == 0 ? nk : nv;
                                    dd[u] = dst;
                                }
                            }
#pragma unroll
                            for (int u = 0; u < UM; ++u)
                                if (dd[u] >= 0) store16(base + (int64_t)dd[u] * ROWB + sub * 16, rr[u]);
                        }
                    }
                }
            } else {
            // rows only move down; the prefix with src(j) == j stays (the new row always
            // counts as moved: it comes from k_new / v_new)
            int j0;
            if (have_list) {
                int lo = 0, hi = keep;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    const int sm = (int)s_kept[mid];
                    if (sm == mid && sm != len) lo = mid + 1; else hi = mid;
                }
                j0 = lo;
            } else {
                j0 = jstar < len ? jstar : len;
            }
            constexpr int UC = 4;
            constexpr int CH = NG * UC;
            for (int c0 = j0; c0 < keep; c0 += CH) {
                Vec16 kk[UC], vv2[UC];
                int dst[UC];
#pragma unroll
                for (int u = 0; u < UC; ++u) {
                    const int j = c0 + u * NG + grp;
                    dst[u] = -1;
                    if (j < keep) {
                        int src = src_of(j);
                        src = src < 0 ? 0 : (src > len ? len : src);
                        const char* ks = (src >= stash_lo) ? s_stK + (src - stash_lo) * ROWB : Kp + (int64_t)src * ROWB;
                        const char* vs = (src >= stash_lo) ? s_stV + (src - stash_lo) * ROWB : Vp + (int64_t)src * ROWB;
                        kk[u] = load16(ks + sub * 16);
                        vv2[u] = load16(vs + sub * 16);
                        if (src == len) {
                            kk[u] = nk;
                            vv2[u] = nv;
                        }
                        dst[u] = j;
                    }
                }
                // every source of the chunk is in registers before any destination is written
                asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
                __syncthreads();
#pragma unroll
                for (int u = 0; u < UC; ++u) {
                    if (dst[u] >= 0) {
                        store16(Kp + (int64_t)dst[u] * ROWB + sub * 16, kk[u]);
                        store16(Vp + (int64_t)dst[u] * ROWB + sub * 16, vv2[u]);
                    }
                }
            }
            }
        }
    }

    if (fc) {
        // The new length is published through kept_cnt (every head writes the same value);
        // cache_len is only read, so no workgroup can observe a half-updated step.
        // (every head of a sequence computes the same value: head 0 writes it)
        if (tid == 0) {
            if (overflow) atomicOr(a.status, kStatusCapacityBit);
            if (pair - (int64_t)s * a.h == 0) a.kept_cnt[s] = overflow ? len : keep;
        }
        return;
    }

    // ---- per-sequence arrival: the last head to finish publishes the new length --------
    // Every workgroup read cache_len[s] before it arrives here, and the publishing
    // store is issued only after the atomic has returned, so no reader can see it.
    if (tid == 0) {
        if (overflow) {
            atomicOr(a.status, kStatusCapacityBit);
        } else {
            a.kept_cnt[s] = keep;
            if (a.phase == 3) a.ws_ok[pair] = 1;
        }
        const int old = atomicAdd(&a.arrive[s], 1);
        if (old == a.h - 1) {
            atomicExch(&a.arrive[s], 0);
            if (!overflow) a.cache_len[s] = m;
        }
    }
}

// Local attention sum reduced along the head dimension (the note in Algorithm 1's header):
// tot[s, i] = sum over the heads of the new importance, fp32, head 0 first.
constexpr int kHeadSumThreads = 64;
__global__ void __launch_bounds__(kHeadSumThreads) swa_headsum_kernel(const float* snew, const int32_t* cache_len,
                                                                      float* tot, int h, int cap)
{
    const int s = blockIdx.y;
    const int i = blockIdx.x * kHeadSumThreads + threadIdx.x;
    const int m = cache_len[s] + 1;
    if (i >= m || i >= cap) return;
    const float* Sh = snew + (int64_t)s * h * cap + i;
    float t = 0.f;
    // eight loads in flight, added in head order
    int hh = 0;
    for (; hh + 8 <= h; hh += 8) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = Sh[(int64_t)(hh + k) * cap];
#pragma unroll
        for (int k = 0; k < 8; ++k) t += v[k];
    }
    for (; hh < h; ++hh) t += Sh[(int64_t)hh * cap];
    tot[(int64_t)s * cap + i] = t;
}

template <typename T, int D, int NT, bool RING>
static int launch_decode_nt(const DecodeArgs& a, int64_t pairs, size_t lds_bytes, hipStream_t stream)
{
    auto kern = swa_decode_kernel<T, D, NT, RING>;
    int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes);
    if (rc != SWA_OK) return rc;
    hipLaunchKernelGGL(kern, dim3((unsigned)pairs), dim3(NT), lds_bytes, stream, a);
    return hipGetLastError() == hipSuccess ? SWA_OK : SWA_ERR_HIP;
}

template <typename T, int D>
static int launch_decode_t(const DecodeArgs& a, int64_t pairs, size_t lds_bytes, int nt, hipStream_t stream)
{
    if (a.ring) {
        switch (nt) {
            case 128: return launch_decode_nt<T, D, 128, true>(a, pairs, lds_bytes, stream);
            case 256: return launch_decode_nt<T, D, 256, true>(a, pairs, lds_bytes, stream);
            default: return launch_decode_nt<T, D, 512, true>(a, pairs, lds_bytes, stream);
        }
    }
    switch (nt) {
        case 128: return launch_decode_nt<T, D, 128, false>(a, pairs, lds_bytes, stream);
        case 256: return launch_decode_nt<T, D, 256, false>(a, pairs, lds_bytes, stream);
        default: return launch_decode_nt<T, D, 512, false>(a, pairs, lds_bytes, stream);
    }
}

// Raise the dynamic-LDS limit of every instantiation to what the device allows next to the
// kernel's static LDS, so that no later launch has to (a launch inside a stream capture then
// makes no runtime call besides the launch itself).
template <typename T, int D, int NT, bool RING>
static int prepare_one()
{
    auto kern = swa_decode_kernel<T, D, NT, RING>;
    hipFuncAttributes fa;
    if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(kern)) != hipSuccess) {
        (void)hipGetLastError();
        return SWA_ERR_HIP;
    }
    int dev = 0, lds_max = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) {
        (void)hipGetLastError();
        return SWA_ERR_HIP;
    }
    const long long room = (long long)lds_max - (long long)fa.sharedSizeBytes;
    if (room <= 48 * 1024) return SWA_OK;
    return ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (size_t)room);
}

template <typename T, int D>
static int prepare_t()
{
    int rc = prepare_one<T, D, 128, false>();
    if (rc == SWA_OK) rc = prepare_one<T, D, 256, false>();
    if (rc == SWA_OK) rc = prepare_one<T, D, 512, false>();
    if (rc == SWA_OK) rc = prepare_one<T, D, 128, true>();
    if (rc == SWA_OK) rc = prepare_one<T, D, 256, true>();
    if (rc == SWA_OK) rc = prepare_one<T, D, 512, true>();
    return rc;
}

int prepare_decode()
{
    int rc = prepare_t<F32, 64>();
    if (rc == SWA_OK) rc = prepare_t<F32, 128>();
    if (rc == SWA_OK) rc = prepare_t<F16, 64>();
    if (rc == SWA_OK) rc = prepare_t<F16, 128>();
    if (rc == SWA_OK) rc = prepare_t<BF16, 64>();
    if (rc == SWA_OK) rc = prepare_t<BF16, 128>();
    if (rc == SWA_OK) rc = prepare_t<Q8, 64>();
    if (rc == SWA_OK) rc = prepare_t<Q8, 128>();
    return rc;
}

int launch_decode(const swa_params& p, float scale, const void* q, const void* k_new, const void* v_new,
                  void* k_cache, void* v_cache, float* score, int32_t* pos, int32_t* cache_len,
                  const int32_t* seq_len, int32_t* kept_idx, int32_t* kept_cnt, void* out,
                  float* probs_dbg, void* workspace, const float* qparams, float* ring, int32_t ring_rows,
                  int32_t ring_row, hipStream_t stream)
{
    DecodeArgs a;
    a.ring = ring;
    a.ring_rows = ring_rows;
    a.ring_row = ring_row;
    a.qparams = qparams;
    a.qstride = (int64_t)p.b * p.h * p.d;
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
    const int bound = (p.len_bound > 0 && p.len_bound < p.cap) ? p.len_bound : p.cap;
    a.lds_slots = (bound + 63) & ~63;
    a.w = p.w;
    a.sparsity_bp = p.sparsity_bp;
    a.scale = scale;
    a.fuse_compaction = (p.flags & SWA_FUSE_COMPACTION) ? 1 : 0;
    a.unordered = (a.fuse_compaction && (p.flags & SWA_UNORDERED)) ? 1 : 0;
    const bool shared = a.unordered && (p.flags & SWA_HEAD_SHARED);
    a.phase = 0;
    a.ws_z = nullptr;
    a.ws_ok = nullptr;
    a.ws_p = a.ws_snew = a.ws_abar = a.ws_tot = nullptr;
    if (shared) {
        char* base = static_cast<char*>(workspace) + shared_workspace_offset(p);
        const size_t slab = (size_t)p.b * p.h * p.cap * sizeof(float);
        a.ws_p = reinterpret_cast<float*>(base);
        a.ws_snew = reinterpret_cast<float*>(base + slab);
        a.ws_abar = reinterpret_cast<float*>(base + 2 * slab);
        a.ws_tot = reinterpret_cast<float*>(base + 2 * slab + (size_t)p.b * p.h * p.d * sizeof(float));
    }
    a.stash_rows = (a.fuse_compaction && !a.unordered) ? decode_stash_rows(p) : 0;

    const int64_t pairs = (int64_t)p.b * p.h;
    const int rowb = cache_row_bytes(p);
    const size_t lds_bytes = (size_t)a.lds_slots * (a.fuse_compaction ? (a.unordered ? 20 : 16) : 8) +
                             (size_t)a.stash_rows * rowb * 2;
    const int nt = decode_block_threads(pairs, bound, (p.flags & SWA_KV_INT8) != 0);

    auto launch = [&](const DecodeArgs& args) -> int {
        if (p.flags & SWA_KV_INT8) {
            return p.d == 64 ? launch_decode_t<Q8, 64>(args, pairs, lds_bytes, nt, stream)
                             : launch_decode_t<Q8, 128>(args, pairs, lds_bytes, nt, stream);
        } else if (p.dtype == SWA_F32) {
            return p.d == 64 ? launch_decode_t<F32, 64>(args, pairs, lds_bytes, nt, stream)
                             : launch_decode_t<F32, 128>(args, pairs, lds_bytes, nt, stream);
        } else if (p.dtype == SWA_F16) {
            return p.d == 64 ? launch_decode_t<F16, 64>(args, pairs, lds_bytes, nt, stream)
                             : launch_decode_t<F16, 128>(args, pairs, lds_bytes, nt, stream);
        }
        return p.d == 64 ? launch_decode_t<BF16, 64>(args, pairs, lds_bytes, nt, stream)
                         : launch_decode_t<BF16, 128>(args, pairs, lds_bytes, nt, stream);
    };
    if (p.flags & SWA_SPLIT_ROWS) {
        // rows of a pair over G workgroups: logits, then selection (this kernel, phase 3), then the output
        const int G = split_factor(pairs, bound);
        if (G > 1) {
            char* base = static_cast<char*>(workspace) + shared_workspace_offset(p);
            const size_t slab = (size_t)p.b * p.h * p.cap * sizeof(float);
            float* ws_z = reinterpret_cast<float*>(base);
            float* ws_pp = reinterpret_cast<float*>(base + slab);
            float* ws_part = reinterpret_cast<float*>(base + 2 * slab);
            int32_t* ws_ok = reinterpret_cast<int32_t*>(base + 2 * slab +
                                                        (size_t)pairs * kMaxSplit * (p.d + 1) * sizeof(float));
            int rc = launch_split(p, scale, 1, G, q, k_new, v_new, k_cache, v_cache, cache_len, kept_idx, kept_cnt,
                                  ws_z, ws_pp, ws_part, ws_ok, out, stream);
            if (rc != SWA_OK) return rc;
            a.phase = 3;
            a.ws_z = ws_z;
            a.ws_p = ws_pp;
            a.ws_ok = ws_ok;
            rc = launch(a);
            if (rc != SWA_OK) return rc;
            return launch_split(p, scale, 2, G, q, k_new, v_new, k_cache, v_cache, cache_len, kept_idx, kept_cnt,
                                ws_z, ws_pp, ws_part, ws_ok, out, stream);
        }
    }
    if (!shared) return launch(a);
    a.phase = 1;
    int rc = launch(a);
    if (rc != SWA_OK) return rc;
    hipLaunchKernelGGL(swa_headsum_kernel, dim3((unsigned)((bound + kHeadSumThreads - 1) / kHeadSumThreads), (unsigned)p.b),
                       dim3(kHeadSumThreads), 0, stream,
                       a.ws_snew, a.cache_len, a.ws_tot, (int)p.h, (int)p.cap);
    if (hipGetLastError() != hipSuccess) return SWA_ERR_HIP;
    a.phase = 2;
    return launch(a);
}

}  // namespace swa
