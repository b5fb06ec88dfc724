/*
 * swa_oracle.c -- fp64 CPU oracle for the decode-step Sparse Window Attention
 * (SWA) of ALISA (arXiv 2403.17312).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * statement of what the method computes.  It shares no code with the HIP
 * library, is never called by it, and must only be used by the tests, the
 * smoke check and the bench's cpu_baseline leg.
 *
 * Every floating-point value is a double.  Callers widen fp16/bf16/fp32 inputs
 * exactly.  Parallelism: an OpenMP "parallel for" over independent
 * (sequence, head) pairs and nothing else -- no blocking, no fusion, no SIMD
 * intrinsics, no BLAS.
 *
 * Tensors (row-major, C order):
 *   K, V        [b, h, cap, d]   cached keys / values; slot i of pair (s,hd)
 *   score       [b, h, cap]      running importance (local attention sum)
 *   pos         [b, h, cap]      original token position held by each slot
 *   cache_len   [b]              number of valid slots (shared by the heads)
 *   seq_len     [b]              logical length n, counting the token decoded
 *   kept_idx    [b, h, cap]      ascending slot list, first kept_cnt[s] valid
 *   kept_cnt    [b]
 *
 * Paper passages followed: Section II-A Eq. 1-2 (attention weights and
 * attention scores), the KV-caching paragraph of Section II-A and the caption
 * of the KV-caching figure (a decode step attends over stored K,V joined with
 * the new token's K,V and then stores them), and Section IV-B Algorithm 1
 * (budget, local attention sum, locally static + globally dynamic tokens,
 * gather, softmax over the gathered keys, weighted sum of gathered values).
 *
 * Readings taken where the paper leaves a choice (all listed in the design
 * document of this repository):
 *   - kept-set size is nearest-integer(n * r) with r = 1 - sparsity, halves
 *     rounded up, evaluated in integers on basis points (Alg. 1 line 1 uses the
 *     nearest-integer bracket on n*r/2 for each half);
 *   - the local window w is a separate argument; Algorithm 1's even split is
 *     the special case w = nearest-integer(n*r/2);
 *   - the importance score is a running sum of attention-weight rows: seeded
 *     with the sum of the last R prompt rows (Alg. 1 line 2) and increased by
 *     the current row at every decode step; the *_window routines instead keep
 *     the last R rows and sum exactly those, which is Alg. 1 line 2 to the
 *     letter (with the current row counted, as everywhere here);
 *   - global candidates exclude the local window, selection is per
 *     (sequence, head) -- or, on request, per sequence from the local
 *     attention sum reduced over the heads, as Algorithm 1's header notes --
 *     and ties go to the lowest slot;
 *   - the kept list is in ascending slot order and compaction preserves it.
 *
 * KV compression (Section V-B): the three quantisation routines at the end of
 * this file are the one place where single precision is used on purpose.  A
 * code is an integer decided by floating-point arithmetic, so the decision is
 * taken in the precision of the device library (IEEE fp32, one rounding per
 * operation, no contraction); de-quantisation back to the values the attention
 * reads is exact in fp64.  Readings: 8-bit unsigned codes; one (scale,
 * zero-point) pair per channel of every (sequence, head) pair, taken over the
 * cached tokens when the cache is quantised; the printed zero-point formula is
 * garbled, the zero point is nearest-integer(-min / scale) so that min maps to
 * code 0; "round" is nearest with ties to even; codes saturate at 0 and 255
 * (tokens appended later reuse the parameters); a channel whose range is below
 * 2^-7 takes that range, so the scale is never zero.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define SWA_ORACLE_OK 0
#define SWA_ORACLE_ERR_CAPACITY (-1)
#define SWA_ORACLE_ERR_ALLOC (-2)

int swa_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void swa_oracle_set_num_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* ------------------------------------------------------------------------ */
/* Budget (Alg. 1 line 1, generalised to an independent window w).          */
/*   keep_raw = nearest integer of n * (1 - sparsity), halves up            */
/*   n_local  = min(w, m)                                                   */
/*   keep     = min(m, max(keep_raw, n_local))                              */
/*   n_global = keep - n_local                                              */
/* n is the logical sequence length, m the number of slots in the cache.    */
/* w < 0 selects Algorithm 1's own even split: k = nearest integer of      */
/* n*r/2 locally static tokens and as many globally dynamic ones, i.e.     */
/* w = k and keep_raw = 2k.                                                 */
/* ------------------------------------------------------------------------ */
void swa_oracle_budget(int32_t n, int32_t m, int32_t w, int32_t sparsity_bp,
                       int32_t *keep, int32_t *n_local, int32_t *n_global)
{
    int64_t keep_raw = ((int64_t)n * (int64_t)(10000 - sparsity_bp) + 5000) / 10000;
    if (w < 0) {
        int64_t k = ((int64_t)n * (int64_t)(10000 - sparsity_bp) + 10000) / 20000;
        w = (int32_t)k;
        keep_raw = 2 * k;
    }
    int64_t wl = w < m ? w : m;
    int64_t k = keep_raw > wl ? keep_raw : wl;
    if (k > m) k = m;
    *keep = (int32_t)k;
    *n_local = (int32_t)wl;
    *n_global = (int32_t)(k - wl);
}

/* ------------------------------------------------------------------------ */
/* Append (KV caching, Section II-A): the new token's key and value join    */
/* the stored ones in slot cache_len, its position is n-1, its importance   */
/* starts at zero.  cache_len grows by one.                                  */
/* ------------------------------------------------------------------------ */
int swa_oracle_append(int32_t b, int32_t h, int32_t d, int32_t cap,
                      const double *k_new, const double *v_new,
                      double *K, double *V, double *score, int32_t *pos,
                      int32_t *cache_len, const int32_t *seq_len)
{
    for (int32_t s = 0; s < b; ++s)
        if (cache_len[s] + 1 > cap) return SWA_ORACLE_ERR_CAPACITY;
    for (int32_t s = 0; s < b; ++s) {
        int32_t slot = cache_len[s];
        for (int32_t hd = 0; hd < h; ++hd) {
            size_t pair = (size_t)s * h + hd;
            for (int32_t c = 0; c < d; ++c) {
                K[(pair * cap + slot) * d + c] = k_new[pair * d + c];
                V[(pair * cap + slot) * d + c] = v_new[pair * d + c];
            }
            score[pair * cap + slot] = 0.0;
            pos[pair * cap + slot] = seq_len[s] - 1;
        }
        cache_len[s] = slot + 1;
    }
    return SWA_ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Attention weights of one query row over the cached keys (Eq. 1):         */
/*   z_i = scale * sum_c q_c k_{i,c},  p = softmax(z) over the m slots.     */
/* probs beyond slot m are set to 0.                                         */
/* ------------------------------------------------------------------------ */
void swa_oracle_probs(int32_t b, int32_t h, int32_t d, int32_t cap, double scale,
                      const double *q, const double *K, const int32_t *cache_len,
                      double *probs)
{
    int64_t pairs = (int64_t)b * h;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t m = cache_len[pair / h];
        const double *qp = q + pair * d;
        const double *Kp = K + pair * (int64_t)cap * d;
        double *pp = probs + pair * (int64_t)cap;
        double zmax = -INFINITY;
        for (int32_t i = 0; i < m; ++i) {
            double z = 0.0;
            for (int32_t c = 0; c < d; ++c) z += qp[c] * Kp[(int64_t)i * d + c];
            z *= scale;
            pp[i] = z;
            if (z > zmax) zmax = z;
        }
        double denom = 0.0;
        for (int32_t i = 0; i < m; ++i) {
            pp[i] = exp(pp[i] - zmax);
            denom += pp[i];
        }
        for (int32_t i = 0; i < m; ++i) pp[i] /= denom;
        for (int32_t i = m; i < cap; ++i) pp[i] = 0.0;
    }
}

/* ------------------------------------------------------------------------ */
/* Importance accumulation: the local attention sum S of Alg. 1 line 2 kept */
/* as a running sum, S_i <- S_i + p_i for every cached slot.                 */
/* ------------------------------------------------------------------------ */
void swa_oracle_accumulate(int32_t b, int32_t h, int32_t cap, const double *probs,
                           const int32_t *cache_len, double *score)
{
    int64_t pairs = (int64_t)b * h;
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t m = cache_len[pair / h];
        for (int32_t i = 0; i < m; ++i)
            score[pair * cap + i] += probs[pair * cap + i];
    }
}

/* ------------------------------------------------------------------------ */
/* Selection (Alg. 1 lines 3-5).                                             */
/*   locally static  : the last n_local slots, kept unconditionally          */
/*   globally dynamic: the n_global earlier slots of largest S, found by a   */
/*                     full sort on (S descending, slot ascending)           */
/* Output: ascending slot list.                                               */
/* ------------------------------------------------------------------------ */
typedef struct {
    double s;
    int32_t slot;
} swa_cand;

static int cand_cmp(const void *a, const void *b)
{
    const swa_cand *x = (const swa_cand *)a, *y = (const swa_cand *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->slot > y->slot) - (x->slot < y->slot);
}

static int int32_cmp(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int swa_oracle_select(int32_t b, int32_t h, int32_t cap, int32_t w, int32_t sparsity_bp,
                      const double *score, const int32_t *cache_len, const int32_t *seq_len,
                      int32_t *kept_idx, int32_t *kept_cnt)
{
    int64_t pairs = (int64_t)b * h;
    int failed = 0;
    for (int32_t s = 0; s < b; ++s) {
        int32_t keep, nl, ng;
        swa_oracle_budget(seq_len[s], cache_len[s], w, sparsity_bp, &keep, &nl, &ng);
        kept_cnt[s] = keep;
    }
#pragma omp parallel for schedule(dynamic, 1) reduction(| : failed)
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t s = (int32_t)(pair / h);
        int32_t m = cache_len[s];
        int32_t keep, nl, ng;
        swa_oracle_budget(seq_len[s], m, w, sparsity_bp, &keep, &nl, &ng);
        int32_t ncand = m - nl;
        int32_t *out = kept_idx + pair * (int64_t)cap;
        swa_cand *cand = (swa_cand *)malloc(sizeof(swa_cand) * (size_t)(ncand > 0 ? ncand : 1));
        if (!cand) {
            failed = 1;
            continue;
        }
        for (int32_t i = 0; i < ncand; ++i) {
            cand[i].s = score[pair * cap + i];
            cand[i].slot = i;
        }
        qsort(cand, (size_t)ncand, sizeof(swa_cand), cand_cmp);
        int32_t cnt = 0;
        for (int32_t j = 0; j < ng; ++j) out[cnt++] = cand[j].slot; /* I^g */
        for (int32_t i = m - nl; i < m; ++i) out[cnt++] = i;        /* I^l */
        qsort(out, (size_t)cnt, sizeof(int32_t), int32_cmp);
        for (int32_t i = cnt; i < cap; ++i) out[i] = -1;
        free(cand);
    }
    return failed ? SWA_ORACLE_ERR_ALLOC : SWA_ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Selection with the local attention sum reduced along the head dimension   */
/* (the note in Algorithm 1's header): S_i = sum over heads of score[s,hd,i], */
/* one selection per sequence, every head of the sequence gets the same list. */
/* ------------------------------------------------------------------------ */
int swa_oracle_select_shared(int32_t b, int32_t h, int32_t cap, int32_t w, int32_t sparsity_bp,
                             const double *score, const int32_t *cache_len, const int32_t *seq_len,
                             int32_t *kept_idx, int32_t *kept_cnt)
{
    double *summed = (double *)calloc((size_t)b * cap, sizeof(double));
    int32_t *one = (int32_t *)malloc(sizeof(int32_t) * (size_t)b * cap);
    if (!summed || !one) {
        free(summed);
        free(one);
        return SWA_ORACLE_ERR_ALLOC;
    }
    for (int32_t s = 0; s < b; ++s)
        for (int32_t i = 0; i < cap; ++i) {
            double t = 0.0;
            for (int32_t hd = 0; hd < h; ++hd) t += score[((size_t)s * h + hd) * cap + i];
            summed[(size_t)s * cap + i] = t;
        }
    int rc = swa_oracle_select(b, 1, cap, w, sparsity_bp, summed, cache_len, seq_len, one, kept_cnt);
    if (rc == SWA_ORACLE_OK)
        for (int32_t s = 0; s < b; ++s)
            for (int32_t hd = 0; hd < h; ++hd)
                memcpy(kept_idx + ((size_t)s * h + hd) * cap, one + (size_t)s * cap, sizeof(int32_t) * (size_t)cap);
    free(summed);
    free(one);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Sparse attention (Alg. 1 lines 6-8): gather K_s, V_s by the kept list,    */
/* AW = softmax(q K_s^T * scale), Attn = AW V_s.                              */
/* ------------------------------------------------------------------------ */
int swa_oracle_sparse_attention(int32_t b, int32_t h, int32_t d, int32_t cap, double scale,
                                const double *q, const double *K, const double *V,
                                const int32_t *kept_idx, const int32_t *kept_cnt, double *out)
{
    int64_t pairs = (int64_t)b * h;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : failed)
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t cnt = kept_cnt[pair / h];
        const int32_t *I = kept_idx + pair * (int64_t)cap;
        double *Ks = (double *)malloc(sizeof(double) * (size_t)(cnt > 0 ? cnt : 1) * d);
        double *Vs = (double *)malloc(sizeof(double) * (size_t)(cnt > 0 ? cnt : 1) * d);
        double *aw = (double *)malloc(sizeof(double) * (size_t)(cnt > 0 ? cnt : 1));
        if (!Ks || !Vs || !aw) {
            failed = 1;
            free(Ks);
            free(Vs);
            free(aw);
            continue;
        }
        for (int32_t j = 0; j < cnt; ++j) {
            memcpy(Ks + (size_t)j * d, K + (pair * cap + I[j]) * d, sizeof(double) * d);
            memcpy(Vs + (size_t)j * d, V + (pair * cap + I[j]) * d, sizeof(double) * d);
        }
        double zmax = -INFINITY;
        for (int32_t j = 0; j < cnt; ++j) {
            double z = 0.0;
            for (int32_t c = 0; c < d; ++c) z += q[pair * d + c] * Ks[(size_t)j * d + c];
            aw[j] = z * scale;
            if (aw[j] > zmax) zmax = aw[j];
        }
        double denom = 0.0;
        for (int32_t j = 0; j < cnt; ++j) {
            aw[j] = exp(aw[j] - zmax);
            denom += aw[j];
        }
        for (int32_t c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int32_t j = 0; j < cnt; ++j) acc += (aw[j] / denom) * Vs[(size_t)j * d + c];
            out[pair * d + c] = acc;
        }
        free(Ks);
        free(Vs);
        free(aw);
    }
    return failed ? SWA_ORACLE_ERR_ALLOC : SWA_ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Compaction: pack the kept rows of K, V, score, pos into slots             */
/* 0..kept_cnt-1 in list order (the gather of Alg. 1 line 6 applied to the   */
/* cache itself); cache_len becomes kept_cnt.  Done through a scratch copy   */
/* so the result is the plain gather, with no in-place subtlety.             */
/* ------------------------------------------------------------------------ */
int swa_oracle_compact(int32_t b, int32_t h, int32_t d, int32_t cap,
                       double *K, double *V, double *score, int32_t *pos,
                       const int32_t *kept_idx, const int32_t *kept_cnt, int32_t *cache_len)
{
    int64_t pairs = (int64_t)b * h;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : failed)
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t cnt = kept_cnt[pair / h];
        const int32_t *I = kept_idx + pair * (int64_t)cap;
        size_t rows = (size_t)(cnt > 0 ? cnt : 1);
        double *Kt = (double *)malloc(sizeof(double) * rows * d);
        double *Vt = (double *)malloc(sizeof(double) * rows * d);
        double *st = (double *)malloc(sizeof(double) * rows);
        int32_t *pt = (int32_t *)malloc(sizeof(int32_t) * rows);
        if (!Kt || !Vt || !st || !pt) {
            failed = 1;
        } else {
            for (int32_t j = 0; j < cnt; ++j) {
                memcpy(Kt + (size_t)j * d, K + (pair * cap + I[j]) * d, sizeof(double) * d);
                memcpy(Vt + (size_t)j * d, V + (pair * cap + I[j]) * d, sizeof(double) * d);
                st[j] = score[pair * cap + I[j]];
                pt[j] = pos[pair * cap + I[j]];
            }
            memcpy(K + pair * (int64_t)cap * d, Kt, sizeof(double) * (size_t)cnt * d);
            memcpy(V + pair * (int64_t)cap * d, Vt, sizeof(double) * (size_t)cnt * d);
            memcpy(score + pair * (int64_t)cap, st, sizeof(double) * (size_t)cnt);
            memcpy(pos + pair * (int64_t)cap, pt, sizeof(int32_t) * (size_t)cnt);
        }
        free(Kt);
        free(Vt);
        free(st);
        free(pt);
    }
    if (failed) return SWA_ORACLE_ERR_ALLOC;
    for (int32_t s = 0; s < b; ++s) cache_len[s] = kept_cnt[s];
    return SWA_ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* One decode step, in the order the method is stated for this build:        */
/* append -> attention weights over the whole cache -> importance            */
/* accumulation -> budget + selection -> sparse attention over the kept set. */
/* probs may be NULL.  head_shared != 0 selects one token set per sequence   */
/* from the head-summed local attention sum.                                  */
/* ------------------------------------------------------------------------ */
int swa_oracle_decode_step(int32_t b, int32_t h, int32_t d, int32_t cap, int32_t w,
                           int32_t sparsity_bp, double scale,
                           const double *q, const double *k_new, const double *v_new,
                           double *K, double *V, double *score, int32_t *pos,
                           int32_t *cache_len, const int32_t *seq_len,
                           int32_t *kept_idx, int32_t *kept_cnt, double *out, double *probs,
                           int32_t head_shared)
{
    int rc = swa_oracle_append(b, h, d, cap, k_new, v_new, K, V, score, pos, cache_len, seq_len);
    if (rc) return rc;
    double *p = probs;
    if (!p) {
        p = (double *)malloc(sizeof(double) * (size_t)b * h * cap);
        if (!p) return SWA_ORACLE_ERR_ALLOC;
    }
    swa_oracle_probs(b, h, d, cap, scale, q, K, cache_len, p);
    swa_oracle_accumulate(b, h, cap, p, cache_len, score);
    if (!probs) free(p);
    rc = head_shared
             ? swa_oracle_select_shared(b, h, cap, w, sparsity_bp, score, cache_len, seq_len, kept_idx, kept_cnt)
             : swa_oracle_select(b, h, cap, w, sparsity_bp, score, cache_len, seq_len, kept_idx, kept_cnt);
    if (rc) return rc;
    return swa_oracle_sparse_attention(b, h, d, cap, scale, q, K, V, kept_idx, kept_cnt, out);
}

/* ------------------------------------------------------------------------ */
/* Prefill importance seed (Alg. 1 line 2 evaluated at the end of the        */
/* prompt): S_j = sum over the last R prompt rows of the causal attention    */
/* weight matrix.  Row r of q_tail is the query at position t = s - R + r    */
/* (s = cache_len); it attends to keys 0..t.  Rows with t < 0 do not exist   */
/* and contribute nothing.  score beyond slot s is set to 0.                  */
/* q_tail is [b, h, R, d].                                                    */
/* ------------------------------------------------------------------------ */
int swa_oracle_prefill_scores(int32_t b, int32_t h, int32_t d, int32_t cap, int32_t R,
                              double scale, const double *q_tail, const double *K,
                              const int32_t *cache_len, double *score)
{
    int64_t pairs = (int64_t)b * h;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : failed)
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t s = cache_len[pair / h];
        double *S = score + pair * (int64_t)cap;
        for (int32_t j = 0; j < cap; ++j) S[j] = 0.0;
        double *aw = (double *)malloc(sizeof(double) * (size_t)(s > 0 ? s : 1));
        if (!aw) {
            failed = 1;
            continue;
        }
        for (int32_t r = 0; r < R; ++r) {
            int32_t t = s - R + r;
            if (t < 0) continue;
            const double *qr = q_tail + (pair * R + r) * d;
            double zmax = -INFINITY;
            for (int32_t j = 0; j <= t; ++j) {
                double z = 0.0;
                for (int32_t c = 0; c < d; ++c) z += qr[c] * K[(pair * cap + j) * d + c];
                aw[j] = z * scale;
                if (aw[j] > zmax) zmax = aw[j];
            }
            double denom = 0.0;
            for (int32_t j = 0; j <= t; ++j) {
                aw[j] = exp(aw[j] - zmax);
                denom += aw[j];
            }
            for (int32_t j = 0; j <= t; ++j) S[j] += aw[j] / denom;
        }
        free(aw);
    }
    return failed ? SWA_ORACLE_ERR_ALLOC : SWA_ORACLE_OK;
}


/* ------------------------------------------------------------------------ */
/* Prefill attention: Eq. 1-2 over the whole prompt with the causal mask     */
/* (the grey upper triangle of the attention-weight figures).  For every     */
/* pair and every prompt position t < s = cache_len:                         */
/*   out[t] = sum_{j<=t} softmax_{j<=t}(q_t . k_j * scale) v_j.              */
/* Q and out are [b, h, cap, d] like the caches; rows >= s are left alone.   */
/* ------------------------------------------------------------------------ */
int swa_oracle_prefill_attention(int32_t b, int32_t h, int32_t d, int32_t cap, double scale,
                                 const double *Q, const double *K, const double *V,
                                 const int32_t *cache_len, double *out)
{
    int64_t pairs = (int64_t)b * h;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : failed)
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t s = cache_len[pair / h];
        double *aw = (double *)malloc(sizeof(double) * (size_t)(s > 0 ? s : 1));
        if (!aw) {
            failed = 1;
            continue;
        }
        for (int32_t t = 0; t < s; ++t) {
            const double *qt = Q + (pair * cap + t) * d;
            double zmax = -INFINITY;
            for (int32_t j = 0; j <= t; ++j) {
                double z = 0.0;
                for (int32_t c = 0; c < d; ++c) z += qt[c] * K[(pair * cap + j) * d + c];
                aw[j] = z * scale;
                if (aw[j] > zmax) zmax = aw[j];
            }
            double denom = 0.0;
            for (int32_t j = 0; j <= t; ++j) {
                aw[j] = exp(aw[j] - zmax);
                denom += aw[j];
            }
            double *o = out + (pair * cap + t) * d;
            for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
            for (int32_t j = 0; j <= t; ++j) {
                double p = aw[j] / denom;
                for (int32_t c = 0; c < d; ++c) o[c] += p * V[(pair * cap + j) * d + c];
            }
        }
        free(aw);
    }
    return failed ? SWA_ORACLE_ERR_ALLOC : SWA_ORACLE_OK;
}


/* ------------------------------------------------------------------------ */
/* Strict local attention sum (Alg. 1 line 2 taken literally): S is the sum  */
/* of the R most recent rows of the attention-weight matrix and nothing      */
/* older.  The rows are kept per pair in ring [b, h, R, cap]: ring row j     */
/* holds, slot by slot, the weights that one of the last R queries gave to   */
/* the tokens now cached (0 where the token did not exist yet).  A step      */
/* overwrites ring row `row` (the caller advances it modulo R, so the oldest */
/* row goes first).                                                          */
/* ------------------------------------------------------------------------ */

/* The last R rows of the prompt's causal attention-weight matrix, one per   */
/* ring row: ring row r is the query at position t = s - R + r over keys     */
/* 0..t; rows with t < 0 and entries beyond t are 0.                         */
int swa_oracle_prefill_rows(int32_t b, int32_t h, int32_t d, int32_t cap, int32_t R,
                            double scale, const double *q_tail, const double *K,
                            const int32_t *cache_len, double *ring)
{
    int64_t pairs = (int64_t)b * h;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t s = cache_len[pair / h];
        for (int32_t r = 0; r < R; ++r) {
            double *row = ring + (pair * R + r) * (int64_t)cap;
            for (int32_t j = 0; j < cap; ++j) row[j] = 0.0;
            int32_t t = s - R + r;
            if (t < 0) continue;
            const double *qr = q_tail + (pair * R + r) * d;
            double zmax = -INFINITY;
            for (int32_t j = 0; j <= t; ++j) {
                double z = 0.0;
                for (int32_t c = 0; c < d; ++c) z += qr[c] * K[(pair * cap + j) * d + c];
                row[j] = z * scale;
                if (row[j] > zmax) zmax = row[j];
            }
            double denom = 0.0;
            for (int32_t j = 0; j <= t; ++j) {
                row[j] = exp(row[j] - zmax);
                denom += row[j];
            }
            for (int32_t j = 0; j <= t; ++j) row[j] /= denom;
        }
    }
    return SWA_ORACLE_OK;
}

/* The current row replaces ring row `row`; score = sum of the R ring rows.  */
/* The token appended in this step (slot m-1) has no earlier rows.           */
void swa_oracle_window_accumulate(int32_t b, int32_t h, int32_t cap, int32_t R, int32_t row,
                                  const double *probs, const int32_t *cache_len, double *ring,
                                  double *score)
{
    int64_t pairs = (int64_t)b * h;
#pragma omp parallel for schedule(static)
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t m = cache_len[pair / h];
        double *Rg = ring + pair * (int64_t)R * cap;
        for (int32_t j = 0; j < R; ++j) Rg[(int64_t)j * cap + (m - 1)] = 0.0;
        for (int32_t i = 0; i < m; ++i) Rg[(int64_t)row * cap + i] = probs[pair * cap + i];
        for (int32_t i = 0; i < m; ++i) {
            double t = 0.0;
            for (int32_t j = 0; j < R; ++j) t += Rg[(int64_t)j * cap + i];
            score[pair * cap + i] = t;
        }
    }
}

/* The ring's columns follow their tokens through a compaction. */
int swa_oracle_compact_ring(int32_t b, int32_t h, int32_t cap, int32_t R, double *ring,
                            const int32_t *kept_idx, const int32_t *kept_cnt)
{
    int64_t pairs = (int64_t)b * h;
    int failed = 0;
#pragma omp parallel for schedule(static) reduction(| : failed)
    for (int64_t pair = 0; pair < pairs; ++pair) {
        int32_t cnt = kept_cnt[pair / h];
        double *tmp = (double *)malloc(sizeof(double) * (size_t)(cnt > 0 ? cnt : 1));
        if (!tmp) {
            failed = 1;
            continue;
        }
        for (int32_t j = 0; j < R; ++j) {
            double *row = ring + (pair * R + j) * (int64_t)cap;
            for (int32_t k = 0; k < cnt; ++k) tmp[k] = row[kept_idx[pair * cap + k]];
            for (int32_t k = 0; k < cnt; ++k) row[k] = tmp[k];
            for (int32_t k = cnt; k < cap; ++k) row[k] = 0.0;
        }
        free(tmp);
    }
    return failed ? SWA_ORACLE_ERR_ALLOC : SWA_ORACLE_OK;
}

/* One decode step with the strict local attention sum: as swa_oracle_decode_step, with the    */
/* importance taken from the ring instead of the running sum.  head_shared: the selection key  */
/* is that importance summed over the heads (the note in Algorithm 1's header applied to the   */
/* sum of its line 2), one token set per sequence.                                             */
int swa_oracle_decode_step_window(int32_t b, int32_t h, int32_t d, int32_t cap, int32_t w,
                                  int32_t sparsity_bp, double scale, int32_t R, int32_t row,
                                  const double *q, const double *k_new, const double *v_new,
                                  double *K, double *V, double *ring, double *score, int32_t *pos,
                                  int32_t *cache_len, const int32_t *seq_len,
                                  int32_t *kept_idx, int32_t *kept_cnt, double *out, double *probs,
                                  int32_t head_shared)
{
    int rc = swa_oracle_append(b, h, d, cap, k_new, v_new, K, V, score, pos, cache_len, seq_len);
    if (rc) return rc;
    swa_oracle_probs(b, h, d, cap, scale, q, K, cache_len, probs);
    swa_oracle_window_accumulate(b, h, cap, R, row, probs, cache_len, ring, score);
    rc = head_shared
             ? swa_oracle_select_shared(b, h, cap, w, sparsity_bp, score, cache_len, seq_len, kept_idx, kept_cnt)
             : swa_oracle_select(b, h, cap, w, sparsity_bp, score, cache_len, seq_len, kept_idx, kept_cnt);
    if (rc) return rc;
    return swa_oracle_sparse_attention(b, h, d, cap, scale, q, K, V, kept_idx, kept_cnt, out);
}


/* ------------------------------------------------------------------------ */
/* KV compression (Section V-B): x_q = round(x / lambda + z),               */
/* x = lambda * (x_q - z), lambda = (max - min) / (2^8 - 1).                */
/* X [b,h,rows,d] holds values exactly representable in fp32; count[s] rows */
/* of every pair of sequence s are valid.  lambda, zero: [b,h,d] fp32.      */
/* ------------------------------------------------------------------------ */
#define SWA_ORACLE_MIN_RANGE 0.0078125f /* 2^-7 */

void swa_oracle_kv_qparams(int32_t b, int32_t h, int32_t d, int32_t rows, const double *X,
                           const int32_t *count, float *lambda, float *zero)
{
    int64_t pairs = (int64_t)b * h;
#pragma omp parallel for schedule(static)
    for (int64_t pr = 0; pr < pairs; ++pr) {
        int32_t cnt = count[pr / h];
        const double *Xp = X + pr * (int64_t)rows * d;
        for (int32_t c = 0; c < d; ++c) {
            float lo = 0.0f, hi = 0.0f;
            for (int32_t i = 0; i < cnt; ++i) {
                float x = (float)Xp[(int64_t)i * d + c];
                if (i == 0 || x < lo) lo = x;
                if (i == 0 || x > hi) hi = x;
            }
            float range = hi - lo;
            if (range < SWA_ORACLE_MIN_RANGE) range = SWA_ORACLE_MIN_RANGE;
            float lam = range / 255.0f;
            float t = -lo / lam;
            lambda[pr * d + c] = lam;
            zero[pr * d + c] = rintf(t);
        }
    }
}

static uint8_t quantise_one(float x, float lam, float z)
{
    float t = x / lam;
    t = t + z;
    t = rintf(t);
    if (t < 0.0f) t = 0.0f;
    if (t > 255.0f) t = 255.0f;
    return (uint8_t)t;
}

void swa_oracle_kv_quantize(int32_t b, int32_t h, int32_t d, int32_t rows, const double *X,
                            const int32_t *count, const float *lambda, const float *zero,
                            uint8_t *codes)
{
    int64_t pairs = (int64_t)b * h;
#pragma omp parallel for schedule(static)
    for (int64_t pr = 0; pr < pairs; ++pr) {
        int32_t cnt = count[pr / h];
        for (int32_t i = 0; i < cnt; ++i)
            for (int32_t c = 0; c < d; ++c) {
                int64_t at = (pr * rows + i) * (int64_t)d + c;
                codes[at] = quantise_one((float)X[at], lambda[pr * d + c], zero[pr * d + c]);
            }
    }
}

void swa_oracle_kv_dequantize(int32_t b, int32_t h, int32_t d, int32_t rows, const uint8_t *codes,
                              const int32_t *count, const float *lambda, const float *zero,
                              double *X)
{
    int64_t pairs = (int64_t)b * h;
#pragma omp parallel for schedule(static)
    for (int64_t pr = 0; pr < pairs; ++pr) {
        int32_t cnt = count[pr / h];
        for (int32_t i = 0; i < cnt; ++i)
            for (int32_t c = 0; c < d; ++c) {
                int64_t at = (pr * rows + i) * (int64_t)d + c;
                X[at] = (double)lambda[pr * d + c] * ((double)codes[at] - (double)zero[pr * d + c]);
            }
    }
}
