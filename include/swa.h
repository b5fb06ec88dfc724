/*
 * swa.h -- C ABI of the MI355X (gfx950) Sparse Window Attention decode library.
 *
 * The library implements one transformer layer's batched decode-step Sparse
 * Window Attention (SWA) of ALISA (arXiv 2403.17312, Section IV-B, Algorithm 1)
 * over a KV cache that lives in device memory, for b sequences x h heads of
 * head dimension d.  Every (sequence, head) pair is independent.
 *
 * Conventions that hold for every entry point unless stated otherwise
 *   - `swa_params*` is a HOST pointer; every other pointer is a DEVICE pointer
 *     owned by the caller.  The library never allocates or frees device memory.
 *     The state it keeps per process is small and internal: which kernels have had
 *     their LDS limit raised, and the device address of the fixed scratch array of
 *     swa_decode_step_static.  Everything a call computes goes through its arguments.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     only enqueue work: they never synchronise and never read device memory on
 *     the host, so a sequence of calls can be captured into a HIP graph.  A decode
 *     launch that needs more than 48 KiB of LDS first raises the kernel's limit
 *     (a host-side runtime call, once per kernel); call swa_prepare() once per
 *     device beforehand and no call made during a capture does anything but launch.
 *   - Return value: SWA_OK (0) or a negative swa_status.  Errors that the host
 *     can see (null pointers, unsupported shapes) are reported before anything
 *     is enqueued.  A condition only the device can see (a sequence whose cache
 *     is full) never writes out of bounds: the affected pairs are skipped and a
 *     sticky bit is set in the workspace, readable with swa_check_status().
 *   - Tensors are dense, row-major:
 *       k_cache, v_cache  [b, h, cap, d]   element type params->dtype (8-bit codes with SWA_KV_INT8)
 *       score             [b, h, cap]      float32 running importance
 *       pos               [b, h, cap]      int32 original token position
 *       kept_idx          [b, h, cap]      int32 ascending slot list
 *       cache_len, seq_len, kept_cnt [b]   int32 (shared by the heads)
 *     Slot i < cache_len[s] of pair (s, hd) is valid; higher slots are free.
 *   - Supported shapes: d in {64, 128}; dtype float32, float16 or bfloat16;
 *     cap <= SWA_MAX_CAP.
 */
#ifndef SWA_H_
#define SWA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SWA_MAX_CAP 16384 /* slots per (sequence, head); bounded by LDS per workgroup */
#define SWA_MAX_PREFILL_ROWS 128
#define SWA_W_EVEN_SPLIT (-1)

typedef enum { SWA_F32 = 0, SWA_F16 = 1, SWA_BF16 = 2 } swa_dtype;

typedef enum {
    SWA_OK = 0,
    SWA_ERR_NULL = -1,              /* a required pointer is NULL */
    SWA_ERR_BAD_SHAPE = -2,         /* b, h, cap, w or R out of range */
    SWA_ERR_UNSUPPORTED_D = -3,     /* d not in {64, 128} */
    SWA_ERR_UNSUPPORTED_DTYPE = -4, /* dtype not a swa_dtype, or a cache format the call does not take */
    SWA_ERR_BAD_SPARSITY = -5,      /* sparsity_bp outside 0..9999 */
    SWA_ERR_CAPACITY = -6,          /* cap above SWA_MAX_CAP, or (status) a cache was full */
    SWA_ERR_HIP = -7,               /* a HIP runtime call failed */
    SWA_ERR_ALIGNMENT = -8,         /* a row pointer is not 16-byte aligned */
    SWA_ERR_HOST_STORE_FULL = -9,   /* (status) a pair's host store had no room for its evicted tokens */
    SWA_ERR_BAD_REQUEST = -10       /* (status) a reload named a token that the host store does not hold */
} swa_status;

typedef struct {
    int32_t b;           /* sequences */
    int32_t h;           /* heads */
    int32_t d;           /* head dimension, 64 or 128 */
    int32_t cap;         /* slots per (sequence, head) in every cache tensor */
    int32_t w;           /* local window: the most recent w tokens are always kept (>= 0), or
                            SWA_W_EVEN_SPLIT for Algorithm 1's own rule, w = nint(n*r/2) per
                            sequence with as many globally dynamic tokens */
    int32_t sparsity_bp; /* KV sparsity in basis points, 0..9999; caching ratio r = 1 - sparsity */
    int32_t dtype;       /* swa_dtype of q, k_new, v_new, caches, out */
    float scale;         /* logit scale; 0 selects 1/sqrt(d) (Eq. 1) */
    int32_t len_bound;   /* 0, or an upper bound on cache_len[s] + 1 over all sequences for this
                            call: lets swa_decode_step size its LDS to the live cache instead of
                            cap.  A sequence that exceeds it is skipped and reported exactly like
                            a full cache (capacity status bit). */
    int32_t flags;       /* 0 or a combination of the SWA_* flag bits below */
} swa_params;

/*
 * swa_params.flags bit: swa_decode_step also compacts the cache (the work of
 * swa_compact_kv) inside the same kernel.  In this mode
 *   - cache_len is only READ; the new length of sequence s is written to kept_cnt[s]
 *     (kept_cnt[s] = cache_len[s] for a skipped sequence).  The caller passes the two arrays
 *     swapped on the next call.  (Publishing the length through the array that the same
 *     launch reads would need a grid-wide ordering; a second array needs none.)
 *   - on return the kept rows of k_cache, v_cache, score and pos sit in slots 0..kept_cnt-1,
 *     order preserved; swa_compact_kv must not be called for this step;
 *   - kept_idx may be NULL; when given it receives the ascending list of PRE-compaction
 *     slots that were kept, as in the unfused call.
 *   - LDS holds 16 bytes per live slot instead of 8: len_bound (or cap) above 9216 is
 *     refused with SWA_ERR_CAPACITY.
 */
#define SWA_FUSE_COMPACTION 1
#define SWA_MAX_FUSED_SLOTS 9216

/*
 * swa_params.flags bit, only together with SWA_FUSE_COMPACTION: the compacted cache need not be
 * in token order.  The method's result does not depend on the order of the cached rows once the
 * window and the tie rule are stated on token positions, so in this mode
 *   - the local window is the set of slots with pos >= seq_len - w (the most recent w tokens),
 *     and ties of the top-k go to the EARLIEST token (lowest pos); for a cache in token order
 *     both coincide with the slot-based rules of the ordered mode;
 *   - compaction fills the holes below kept_cnt with the kept rows above it (in the steady
 *     state the new token simply takes the evicted token's slot: no row moves at all);
 *   - kept_idx[j], when given, is the PRE-compaction slot of the token that ends in slot j.
 * pos must hold each slot's token position (it does after any sequence of calls that started
 * from a cache filled in token order with pos = 0..len-1).  Up to 7168 live slots.
 * The most recent min(w, m) tokens are all still cached as long as the effective window grows by
 * at most one token per step (always true for a fixed w, and for SWA_W_EVEN_SPLIT at a fixed
 * sparsity).  If a caller widens it faster, some positions of the new window were evicted
 * earlier: the step keeps every window token that is present and makes up the rest of the budget
 * with global tokens, so the cache stays dense and holds exactly `keep` tokens.  (The ordered
 * forms keep the most recent SLOTS instead; the two agree whenever no window position is missing.)
 */
#define SWA_UNORDERED 2
#define SWA_MAX_UNORDERED_SLOTS 7168

/*
 * swa_params.flags bit, only together with SWA_FUSE_COMPACTION | SWA_UNORDERED: the local attention
 * sum is reduced along the head dimension before the selection (the note in Algorithm 1's header):
 * the globally dynamic tokens of sequence s are the top-k of sum_hd score[s, hd, i], and all heads
 * of the sequence keep the same token set.  score stays per head (each head accumulates its own
 * attention weights); the sum over the heads is taken in fp32, head 0 first.  The call enqueues
 * three kernels (stream and publish; sum over the heads; select and finish) and needs the larger
 * workspace that swa_workspace_bytes reports for these flags.
 */
#define SWA_HEAD_SHARED 4

/*
 * swa_params.flags bit: k_cache and v_cache hold 8-bit codes (Section V-B, KV compression): rows
 * of d bytes, [b,h,cap,d] uint8, produced by swa_quantize_kv.  dtype must be SWA_F16 (the format
 * the paper de-quantises to) and describes q, k_new, v_new and out.  Set for
 * swa_decode_step_q8 and for swa_compact_kv on such a cache; swa_decode_step refuses it.
 */
#define SWA_KV_INT8 8

/*
 * One-time set-up on the current device, optional but needed before stream capture: raises the
 * LDS limit of every decode kernel to the device's maximum and looks up the scratch array of
 * swa_decode_step_static.  Host-side only; enqueues nothing.  Call it again after hipSetDevice
 * to another GPU.
 */
int swa_prepare(void);

/*
 * swa_params.flags bit, on its own (the two-call form: swa_decode_step, then swa_compact_kv whenever
 * the caller wants): the rows of one (sequence, head) pair are split over several workgroups.  For
 * few pairs with long caches - small batches, long contexts, caches that are compacted rarely or
 * never - one workgroup per pair leaves most of the GPU idle.  The call then enqueues four kernels
 * (logits of a slice of the keys per workgroup; softmax, importance and selection per pair;
 * partial outputs over slices of the kept list; their sum) and needs the larger workspace that
 * swa_workspace_bytes reports for this flag.  Attention weights, importance and the kept set are
 * bit-identical to the one-workgroup form; the output's partial sums are added in another order.
 * With many pairs or short caches (more than 128 pairs, or a length bound below 2048 rows: there the
 * extra launches cost more than the slices gain) the call runs the one-workgroup kernel.
 */
#define SWA_SPLIT_ROWS 16

/* Message for a swa_status code (static storage, never NULL). */
const char *swa_strerror(int code);

/* Bytes of device workspace the other calls need for these params (0 on invalid params).
 * The caller allocates it (256-byte aligned) and calls swa_workspace_init once. */
size_t swa_workspace_bytes(const swa_params *params);

/* Enqueue a fill that zeroes the workspace (status bits and arrival counters). */
int swa_workspace_init(const swa_params *params, void *workspace, void *stream);

/* Synchronises `stream`, copies the sticky status bits to the host and clears them.
 * *status_out = SWA_OK, SWA_ERR_CAPACITY (some step met a full cache), SWA_ERR_HOST_STORE_FULL or
 * SWA_ERR_BAD_REQUEST (offload tier), the first of these that applies.
 * workspace == NULL reads the status word of swa_decode_step_static on the current device.
 * This is the only entry point that blocks. */
int swa_check_status(const swa_params *params, void *workspace, void *stream, int32_t *status_out);

/*
 * Budget of Algorithm 1 line 1, generalised to an independent local window.
 * Host-only helper (no device work): for logical length n and m cached slots,
 *   keep_raw = nearest integer of n * (1 - sparsity)   (halves round up)
 *   n_local  = min(w, m)
 *   keep     = min(m, max(keep_raw, n_local)),  n_global = keep - n_local.
 * w = SWA_W_EVEN_SPLIT is Algorithm 1 line 1 itself: k = nearest integer of n*r/2 (halves
 * round up), w = k and keep_raw = 2k.
 * Without a local window and with n*r below one half the budget is keep = 0: the decode step then
 * attends over the empty set, writes out = 0, and leaves an empty cache.
 */
int swa_budget(int32_t n, int32_t m, int32_t w, int32_t sparsity_bp, int32_t *keep,
               int32_t *n_local, int32_t *n_global);

/*
 * Prefill importance seed: Algorithm 1 line 2 ("local attention sum")
 * evaluated at the end of the prompt.  For every pair,
 *   score[j] = sum over r < R of softmax_causal(q_tail[r] . K^T * scale)[j]
 * where row r of q_tail is the query at position t = cache_len - R + r and
 * attends to keys 0..t (Eq. 1 with the causal mask); rows with t < 0 are
 * ignored.  score[j] = 0 for cache_len <= j < cap.  Runs on MFMA.
 *   q_tail [b,h,R,d] dtype (in), 1 <= R <= SWA_MAX_PREFILL_ROWS
 *   k_cache (in), cache_len [b] (in), score (out).
 */
int swa_prefill_scores(const swa_params *params, const void *q_tail, int32_t R,
                       const void *k_cache, const int32_t *cache_len, float *score,
                       void *workspace, void *stream);

/*
 * One decode step of Sparse Window Attention for every pair (Section II-A
 * KV caching; Algorithm 1):
 *   1. append: k_new, v_new go to slot len = cache_len[s]; pos[len] = seq_len[s]-1;
 *      score[len] = 0; m = len + 1;
 *   2. attention weights over the whole cache (Eq. 1): p = softmax(q . K^T * scale)
 *      over the m slots, fp32;
 *   3. importance: score[i] += p[i]  (running local attention sum, Alg. 1 line 2);
 *   4. budget + selection (Alg. 1 lines 1, 3-5): keep/n_local/n_global from
 *      swa_budget(seq_len[s], m, w, sparsity); kept = the last n_local slots plus
 *      the n_global earlier slots of largest score (ties: lowest slot);
 *      kept_idx gets the ascending list, kept_cnt[s] = keep;
 *   5. output (Alg. 1 lines 6-8): softmax over the kept keys times their
 *      values, i.e. out = sum_kept p_i v_i / sum_kept p_i, rounded once to dtype.
 * The cache is left uncompacted; cache_len[s] becomes m.  Calling again without
 * swa_compact_kv is legal (all m slots stay candidates).
 *   q, k_new, v_new [b,h,d] (in); k_cache, v_cache, score, pos (in/out);
 *   cache_len [b] (in/out); seq_len [b] (in) logical length n counting this token;
 *   kept_idx, kept_cnt, out [b,h,d] (out); see SWA_FUSE_COMPACTION for the fused variant;
 *   probs_dbg [b,h,cap] float32 or NULL: receives p (0 beyond m) when given.
 * A sequence with cache_len[s] + 1 > cap is skipped (nothing written for it)
 * and the capacity status bit is set.
 */
int swa_decode_step(const swa_params *params, const void *q, const void *k_new, const void *v_new,
                    void *k_cache, void *v_cache, float *score, int32_t *pos, int32_t *cache_len,
                    const int32_t *seq_len, int32_t *kept_idx, int32_t *kept_cnt, void *out,
                    float *probs_dbg, void *workspace, void *stream);

/*
 * swa_decode_step for callers that cannot allocate device memory or carry a workspace around:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, steps, flag variants (SWA_KV_INT8 excepted) and results as swa_decode_step, without
 * the workspace: status word, arrival counters and the head-shared slabs live in a fixed array
 * of SWA_STATIC_SCRATCH_BYTES inside the library, one per GPU, held until the process ends.
 *   - params whose swa_workspace_bytes() exceeds SWA_STATIC_SCRATCH_BYTES are refused with
 *     SWA_ERR_CAPACITY before anything is enqueued (in practice: b beyond two million, or a
 *     head-shared step whose b*h*cap slabs do not fit).
 *   - Calls no hipMalloc/hipFree and no allocating routine; the first call on a device looks the
 *     array's address up (swa_prepare does the same ahead of time).
 *   - Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU
 *     (different streams, or graphs replayed concurrently) race.  Calls on one stream are safe.
 *   - The two-call form enqueues one small fill kernel that zeroes the arrival counters first.
 *   - The sticky status word is read with swa_check_status(params, NULL, stream, &st).
 */
#define SWA_STATIC_SCRATCH_BYTES (8u << 20)
int swa_decode_step_static(const swa_params *params, const void *q, const void *k_new,
                           const void *v_new, void *k_cache, void *v_cache, float *score,
                           int32_t *pos, int32_t *cache_len, const int32_t *seq_len,
                           int32_t *kept_idx, int32_t *kept_cnt, void *out, float *probs_dbg,
                           void *stream);

/*
 * In-place compaction of the cache to the kept set (the gather of Algorithm 1
 * line 6 applied to the cache itself): for every pair, row kept_idx[j] of
 * k_cache, v_cache, score and pos moves to slot j, j < kept_cnt[s], order
 * preserved; cache_len[s] = kept_cnt[s].  kept_idx must be ascending (as
 * swa_decode_step writes it).  Bit-exact copies.
 */
int swa_compact_kv(const swa_params *params, void *k_cache, void *v_cache, float *score,
                   int32_t *pos, const int32_t *kept_idx, const int32_t *kept_cnt,
                   int32_t *cache_len, void *workspace, void *stream);

/*
 * KV compression, Section V-B: x_q = round(x / lambda + z), x = lambda (x_q - z),
 * lambda = (max - min) / (2^8 - 1), channel-wise.  For every pair and every channel c < d the
 * extrema run over the cached tokens 0..cache_len[s]-1; z = nint(-min / lambda) (the code that min
 * maps to 0 with; the paper's printed zero point is garbled); "round" is to nearest, ties to
 * even; codes saturate at 0 and 255; a channel whose range is below 2^-7 (or an empty cache)
 * takes that range.  All of it in fp32, one rounding per operation.
 *   k_cache, v_cache [b,h,cap,d] fp16 (in); cache_len [b] (in);
 *   k_codes, v_codes [b,h,cap,d] uint8 (out; slots >= cache_len untouched);
 *   qparams [4, b,h,d] float32 (out): lambda_K, z_K, lambda_V, z_V.
 * params->dtype must be SWA_F16; SWA_KV_INT8 in flags is accepted and ignored.
 */
int swa_quantize_kv(const swa_params *params, const void *k_cache, const void *v_cache,
                    const int32_t *cache_len, void *k_codes, void *v_codes, float *qparams,
                    void *stream);

/*
 * swa_decode_step over a compressed cache (Section V-B: KV tensors are integers in memory and
 * are de-quantised for the computation).  Same steps, arguments and flag variants as
 * swa_decode_step, except
 *   - params->flags must contain SWA_KV_INT8, dtype must be SWA_F16;
 *   - k_codes, v_codes [b,h,cap,d] uint8 (in/out) take the place of k_cache, v_cache;
 *   - qparams [4, b,h,d] float32 (in) as written by swa_quantize_kv;
 *   - the new token's k_new, v_new (fp16) are quantised with the pair's parameters on arrival
 *     (saturating), and the step attends over the de-quantised codes of all m slots, the new
 *     one included: every value the attention reads is lambda_c (code - z_c), exactly.
 * Scores are accumulated in fp32 as q_c lambda_c times the code; out is rounded once to fp16.
 */
int swa_decode_step_q8(const swa_params *params, const void *q, const void *k_new,
                       const void *v_new, void *k_codes, void *v_codes, const float *qparams,
                       float *score, int32_t *pos, int32_t *cache_len, const int32_t *seq_len,
                       int32_t *kept_idx, int32_t *kept_cnt, void *out, float *probs_dbg,
                       void *workspace, void *stream);

/*
 * Strict local attention sum: Algorithm 1 line 2 to the letter.  The importance of a cached
 * token is the sum of the attention weights it received from the R most recent queries and from
 * no older one (swa_decode_step keeps a running sum instead).  The rows are kept per pair in
 *   ring [b,h,R,cap] float32: ring[s,hd,j,i] = weight that the query of ring row j gave to the
 *   token now in slot i (0 where the token did not exist yet, or for a row not written yet).
 */
#define SWA_MAX_WINDOW_ROWS 64

/*
 * The ring at the end of the prompt: ring row r = attention weights of the prompt query at
 * position t = cache_len - R + r over keys 0..t (Eq. 1 with the causal mask); rows with t < 0 and
 * entries beyond t or beyond cache_len are 0.  Their sum over r is what swa_prefill_scores gives.
 * Decode step number k (0-based) after this call should replace ring row k mod R (oldest first).
 *   q_tail [b,h,R,d] dtype (in), 1 <= R <= SWA_MAX_WINDOW_ROWS; k_cache, cache_len (in); ring (out).
 */
int swa_prefill_rows(const swa_params *params, const void *q_tail, int32_t R, const void *k_cache,
                     const int32_t *cache_len, float *ring, void *workspace, void *stream);

/*
 * swa_decode_step with the strict local attention sum.  params->flags must contain
 * SWA_FUSE_COMPACTION | SWA_UNORDERED (the ring's columns follow their tokens through the
 * hole-filling compaction only) and may add SWA_HEAD_SHARED: the selection key is then the sum
 * over the heads of the per-head window sums (Algorithm 1's header note together with its
 * line 2), with the larger workspace of that flag.  Differences from swa_decode_step:
 *   3'. importance: ring row `ring_row` (0 <= ring_row < R) is replaced by this step's weights p,
 *       and score[i] = sum over the R ring rows at slot i, added in row order in fp32; the token
 *       appended in this step has no earlier rows.  score is output only (the old content is
 *       not read); selection, output and compaction then proceed as usual, and the ring's
 *       columns move with their tokens, so ring stays aligned with the compacted cache.
 * ring [b,h,R,cap] (in/out).  The caller advances ring_row by one modulo R per step.
 */
int swa_decode_step_window(const swa_params *params, const void *q, const void *k_new,
                           const void *v_new, void *k_cache, void *v_cache, float *ring, int32_t R,
                           int32_t ring_row, float *score, int32_t *pos, int32_t *cache_len,
                           const int32_t *seq_len, int32_t *kept_idx, int32_t *kept_cnt, void *out,
                           float *probs_dbg, void *workspace, void *stream);

/*
 * swa_decode_step_window over a compressed cache (Section V-B together with Algorithm 1 line 2):
 * arguments as swa_decode_step_q8 (k_codes, v_codes, qparams; flags contain SWA_KV_INT8) plus the
 * ring arguments of swa_decode_step_window.  The ring at the end of the prompt comes from
 * swa_prefill_rows on the fp16 cache, before swa_quantize_kv compresses it.
 */
int swa_decode_step_window_q8(const swa_params *params, const void *q, const void *k_new,
                              const void *v_new, void *k_codes, void *v_codes, const float *qparams,
                              float *ring, int32_t R, int32_t ring_row, float *score, int32_t *pos,
                              int32_t *cache_len, const int32_t *seq_len, int32_t *kept_idx,
                              int32_t *kept_cnt, void *out, float *probs_dbg, void *workspace,
                              void *stream);

/*
 * Prefill: dense causal attention over the whole prompt (Eq. 1-2 with the causal mask) plus the
 * importance seed of swa_prefill_scores (every dtype; tuned for the 16-bit ones).  For every pair and every prompt
 * position t < cache_len[s]:
 *   out[t] = sum_{j<=t} softmax_{j<=t}(q[t] . K[j] * scale) V[j], rounded once to dtype;
 * if R > 0, score gets the column sums of the last R rows of that attention-weight matrix
 * (queries q[cache_len-R .. cache_len-1]), exactly as swa_prefill_scores would with those rows.
 * Runs on MFMA (flash-style: the s x s weight matrix is never stored).
 *   q, out [b,h,cap,d] dtype (rows >= cache_len are neither read nor written);
 *   k_cache, v_cache (in); cache_len [b] (in); 0 <= R <= SWA_MAX_PREFILL_ROWS;
 *   score [b,h,cap] (out) or NULL when R == 0.  params->len_bound, if set, bounds cache_len.
 */
int swa_prefill_attention(const swa_params *params, const void *q, const void *k_cache,
                          const void *v_cache, const int32_t *cache_len, void *out, int32_t R,
                          float *score, void *workspace, void *stream);

/*
 * Token-level offload tier: the store and load halves of the GPU-CPU caching phase of the
 * paper's dynamic scheduling (Section V-A, Algorithm 2, Phase II: tokens that leave GPU memory are
 * stored in CPU memory, tokens needed again are loaded back; KV tensors are managed per token, not
 * per head).  When to offload and what to load back is the scheduler's policy and not part of this
 * library; recomputation (Phase III) needs the model and is out of scope.
 *
 * The host store of one layer, owned by the caller:
 *   k, v    [b, h, host_cap, d]  PINNED host memory that the device can address (hipHostMalloc,
 *                                 or a framework's pinned allocation), element type of the cache
 *                                 (8-bit codes with SWA_KV_INT8);
 *   score   [b, h, host_cap]     float32, pinned host: importance at the time of eviction;
 *   pos     [b, h, host_cap]     int32, pinned host: token position;
 *   len     [b, h]               int32, DEVICE memory: tokens held per (sequence, head) pair.
 * Rows 0..len-1 of a pair are valid, in the order in which they were evicted.
 */
typedef struct {
    void *k;
    void *v;
    float *score;
    int32_t *pos;
    int32_t *len;
    int32_t host_cap;
} swa_host_store;

/*
 * Stores what a decode step evicted.  Call between swa_decode_step (two-call form: the cache still
 * holds every row) and swa_compact_kv: for every pair, the slots of [0, cache_len) that are not in
 * kept_idx[0 .. kept_cnt) are appended to the pair's host store in ascending slot order (rows of K,
 * V, score, pos; bit-exact copies) and store->len grows by their number.  Device memory is only read.
 * A pair whose store has no room is skipped as a whole (nothing written) and the
 * SWA_ERR_HOST_STORE_FULL status bit is set.  params->len_bound, if set, must bound cache_len.
 * The copies cross the host link: the call is bound by it, not by HBM.
 */
int swa_offload_evicted(const swa_params *params, const void *k_cache, const void *v_cache,
                        const float *score, const int32_t *pos, const int32_t *kept_idx,
                        const int32_t *kept_cnt, const int32_t *cache_len,
                        const swa_host_store *store, void *workspace, void *stream);

/*
 * Loads tokens back: for every pair, rows req_idx[s, hd, 0 .. req_cnt[s]) of its host store (indices
 * into the store, 0 <= index < store->len) are appended to the cache at slots cache_len[s] ..., with
 * their importance and position; new_len[s] = cache_len[s] + req_cnt[s] (cache_len is only read:
 * pass new_len as cache_len to the next call).  The tokens stay in the store as well.  The cache is
 * then no longer in token order: continue with the SWA_UNORDERED forms, whose window and tie rules
 * go by token position.  A sequence without room is skipped (new_len = cache_len, capacity status
 * bit); an index outside the store sets the SWA_ERR_BAD_REQUEST status bit (row 0 stands in).
 *   req_idx [b, h, max_req] int32, req_cnt [b] int32 (device), 0 <= req_cnt <= max_req.
 */
int swa_reload_tokens(const swa_params *params, const swa_host_store *store, const int32_t *req_idx,
                      const int32_t *req_cnt, int32_t max_req, void *k_cache, void *v_cache,
                      float *score, int32_t *pos, const int32_t *cache_len, int32_t *new_len,
                      void *workspace, void *stream);

/*
 * Measurement aid, not part of the method: reads `bytes` (rounded down to a multiple of 104 KiB)
 * from src with plain streaming 128-bit loads and discards them.  Timing it on a buffer much larger
 * than the caches gives the streaming-read ceiling of the machine, the practical denominator next
 * to the nominal HBM peak.  src: device pointer, 16-byte aligned; sink: 4 bytes of device memory.
 */
int swa_probe_stream_read(const void *src, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SWA_H_ */
