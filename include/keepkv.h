/*
 * keepkv.h -- C ABI of the KeepKV hot path for AMD MI355X (gfx950).
 *
 * KeepKV (arXiv 2504.09936) keeps a compressed per-layer KV cache in which every slot i
 * carries an integer Electoral Votes count p_i (Sec. 3.3.1).  Decoding attends with the
 * vote-weighted softmax of Eq. 6; every `period` steps the cache is compressed back to
 * `budget` slots by scoring (Eq. 8), selecting, matching (Alg. 1, matching step) and ZIP-Merging
 * (Eq. 7 / App. A.3).  This library exposes exactly those steps.
 *
 * Conventions common to all calls
 *  - Every pointer marked DEVICE is GPU memory of the current HIP device; the library
 *    allocates nothing and owns nothing.  Pointers must be 16-byte aligned.
 *  - One cache holds one layer: for every (batch b, kv head h) `capacity` slots of which
 *    the first len[b,h] are live.  Tensors are dense row-major in the order written.
 *  - Calls enqueue work on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *    and return without waiting.  Calls on one stream execute in order.
 *  - Arguments are validated on the host before anything is enqueued; on a non-OK status
 *    nothing was launched and no output was touched.  KEEPKV_ERR_DEVICE reports a failed
 *    launch (hipGetLastError).  No exception crosses this boundary; there is no global state
 *    and no environment variable is read.
 *  - Storage dtype of Q, K, V, O is f32 or bf16; all accumulation is f32 (f64 where an
 *    integer decision or a merge weight depends on it).
 *  - Scores are natural logarithms: log_s holds ln S_i of Eq. 8 (uncorrected EMA of the
 *    unnormalised score s_i = exp(q.k_i/sqrt(d)) of Eq. 3), -inf while the slot has no observation.
 *    The bias-corrected score is ln s_hat_i = log_s_i - ln(1 - alpha^n_i), n_i the slot's
 *    observation count (keepkv_cache.born / t_obs).
 */
#ifndef KEEPKV_H
#define KEEPKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KEEPKV_OK = 0,
  KEEPKV_ERR_INVALID_ARG = 1,  /* null pointer, bad shape, bad parameter            */
  KEEPKV_ERR_UNSUPPORTED = 2,  /* head_dim / group size / budget / batch * heads outside the built set */
  KEEPKV_ERR_WORKSPACE = 3,    /* workspace missing or smaller than required         */
  KEEPKV_ERR_DEVICE = 4        /* HIP reported a launch error                        */
} keepkv_status;

typedef enum { KEEPKV_F32 = 0, KEEPKV_BF16 = 1 } keepkv_dtype;

/* Shape of one layer's attention; plain value struct, caller-owned (HOST memory). */
typedef struct {
  int32_t batch;        /* B  >= 1; B * Hkv <= 16384                                   */
  int32_t n_q_heads;    /* Hq, multiple of n_kv_heads; group G = Hq/Hkv in {1,2,4,8}    */
  int32_t n_kv_heads;   /* Hkv >= 1                                                   */
  int32_t head_dim;     /* D in {64, 128}                                             */
  int32_t dtype;        /* keepkv_dtype: storage of Q, K, V, O                        */
  float   scale;        /* logit scale 1/sqrt(head_dim) (Eq. 3)                       */
} keepkv_layout;

/* One layer's cache (HOST struct of DEVICE pointers, caller-owned). */
typedef struct {
  void    *k, *v;       /* [B, Hkv, capacity, D] storage dtype                        */
  int32_t *votes;       /* [B, Hkv, capacity]  p_i >= 1 on live slots (Sec. 3.3.1)     */
  float   *log_s;       /* [B, Hkv, capacity]  ln S_i (Eq. 8), -inf if never observed  */
  int32_t *born;        /* [B, Hkv, capacity]  origin of the slot's score history: the  */
                        /* number of observations folded into S_i (the count of Eq. 8's  */
                        /* bias correction) is n_i = t_obs[b,h] - born[b,h,i]            */
  int32_t *t_obs;       /* [B, Hkv]            observation steps this head has seen: +1  */
                        /* per keepkv_score / keepkv_decode_step, +window per             */
                        /* keepkv_score_window.  Every live slot is observed at every     */
                        /* step, so a step advances all counts through this one word and  */
                        /* the per-slot array is written only when a slot is created,     */
                        /* merged, or seen by part of a causal window                     */
  int32_t *len;         /* [B, Hkv]            live slots, 0 <= len <= capacity        */
  int32_t  capacity;    /* slots allocated per (b, h); 1 <= capacity <= 2^20           */
  int32_t  len_hint;    /* optional: an upper bound on every len[b,h] known to the host */
                        /* (0 = unknown).  With a hint the decode kernels start fetching */
                        /* rows without waiting for len; slots in [len, len_hint) may    */
                        /* then be read but never influence a result.  A hint below some */
                        /* len gives undefined (memory-safe) results.                    */
  int32_t  plan_slots_per_split; /* optional launch override for the decode calls (0 = the cost   */
                        /* model of keepkv_decode_plan decides): slots per split, rounded down to */
                        /* a multiple of 32 (bf16 matrix-core kernel) or 64, at least 64.         */
  int32_t  plan_wavefronts;      /* optional (0 = automatic): 4 or 8 wavefronts per workgroup of   */
                        /* the bf16 matrix-core kernel; -1 runs a bf16 cache on the vector-ALU    */
                        /* kernel of the f32 path.  Overrides change the launch shape only (the   */
                        /* summation order of Eq. 6 across splits), never the meaning; with one   */
                        /* the workspace must hold 64 KiB + 256 + B*Hq*n_split*(D+2)*4 bytes,     */
                        /* n_split = ceil(capacity / slots per split) <= 1024.                    */
} keepkv_cache;

/* Human-readable name of a status (static string). */
const char *keepkv_strerror(keepkv_status st);

/* Library version as an integer (major*10000 + minor*100 + patch). */
int32_t keepkv_version(void);

/* Bytes of DEVICE workspace sufficient for any call below on a cache of `capacity` slots
 * compressed to `budget` slots (pure host function; 0 on invalid arguments).  The
 * workspace is scratch and must not be shared by calls that may run concurrently.  Its
 * head (64 KiB + 256 bytes) holds control words that must be zero when a call starts: clear
 * them once with keepkv_workspace_init after allocating; every call leaves them zero again. */
size_t keepkv_workspace_bytes(const keepkv_layout *layout, int32_t capacity, int32_t budget);

/* How keepkv_decode_attn / keepkv_decode_step will be launched for this layout and capacity (host-side
 * arithmetic, no device call): one workgroup of `wavefronts` wavefronts per (b, h, split), n_split splits of
 * slots_per_split slots per head.  The outputs are HOST pointers and may be NULL.  The plan comes from a cost
 * model of the split-K decode (Eq. 6 evaluated per split and combined); it does not change results beyond
 * the summation order of the splits. */
keepkv_status keepkv_decode_plan(const keepkv_layout *layout, int32_t capacity, int32_t *n_split,
                                 int32_t *slots_per_split, int32_t *wavefronts);

/* Clear the control words at the head of a freshly allocated DEVICE workspace (one small
 * kernel on `stream`; no memset, so it may be captured in a HIP graph). */
keepkv_status keepkv_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/* Append one token per (b, h): k_t, v_t [B, Hkv, D] DEVICE are written to slot len[b,h],
 * with votes = 1, log_s = -inf, born = t_obs[b,h] (no observation yet), then len[b,h] += 1 (Sec. 3.1 cache update;
 * votes initialised to 1, Sec. 3.3.1).  A head already at capacity is left unchanged and
 * `overflow` (DEVICE int32, may be NULL) is set to 1. */
keepkv_status keepkv_append(const keepkv_layout *layout, keepkv_cache *cache,
                            const void *k_t, const void *v_t, int32_t *overflow, void *stream);

/* Vote-weighted decode attention (Eq. 6): for every (b, query head h) with kv head
 * h / G, over the live slots i of that kv head,
 *     out[b,h,:] = sum_i p_i s_i v_i / sum_i p_i s_i,   s_i = exp(scale * q[b,h,:] . k_i)
 * i.e. softmax over scale*q.k + ln p.  q, out: [B, Hq, D] DEVICE, storage dtype.
 * logits_out (DEVICE f32 [B, Hkv, capacity], may be NULL): for each live slot the mean over
 * the G query heads of the group of scale*q.k_i = ln s_i of the group-mean query (the
 * score keepkv_score consumes).  lse_out (DEVICE f32 [B, Hq], may be NULL): ln sum_i p_i s_i.
 * An empty cache (len == 0) gives out = 0 and lse = -inf.  Dead slots are never read.
 * Needs workspace (split partial results). */
keepkv_status keepkv_decode_attn(const keepkv_layout *layout, const keepkv_cache *cache,
                                 const void *q, void *out, float *logits_out, float *lse_out,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* One whole decode step of one layer in a single kernel: keepkv_append of (k_t, v_t), then
 * keepkv_decode_attn over the grown cache, then keepkv_score with the logits just computed
 * (the order of App. C.2: the step attends over the cache including its own token, and the
 * EMA of Eq. 8 observes that step).  Arguments as in those three calls; logits_out may be
 * NULL.  A head already at capacity is attended and scored without its new token and
 * `overflow` (DEVICE int32, may be NULL) is set to 1.  Results equal the three separate calls. */
keepkv_status keepkv_decode_step(const keepkv_layout *layout, keepkv_cache *cache, const void *q,
                                 const void *k_t, const void *v_t, void *out, float *logits_out,
                                 float alpha, int32_t *overflow, void *workspace,
                                 size_t workspace_bytes, void *stream);

/* keepkv_decode_step for callers that cannot allocate device memory and hold no workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, meaning and
 * results as keepkv_decode_step, without the workspace: the split partial results and tickets live in a
 * static device array inside the library (64 KiB + 256 bytes of control words + 4 MiB; every GPU the
 * library runs on holds its own copy until the process ends).  Nothing is allocated or freed, by this
 * call or by anything it calls.  A shape whose partial results exceed the array
 * (B * Hq * n_split * (D + 2) * 4 bytes > 4 MiB with n_split > 1, see keepkv_decode_plan) is refused with
 * KEEPKV_ERR_UNSUPPORTED before anything is launched.  All calls on one GPU share that GPU's array: calls
 * that may overlap there (different streams, no dependency) race and must use keepkv_decode_step with
 * workspaces of their own.  The first call on a device looks up the array's address and enqueues one
 * small kernel on `stream` that clears the control words; every call leaves them zero. */
keepkv_status keepkv_decode_step_static(const keepkv_layout *layout, keepkv_cache *cache,
                                        const void *q, const void *k_t, const void *v_t, void *out,
                                        float *logits_out, float alpha, int32_t *overflow,
                                        void *stream);

/* EMA score update (Eq. 8, t > L branch; Alg. 1, score update) on the live slots:
 *     S_i <- alpha S_i + (1 - alpha) exp(logits[i]),  n_i += 1  (t_obs[b,h] += 1)
 * held as log_s_i = ln S_i.  logits: DEVICE f32 [B, Hkv, capacity] as written by
 * keepkv_decode_attn.  0 <= alpha < 1.  Running it w+1 times from the empty state over the
 * prefill cache yields the t = L window sum of Eq. 8. */
keepkv_status keepkv_score(const keepkv_layout *layout, keepkv_cache *cache,
                           const float *logits, float alpha, void *stream);

/* EMA scores from a window of queries in one pass over the keys (Eq. 8, t = L branch: after
 * prefill the scores come from the last w + 1 queries).  q_win: DEVICE [B, Hq, window, D]
 * storage dtype, oldest query first.  With s_{j,i} = exp of the group-mean logit of query j on
 * slot i (as in keepkv_decode_attn), every live slot seen by the last n_i queries of the window
 * gets
 *     S_i <- alpha^{n_i} S_i + sum_{j >= window - n_i} (1 - alpha) alpha^{window-1-j} s_{j,i},
 *     the slot's count += n_i  (t_obs[b,h] += window; born_i += window - n_i where n_i < window)
 * i.e. the result of `window` consecutive keepkv_score calls; on a fresh cache (log_s = -inf,
 * no observation) this is the window sum of Eq. 8.  first_pos < 0: every query sees every live
 * slot (n_i = window).  first_pos >= 0: query j sits at sequence position first_pos + j and
 * sees only slots i <= first_pos + j (causal prefill; first_pos = len - window for the last
 * `window` prompt tokens).  bf16 caches use bf16 MFMA with f32 accumulation.  Requires
 * window * G <= 128 (longer windows: several calls, oldest queries first).  Needs no workspace. */
keepkv_status keepkv_score_window(const keepkv_layout *layout, keepkv_cache *cache,
                                  const void *q_win, int32_t window, float alpha,
                                  int32_t first_pos, void *stream);

/* Token selection (Alg. 1, selection step; fixed-budget policy with sink tokens, a recent
 * window and heavy hitters, App. B.3).  Per (b, h) with len > budget: slots [0, n_sink)
 * and [len - n_recent, len) are kept; of the others the budget - n_sink - n_recent with the
 * largest ln p_i + ln s_hat_i are kept, equal values resolved in favour of the lower
 * index.  keep_idx [B, Hkv, budget] and evict_idx [B, Hkv, capacity - budget] (DEVICE int32)
 * receive the retained / to-be-evicted slot numbers in ascending order; n_evict [B, Hkv]
 * receives len - budget.  With len <= budget nothing is evicted: n_evict = 0 and keep_idx
 * = 0..len-1 followed by -1.  Requires n_sink + n_recent <= budget <= capacity. */
keepkv_status keepkv_select(const keepkv_layout *layout, const keepkv_cache *cache,
                            int32_t budget, int32_t n_sink, int32_t n_recent, float alpha,
                            int32_t *keep_idx, int32_t *evict_idx, int32_t *n_evict,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Token selection under a caller-supplied ranking (the method places no constraint on the
 * selection strategy, Sec. 3.3.2 last paragraph; combination with other eviction methods,
 * Sec. 4.4): exactly keepkv_select with the ranking value of slot i read from rank[b,h,i]
 * (DEVICE f32 [B, Hkv, capacity]; larger = more important, NaN ranks below every number)
 * instead of ln p_i + ln s_hat_i.  A cumulative-attention heavy-hitter policy, for example,
 * passes its accumulated scores.  Of `cache` only len and capacity are used. */
keepkv_status keepkv_select_by_key(const keepkv_layout *layout, const keepkv_cache *cache,
                                   const float *rank, int32_t budget, int32_t n_sink,
                                   int32_t n_recent, int32_t *keep_idx, int32_t *evict_idx,
                                   int32_t *n_evict, void *workspace, size_t workspace_bytes,
                                   void *stream);

/* Merge-candidate matching (Alg. 1, matching step): for every to-be-evicted slot e the
 * retained slot of highest key cosine similarity U[e,c] = k_e.k_c/(|k_e||k_c|), lowest
 * position winning ties; match[b,h,j] (DEVICE int32 [B, Hkv, capacity - budget]) is that
 * position in keep_idx if U > threshold (strict) and -1 otherwise.  sim_out (DEVICE f32,
 * same shape, may be NULL) receives the best similarity.  bf16 caches use bf16 MFMA with
 * f32 accumulation; rows whose decision lies within rounding of a tie or of the threshold
 * are re-evaluated in f64, so indices equal an f64 evaluation.  budget <= 4096. */
keepkv_status keepkv_match(const keepkv_layout *layout, const keepkv_cache *cache,
                           int32_t budget, const int32_t *keep_idx, const int32_t *evict_idx,
                           const int32_t *n_evict, float threshold, int32_t *match,
                           float *sim_out, void *workspace, size_t workspace_bytes, void *stream);

/* Multi-way Zero Inference-Perturbation Merging with EMA scores (Eq. 7 in its App. A.3 /
 * A.4 form; Alg. 1, merging step).  For retained position r with group g = {keep_idx[r]} +
 * {evict_idx[j] : match[j] = r}, w_i = p_i s_hat_i, W = sum w, P = sum p:
 *     v_r = sum w_i v_i / W,   k_r = (sum w_i k_i / W) * ln(W/P) / (sum w_i ln s_hat_i / W),
 *     p_r = P,   ln s_hat_r = ln(W/P),   n_r = max(count of the retained slot, 1);  dst.t_obs = src.t_obs.
 * When |sum w_i ln s_hat_i / W| < 1e-3 the key scale is taken as 1.  Unmatched evicted
 * slots are dropped and their votes added to dropped_votes[b,h] (DEVICE int64, accumulated,
 * may be NULL).  Results are written to dst slots 0..budget-1 in keep_idx order and
 * dst.len = number of retained slots; heads with n_evict == 0 are copied.  src and dst must
 * not overlap; dst.capacity >= budget; budget <= 4096 and src.capacity - budget <= 32768. */
keepkv_status keepkv_merge(const keepkv_layout *layout, const keepkv_cache *src,
                           keepkv_cache *dst, int32_t budget, const int32_t *keep_idx,
                           const int32_t *evict_idx, const int32_t *n_evict,
                           const int32_t *match, float alpha, int64_t *dropped_votes,
                           void *workspace, size_t workspace_bytes, void *stream);

/* The steady-state event without rewriting the cache (Alg. 1, same selection, matching and merging as the
 * calls above; only where the results are stored differs).  The cache is used in place: its live slots are
 * not in age order.  order (DEVICE int32 [B, Hkv, budget], in/out, owned by the caller) lists the slots below
 * `budget` from the oldest token to the newest; the slots from `budget` to len-1 (appended since the last
 * event) follow in slot order.  It starts as 0..budget-1 for a cache that keepkv_merge has just written.
 *
 * keepkv_select_aged is keepkv_select on that age order: the first n_sink and the last n_recent tokens by
 * age are protected, and keep_idx / evict_idx receive SLOT numbers listed from oldest to newest (so that
 * "lowest position wins ties" in keepkv_match and the summation order of the merge are those of a cache kept
 * in age order).  keepkv_match is then called as usual.
 *
 * keepkv_merge_inplace applies the merge of keepkv_merge to the cache itself: a retained slot that absorbs
 * evicted slots is overwritten with the merged token, all other retained slots below `budget` are not touched,
 * the retained tokens at or beyond `budget` are moved into the slots that evicted tokens leave below `budget`
 * (exactly as many), `order` is rewritten accordingly and len = number of retained slots (= budget); decode
 * steps then append behind them as before.  Votes of unmatched evicted slots go to dropped_votes (may be NULL).
 * Heads with n_evict == 0 are left as they are.  capacity - budget <= 256 (KEEPKV_ERR_UNSUPPORTED beyond:
 * use keepkv_merge).  The merged values are bit for bit those keepkv_merge would write. */
keepkv_status keepkv_select_aged(const keepkv_layout *layout, const keepkv_cache *cache,
                                 const int32_t *order, int32_t budget, int32_t n_sink, int32_t n_recent,
                                 float alpha, int32_t *keep_idx, int32_t *evict_idx, int32_t *n_evict,
                                 void *workspace, size_t workspace_bytes, void *stream);
keepkv_status keepkv_merge_inplace(const keepkv_layout *layout, keepkv_cache *cache, int32_t *order,
                                   int32_t budget, const int32_t *keep_idx, const int32_t *evict_idx,
                                   const int32_t *n_evict, const int32_t *match, float alpha,
                                   int64_t *dropped_votes, void *stream);

/* Merge-first prefill policy, first half (Sec. 3.3.2, last sentence; App. B.4 "Prefill's Merge Policy":
 * during prefill, merge by key similarity first and apply the eviction strategy afterwards).  For every
 * live slot i > 0 of every (b, h): the EARLIER slot j < i of highest key cosine similarity
 * U[i,j] = k_i.k_j/(|k_i||k_j|), the lowest j winning ties; near[b,h,i] (DEVICE int32
 * [B, Hkv, capacity]) is that j if U > threshold (strict) and -1 otherwise; near[b,h,0] = -1.  Entries at or
 * beyond len are not written.  sim_out (DEVICE f32, same shape, may be NULL) receives the best similarity
 * (-inf for slot 0).  bf16 caches use bf16 MFMA with f32 accumulation and re-evaluate rows within rounding
 * of a tie or of the threshold in f64, as keepkv_match does, so the indices equal an f64 evaluation. */
keepkv_status keepkv_prefill_match(const keepkv_layout *layout, const keepkv_cache *cache,
                                   float threshold, int32_t *near, float *sim_out, void *workspace,
                                   size_t workspace_bytes, void *stream);

/* Merge-first prefill policy, second half: the links near[] (from keepkv_prefill_match) form a forest; a slot
 * is absorbed by the slot it links to unless that slot is itself absorbed (slots at odd depth of their tree
 * are absorbed by their parent, slots at even depth stay and receive their children), so every group is one
 * receiving slot plus slots whose best earlier key it is.  Each group is merged in one multi-way ZIP merge
 * with the EMA scores (exactly the arithmetic of keepkv_merge: Eq. 7 in its App. A.3 / A.4 form); nothing is
 * dropped.  The receiving slots are written to dst in ascending slot order and dst.len = their number;
 * the usual event (keepkv_select / keepkv_match / keepkv_merge) then brings dst to the budget.  src and dst
 * must not overlap; dst.capacity >= src.capacity; src.capacity <= 32768 (KEEPKV_ERR_UNSUPPORTED beyond; up to
 * 16384 slots per head the grouping works in LDS, above that in the workspace). */
keepkv_status keepkv_prefill_merge(const keepkv_layout *layout, const keepkv_cache *src,
                                   keepkv_cache *dst, const int32_t *near, float alpha,
                                   void *workspace, size_t workspace_bytes, void *stream);

/* Measurement probes (not part of the method): what the GPU sustains, to set next to the
 * published peaks.  keepkv_probe_read: `n_workgroups` workgroups stream `bytes` (a multiple of
 * 16) of DEVICE memory at `src` once with coalesced 16-byte loads; nothing is written except
 * possibly the DEVICE float `sink`.  keepkv_probe_mfma: every wavefront of `n_workgroups`
 * workgroups (4 wavefronts each) issues 4 * iters independent 32x32x16 bf16 MFMAs, on operands
 * that are all (nearly) one, or, with random_operands != 0, pseudo-random bf16 values (the
 * sustained clock and so the rate depend on the data); *flops (HOST, may be NULL) receives the
 * floating-point operations of the launch.  Time them with events. */
keepkv_status keepkv_probe_read(const void *src, size_t bytes, int32_t n_workgroups, float *sink,
                                void *stream);
keepkv_status keepkv_probe_mfma(int32_t n_workgroups, int32_t iters, int32_t random_operands,
                                float *sink, double *flops, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* KEEPKV_H */
