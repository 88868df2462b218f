/*
 * ngc.h -- C ABI of the MI355X (gfx950) eviction + decode-attention library
 * for Neural Garbage Collection (NGC).
 *
 * The library implements the periodic eviction step of the method and the
 * decode attention that follows it:
 *
 *   ngc_perturbed_keys   logits + Gumbel noise                     (Sec. 4.3)
 *   ngc_evict            Gumbel-top-k sample of the entries to keep, their
 *                        ordered-subset log-probability, and in-place removal
 *                        of everything else                  (Sec. 4.1, 4.3, Eq. 2)
 *   ngc_subset_logprob   Eq. 2 for caller-supplied sampled actions (Sec. 4.3-4.4)
 *   ngc_subset_logprob_backward  its gradient w.r.t. the logits (Eq. 4)
 *   ngc_lmem             the eviction loss of Eq. 4 and the weights it puts on
 *                        every round's log-probability             (Sec. 4.4)
 *   ngc_cache_append     one new entry per token between rounds   (Sec. 4.1)
 *   ngc_decode_attn      softmax(q K^T / sqrt(d_h)) V over the surviving
 *                        entries of every sequence               (Sec. 4.1, 4.2)
 *   ngc_decode_step      append + decode attention of a layer in one launch
 *   ngc_decode_attn_static  ngc_decode_attn without a workspace argument
 *   ngc_replay_attn      training-time attention under the replay mask (Sec. 4.5)
 *   ngc_score_keys       attention-based importance of every cached key, the
 *                        input of the eviction policy                (Sec. 4.2)
 *   ngc_paged_*          the same path over a paged cache, where the blocks of
 *                        Sec. 4.2 are pages and eviction edits a page table
 *                        instead of moving rows
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer unless a comment says "host".  The
 *     structs themselves (ngc_cache, ngc_evict_params) live in HOST memory and
 *     are read during the call only.
 *   - The caller owns every buffer.  The library allocates nothing, keeps no
 *     state between calls (the workspace holds, besides the status words, per-
 *     segment tickets that every launch leaves at zero: zero the workspace once
 *     before its first use, again before it serves a cache of another geometry
 *     (its layout follows the geometry), and do not share it between calls that
 *     overlap in time) and never synchronises: each call only enqueues
 *     kernels on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream).  Ragged lengths and keep counts are read on the device.
 *   - Return value: NGC_OK or a negative NGC_E* code; nothing is enqueued when
 *     an error is returned.  Conditions only the device can see (a keep count
 *     above the segment size, a length above the capacity, ...) never trap:
 *     they are clamped and counted in the status words at the start of the
 *     workspace (see NGC_STATUS_*).
 *   - A "segment" is one independent selection problem: one (layer, sequence,
 *     KV head).  Segment id = (layer * B + sequence) * Hkv + head.
 *   - An "item" is what is kept or evicted as a unit: `block` consecutive rows
 *     of a segment (the block of Sec. 4.2; block = 1 is one cache position).
 *     A segment of n rows has ceil(n / block) items, the last possibly short.
 */
#ifndef NGC_H
#define NGC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NGC_OK            0
#define NGC_EINVAL       (-1)  /* null / misaligned pointer, bad shape or parameter        */
#define NGC_ENOSPC       (-2)  /* workspace too small                                      */
#define NGC_EHIP         (-3)  /* a HIP call failed (launch, attribute)                    */
#define NGC_EUNSUPPORTED (-4)  /* valid request outside what the kernels cover (see below) */

/* Status words: int32 counters at the start of the workspace, one per kind of
 * device-detected anomaly.  The caller zeroes the workspace once; kernels only
 * add to them.  NGC_STATUS_WORDS words are reserved; the last two are the
 * library's own (the work counter of the eviction kernel and a count of its
 * finished workgroups: both zero again when a launch has ended). */
#define NGC_STATUS_WORDS        64
#define NGC_STATUS_KEEP_CLAMPED  0  /* keep[seg] > items (or < 0): clamped                  */
#define NGC_STATUS_LEN_CLAMPED   1  /* len[seg] > cap (or < 0): clamped                     */
#define NGC_STATUS_EMPTY_ATTN    2  /* decode attention over an empty segment: zeros        */
#define NGC_STATUS_APPEND_FULL   3  /* append to a full segment: skipped                    */
#define NGC_STATUS_BAD_SIGMA     4  /* ngc_subset_logprob: index out of range or repeated   */
#define NGC_STATUS_POOL_BOUNDS   5  /* paged cache: free stack would overflow, or a page id
                                       in a table is outside the pool: ignored              */

/* Non-owning view of a KV cache in device memory.
 *   k, v : bf16, dense [L][B][Hkv][cap][D], 16-byte aligned.  Rows [0, len) of
 *          a segment are the surviving entries (in ascending order of their
 *          original position unless a round used NGC_EVICT_UNORDERED); rows
 *          >= len are unspecified.
 *   len  : int32 [L][B][Hkv], rows in use per segment (ragged).
 *   pos  : optional int32 [L][B][Hkv][cap], original token index of each row
 *          (moved together with the rows), or NULL.
 *   D    : 64 or 128.  Hq must be a multiple of Hkv with Hq / Hkv <= 16.
 *   cap  : rows allocated per segment.  Any value works; for speed make a
 *          segment (cap * 2 * D bytes) a multiple of 4 KB and the base 4 KB
 *          aligned (cap a multiple of 16 at D = 128): decode attention reads
 *          8 KB at a time from the segment start, and measured 4-6 % slower
 *          when those reads straddle 4 KB boundaries.                        */
typedef struct ngc_cache {
    void    *k;
    void    *v;
    int32_t *len;
    int32_t *pos;
    int32_t  L, B, Hkv, Hq, D, cap;
} ngc_cache;

/* Parameters of one eviction round.
 *   block        rows per item (>= 1).
 *   share_heads  0: every (layer, sequence, head) draws its own noise;
 *                1: the head index is left out of the noise counter, so all
 *                   KV heads of a (layer, sequence) draw the same noise (one
 *                   decision per layer, Sec. 4.2, when their logits agree too).
 *   noise_scale  tau: key = logit + tau * Gumbel.  1 = sampling (Sec. 4.3),
 *                0 = greedy top-k as used at evaluation (Sec. 5.1).
 *   round        eviction round counter; with `seed` it names the draw, the
 *                same (seed, round) reproduces the same sample.
 *   layer_base, seq_base
 *                the noise of an entry is a function of (seed, round, global
 *                layer, global sequence, head, item) -- every layer takes its
 *                own decisions (Sec. 4.4).  A caller that holds one allocation
 *                per layer, or a slice of the batch, passes where its view
 *                starts: layer l / sequence b of the view then draw the noise
 *                of layer layer_base + l / sequence seq_base + b, exactly what
 *                they draw inside one allocation holding everything.
 *                layer_base + L <= 65535.
 *   flags        NGC_EVICT_SELECT_ONLY: sample (and score) but move nothing
 *                and leave `len` untouched.
 *                NGC_EVICT_UNORDERED (block == 1 only): instead of packing the
 *                survivors in ascending order, leave the kept rows below slot
 *                K in place and move the i-th kept row at or beyond slot K
 *                into the i-th freed slot below K (both counted ascending).
 *                Same surviving set, far fewer rows moved; the cache is then
 *                no longer in order of original position (pos still names it).
 *                NGC_EVICT_POOL_HEADS (block == 1, Hkv * cap <= 65536): one
 *                selection per (layer, sequence) over the rows of all its KV
 *                heads; the budget is the sum of the heads' keep entries and
 *                every head keeps however many of its rows make the pooled
 *                top-K (item order for ties and for sigma: head, then row; the
 *                noise of a row is the one the per-head mode draws for it).
 *                kept_out then holds each head's own kept rows (ascending;
 *                max_keep must cover the largest share), len the per-head
 *                counts; sigma_out holds the pooled sequence, coded as
 *                head * cap + row, in the Hkv rows of the (layer, sequence)
 *                back to back; logp_out holds its log-probability in the entry
 *                of head 0 and 0 in the others.  The workspace must be
 *                ngc_workspace_bytes() + 16 * L * B * Hkv * cap bytes.  The
 *                budget of one (layer, sequence) -- a sum only the device
 *                sees -- is limited to 32000 items (the sort's index buffers
 *                live in LDS); a larger one is clamped to the limit and
 *                counted in NGC_STATUS_KEEP_CLAMPED. */
#define NGC_EVICT_SELECT_ONLY 1u
#define NGC_EVICT_UNORDERED   2u
#define NGC_EVICT_POOL_HEADS  4u
typedef struct ngc_evict_params {
    int32_t  block;
    int32_t  share_heads;
    float    noise_scale;
    uint32_t round;
    uint64_t seed;
    uint32_t flags;
    int32_t  layer_base;   /* global index of the cache view's layer 0 ...                 */
    int32_t  seq_base;     /* ... and of its sequence 0 (both 0 for a whole cache)         */
    int32_t  reserved;     /* 0 */
} ngc_evict_params;

/* Library version (major * 10000 + minor * 100 + patch). */
int ngc_version(void);

/* Static, NUL-terminated description of a return code (host memory). */
const char *ngc_strerror(int code);

/* Bytes of workspace that make every call below succeed for this cache
 * geometry and up to `max_keep` kept items per segment.  Host computation. */
size_t ngc_workspace_bytes(const ngc_cache *c, int32_t max_keep);

/* Perturbed keys (Sec. 4.3): for every segment of `layer` (-1 = all layers)
 * and every item t < ceil(len / block):
 *     keys[seg][t] = fl32( (double)logits[seg][t] + (double)tau * g ),
 *     g = -log(-log u),  u = (r + 1/2) 2^-32,
 *     r = word (t mod 4) of Philox-4x32-10 with key = seed and counter
 *         (t / 4, sequence, layer * 65536 + head selector, round);
 * tau == 0 copies the logits.  logits, keys_out: fp32 [L][B][Hkv][cap], item t
 * of a segment at offset t of its row; entries past the item count are left
 * untouched.  ws needs NGC_STATUS_WORDS * 4 bytes (status only). */
int ngc_perturbed_keys(const ngc_cache *c, int32_t layer, const float *logits,
                       const ngc_evict_params *p, float *keys_out,
                       void *ws, size_t ws_bytes, void *stream);

/* Keep counts from a retention rate, computed where the lengths live (Sec. 4.1:
 * every round keeps the fraction 1 - eps = num / den of what is cached): for
 * segments seg0 .. seg0 + nseg - 1
 *     N = ceil(min(max(len, 0), cap) / block),
 *     keep_out[seg] = min(N, max(1, min_keep, ceil(N * num / den)))   (0 when N == 0)
 * in exact integer arithmetic.  len, keep_out: int32, indexed by segment (for a
 * paged cache pass cap = max_pages * page_rows and block = page_rows).
 * 0 <= num <= den, den >= 1. */
int ngc_keep_counts(const int32_t *len, int32_t seg0, int32_t nseg, int32_t cap, int32_t block,
                    int32_t num, int32_t den, int32_t min_keep, int32_t *keep_out, void *stream);

/* One eviction round (Sec. 4.1, 4.3) for every segment of `layer` (-1 = all).
 *   logits    fp32 [L][B][Hkv][cap]; item t of a segment at offset t of its
 *             row.  NaN is treated as -inf.
 *   keep      int32 [L][B][Hkv]: items to keep per segment (K).  Values above
 *             the item count are clamped (a no-op round), below 0 to 0.
 *   max_keep  row length of kept_out / sigma_out (>= every K that is used).
 *   kept_out  int32 [L][B][Hkv][max_keep]: kept item indices, ascending.
 *   sigma_out int32 [L][B][Hkv][max_keep] or NULL: kept item indices in
 *             sampled order, i.e. by descending perturbed key, equal keys by
 *             ascending index (the sequence sigma of Eq. 2).
 *   logp_out  fp32 [L][B][Hkv] or NULL: log-probability of sigma (Eq. 2).
 * Entries past K of a row of kept_out / sigma_out are unspecified.  Unless
 * NGC_EVICT_SELECT_ONLY is set, the rows of the kept items are then packed to
 * the front of their segment in k, v and pos, in ascending order, in place,
 * and len is updated.  Segments of other layers are not touched.
 * Limits (NGC_EUNSUPPORTED beyond): items = ceil(cap / block) <= 16384 per
 * segment, items + min(max_keep, items) <= 32704 (what fits in LDS: 16384 items
 * go with max_keep <= 16320), cap * D * 2 < 2^31 bytes per segment.  A keep
 * count above max_keep is clamped to it and counted like one above the item
 * count.  ws must hold ngc_workspace_bytes(). */
int ngc_evict(const ngc_cache *c, int32_t layer, const float *logits,
              const int32_t *keep, const ngc_evict_params *p, int32_t max_keep,
              int32_t *kept_out, int32_t *sigma_out, float *logp_out,
              void *ws, size_t ws_bytes, void *stream);

/* Eq. 2 for given actions: for each of nseg independent segments
 *     logp[s] = sum_j ( x[sigma_j] - log sum_{t not in sigma_1..sigma_{j-1}} exp x[t] )
 * over the first n_items[s] logits of row s.
 *   logits   fp32 [nseg][logit_stride]
 *   n_items  int32 [nseg]         items per segment (<= 65536 each)
 *   sigma    int32 [nseg][sigma_stride], first keep[s] entries used, distinct
 *   keep     int32 [nseg]
 *   logp_out fp32 [nseg]
 * fp32 arithmetic, 1e-4 relative.  The logits may span any range: where the
 * finite logits of a segment lie more than 80 apart (exp(x - max x) of the
 * smallest would underflow) every running sum carries its own exponent, so a
 * sequence that reaches those entries after everything larger has been picked
 * still gets its finite log-probability; -inf entries are masked entries (a
 * sequence that picks one has log-probability -inf), NaN counts as -inf.  The
 * same holds for the log-probability ngc_evict returns.
 * ws needs NGC_STATUS_WORDS * 4 bytes (status only). */
int ngc_subset_logprob(const float *logits, const int32_t *n_items,
                       const int32_t *sigma, const int32_t *keep, int32_t nseg,
                       int64_t logit_stride, int32_t sigma_stride,
                       float *logp_out, void *ws, size_t ws_bytes, void *stream);

/* Gradient of Eq. 2 with respect to the logits, as the eviction policy
 * gradient of Eq. 4 needs it: for each segment s and item t < n_items[s]
 *     grad[s][t] = gout[s] * d log p(sigma_s | x_s) / d x_s[t]
 *                = gout[s] * ( 1[t in sigma_s] - sum_{j : t not in sigma_1..sigma_{j-1}}
 *                                                 exp x[t] / sum_{u not in sigma_1..sigma_{j-1}} exp x[u] ).
 *   gout      fp32 [nseg] upstream weights (for Eq. 4: minus the advantage over
 *             the number of rollouts and rounds), or NULL for 1
 *   grad_out  fp32 [nseg][logit_stride]; entries past n_items are untouched
 *   max_keep  upper bound on keep[s] (<= 32768)
 * Accuracy: 1e-4 of an entry plus ~1e-6 * gout; where the finite logits of a
 * segment lie more than 80 apart the absolute error grows with that span (about
 * 1e-6 * span * gout: the ratios are exponentials of differences of numbers
 * of that size), so entries are meaningful up to spans of a few thousand.  Not
 * defined for a sequence that picks a masked (-inf) entry.
 * Other arguments as in ngc_subset_logprob. */
int ngc_subset_logprob_backward(const float *logits, const int32_t *n_items,
                                const int32_t *sigma, const int32_t *keep, int32_t nseg,
                                int64_t logit_stride, int32_t sigma_stride, int32_t max_keep,
                                const float *gout, float *grad_out,
                                void *ws, size_t ws_bytes, void *stream);

/* The eviction loss of Eq. 4 and its derivative with respect to every
 * log-probability that enters it:
 *     A_i   = reward[i] - mean of reward over the `group` rollouts of i's prompt
 *             (rollouts of a prompt are consecutive; B is a multiple of group),
 *     L^l   = -(1/B) sum_i A_i (1/n_i) sum_{t < n_i} sum_h logp[t][l][i][h],   n_i = rounds[i]
 *             (mean over a rollout's rounds, over the rollouts of a prompt and
 *             over the prompts of the batch; a layer's decision is the joint one
 *             of its KV heads, whose log-probabilities add; n_i == 0 adds nothing),
 *     loss  = sum_l L^l,
 *     gout[t][l][i][h] = d loss / d logp[t][l][i][h] = -A_i / (B n_i)  for t < n_i, else 0
 *             -- round t's slice gout[t] is what ngc_subset_logprob_backward takes.
 *   logp        fp32 [R][L][B][Hkv]  log-probabilities as ngc_evict wrote them, round by round
 *   rounds      int32 [B], clamped to [0, R]
 *   reward      fp32 [B]
 *   adv_out     fp32 [B] or NULL;  loss_layer fp32 [L];  loss fp32 [1];  gout as logp, or NULL
 * Accumulation is fp64 in a fixed order (same inputs, same bits).  B <= 8192. */
int ngc_lmem(const float *logp, const int32_t *rounds, const float *reward,
             int32_t R, int32_t L, int32_t B, int32_t Hkv, int32_t group,
             float *adv_out, float *loss_layer, float *loss, float *gout, void *stream);

/* Append one new row per (sequence, head) of `layer` (-1 = all layers) at row
 * len and add 1 to len (Sec. 4.1: between rounds every new token adds its entry).
 *   k_new, v_new  bf16 [B][Hkv][D]  (or [L][B][Hkv][D] for layer = -1)
 *   new_pos       int32 [B] token index stored into pos, or NULL
 * A full segment (len == cap) is skipped and counted. */
int ngc_cache_append(const ngc_cache *c, int32_t layer, const void *k_new,
                     const void *v_new, const int32_t *new_pos,
                     void *ws, size_t ws_bytes, void *stream);

/* Decode attention over the surviving entries (Sec. 4.1; scale of Sec. 4.2):
 * for every sequence b and query head i of `layer` (-1 = all layers), with
 * h = i / (Hq / Hkv) and n = len[layer][b][h],
 *     out[b][i][:] = sum_{j<n} softmax_j( scale * <q[b][i], K[h][j]> ) V[h][j][:]
 *   q    bf16 [B][Hq][D]   (or [L][B][Hq][D] for layer = -1), 16-byte aligned
 *   out  fp32 same shape
 *   scale          usually 1 / sqrt(D)
 *   max_len_hint   an upper bound on len the caller knows (0 = use cap); it
 *                  only steers how the work is split, never the result.
 *   lse_out        optional fp32 [B][Hq] (or [L][B][Hq]): log sum_j exp(scale *
 *                  <q, K[j]>) per query head (natural log; -inf for n == 0), or
 *                  NULL.  ngc_score_keys can reuse it.
 * n == 0 gives zeros (and is counted).  Scores, softmax and accumulation are
 * fp32.  ws must hold ngc_workspace_bytes(). */
int ngc_decode_attn(const ngc_cache *c, int32_t layer, const void *q, float scale,
                    int32_t max_len_hint, float *out, float *lse_out,
                    void *ws, size_t ws_bytes, void *stream);

/* One decode step of a layer in one launch (Sec. 4.1: between rounds every new
 * token adds its entry to the cache, and the token attends to the surviving
 * entries, its own included): exactly ngc_cache_append(c, layer, k_new, v_new,
 * new_pos) followed by ngc_decode_attn(c, layer, q, ...), same results, same
 * status counts (a full segment is not appended to, is counted, and is
 * attended to as it is).  max_len_hint bounds the lengths after the append.
 *   k_new, v_new  bf16 [B][Hkv][D]  (or [L][B][Hkv][D] for layer = -1), 16-byte aligned
 *   new_pos       int32 [B] or NULL
 * Other arguments as in ngc_decode_attn. */
int ngc_decode_step(const ngc_cache *c, int32_t layer, const void *k_new, const void *v_new,
                    const int32_t *new_pos, const void *q, float scale, int32_t max_len_hint,
                    float *out, float *lse_out, void *ws, size_t ws_bytes, void *stream);

/* ngc_decode_attn for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same computation, same kernels and same results as
 * ngc_decode_attn; the split partials live in a fixed array of
 * NGC_STATIC_SCRATCH_BYTES inside the library's device image (one copy per GPU,
 * held until the process ends) instead of a workspace.
 *   status   optional int32 [NGC_STATUS_WORDS] device buffer of the caller for
 *            the anomaly counters (zeroed by the caller, only added to), or
 *            NULL to drop them.
 * Returns NGC_ENOSPC, and enqueues nothing, when the call would need more than
 * the fixed array: 4096 bytes of status words and tickets plus
 *     S * nseg * (Hq / Hkv) * (D + 2) * 4 bytes (plus alignment) of partials,
 *     nseg = segments of the launch, S = workgroups per segment as
 *     ngc_decode_attn chooses them (1 for more than 128 segments, else at most
 *     min(256 / nseg, 64)) -- i.e. only 16 query heads per KV head at D = 128
 *     over 240 or more workgroups exceed it; ngc_decode_attn with a workspace
 *     takes those.
 * The layout inside the array does not depend on the cache's geometry, so caches
 * of different shapes can be served one after the other.
 * The call itself allocates nothing and calls no allocating routine; the first
 * call on a device looks up the array's address (make that call outside graph
 * capture).  All calls on one GPU share the array: calls that overlap in time
 * on the same GPU (different streams) race on the partials and must be
 * serialised by the caller.  Nothing in the array has to be cleared by anyone:
 * every partial a launch reads was written by that launch, and the per-segment
 * tickets (zero when the image is loaded) are back at zero when a launch ends. */
#define NGC_STATIC_SCRATCH_BYTES ((size_t)2 << 20)
int ngc_decode_attn_static(const ngc_cache *c, int32_t layer, const void *q, float scale,
                           int32_t max_len_hint, float *out, float *lse_out,
                           int32_t *status, void *stream);

/* Key importance scores for the eviction policy (Sec. 4.2): for every segment
 * of `layer` (-1 = all layers), with the queries of the w most recent tokens
 * (whose keys are the last w rows of the segment),
 *     A_{q,t}  = softmax_t( scale * <q, K[t]> )   over the rows query q can see,
 *     psi_t    = mean of A_{q,t} over the w queries and the Hq/Hkv query heads
 *                of the KV head,
 * where recent query j (0 = oldest) sees rows t <= len - w + j (its own token
 * and everything before it); NGC_SCORE_NO_CAUSAL lets every query see all rows.
 * With block > 1 the value of item j is the mean of psi over its rows (last
 * block possibly short); with NGC_SCORE_POOL_HEADS it is further averaged over
 * the KV heads of the (layer, sequence) -- the paper's one score per layer and
 * block -- and written to every head.
 *   q_recent    bf16 [B][w][Hq][D] (or [L][B][w][Hq][D] for layer = -1), 16-byte aligned
 *   lse_recent  optional fp32 [B][w][Hq] (or [L][B][w][Hq]): the log-sum-exp of
 *               each recent query over the rows it can see, as ngc_decode_attn
 *               returned it when that token was decoded (causal reading only).
 *               With it the keys are read once instead of twice.  NULL = compute.
 *   scores_out  fp32 [L][B][Hkv][cap], item j of a segment at offset j: the
 *               layout ngc_evict takes as logits.  Entries past the item count
 *               are unspecified.
 * Limit: w * (Hq/Hkv) <= 64 (NGC_EUNSUPPORTED beyond).
 * ws needs NGC_STATUS_WORDS * 4 bytes (status only). */
#define NGC_SCORE_NO_CAUSAL  1u
#define NGC_SCORE_POOL_HEADS 2u
int ngc_score_keys(const ngc_cache *c, int32_t layer, const void *q_recent,
                   const float *lse_recent, int32_t w,
                   float scale, uint32_t flags, int32_t block, float *scores_out,
                   void *ws, size_t ws_bytes, void *stream);

/* Replay attention for the training forward pass (Sec. 4.5, Appendix A.3): one
 * layer, every position of every trajectory at once, each query seeing exactly
 * the keys that were in the cache when its token was generated:
 *     out[b][i][h][:] = sum_j softmax_j( scale * <q[b][i][h], k[b][j][h/G]> ) v[b][j][h/G][:]
 *     over the j with  j <= i < death[b][.][j],
 * where death[..][j] is the first query position that no longer sees key j (the
 * position at which the round that evicted it fired; >= T if it was never
 * evicted).  This replaces the dense B x T x T boolean mask of the paper by one
 * int per key.
 *   q      bf16 [B][T][Hq][D], 16-byte aligned
 *   k, v   bf16 [B][T][Hkv][D]
 *   death  int32 [B][Hkv][T] if death_per_head != 0, else [B][T] (one set of
 *          decisions per layer, shared by its KV heads)
 *   out    fp32 [B][T][Hq][D]
 *   scale  positive and finite (NGC_EINVAL otherwise)
 * D is 64 or 128; T <= 65535 and T * Hkv * D * 2 < 2^32 (NGC_EUNSUPPORTED
 * beyond).  ws must hold ngc_replay_workspace_bytes(B, T, Hkv). */
size_t ngc_replay_workspace_bytes(int32_t B, int32_t T, int32_t Hkv);
int ngc_replay_attn(const void *q, const void *k, const void *v, const int32_t *death,
                    int32_t B, int32_t T, int32_t Hq, int32_t Hkv, int32_t D,
                    int32_t death_per_head, float scale, float *out,
                    void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------
 * Paged layout.  Sec. 4.2 evicts whole blocks of consecutive tokens and notes
 * that such blocks suit paged caches; here a block IS a page: eviction permutes
 * a segment's page table and hands the evicted pages back to a pool shared by
 * all segments, and no K/V row moves.
 *
 *   k_pool, v_pool  bf16 [num_pages][page_rows][D], 16-byte aligned
 *   pos_pool        optional int32 [num_pages][page_rows], or NULL
 *   table           int32 [L][B][Hkv][max_pages]: physical page of every logical
 *                   page of a segment.  Entries [0, ceil(len / page_rows)) are in
 *                   use; row r of a segment is row r % page_rows of page
 *                   table[r / page_rows].  Other entries are unspecified.
 *   len             int32 [L][B][Hkv] rows in use; only the last page in use
 *                   may be partly filled.
 *   free_stack      int32 [num_pages]: entries [0, *free_count) are the pages no
 *                   segment owns.  The caller initialises it (all pages, in any
 *                   order) together with free_count.
 *   page_rows       power of two, >= 32.  max_pages <= 16384.
 * Every page id is in exactly one place: one table (among the entries in use)
 * or the free stack.  The order of pool operations is fixed, so that the same
 * calls always produce the same tables:
 *   release (ngc_paged_evict)  segments in ascending id, the evicted pages of a
 *           segment in ascending logical index, each pushed on top of the stack;
 *   grant   (ngc_paged_append) the segments that need a page, in ascending id,
 *           take pages from the top of the stack downwards.                    */
typedef struct ngc_paged_cache {
    void    *k_pool;
    void    *v_pool;
    int32_t *pos_pool;
    int32_t *table;
    int32_t *len;
    int32_t *free_stack;
    int32_t *free_count;
    int32_t  L, B, Hkv, Hq, D, page_rows, max_pages, num_pages;
} ngc_paged_cache;

/* Bytes of workspace that make every ngc_paged_* call succeed. */
size_t ngc_paged_workspace_bytes(const ngc_paged_cache *pc);

/* One eviction round over pages (Sec. 4.1-4.3 with block = page_rows): the
 * items of a segment are its ceil(len / page_rows) logical pages.  Sampling,
 * kept_out, sigma_out, logp_out, keep, max_keep and the clamping rules are those
 * of ngc_evict (p->block must equal page_rows; of p->flags only
 * NGC_EVICT_SELECT_ONLY is allowed).
 *   logits        fp32, item j of segment s at logits[s * logit_stride + j]
 *                 (logit_stride >= max_pages; ngc_paged_score_keys writes with
 *                 stride max_pages * page_rows)
 * Unless NGC_EVICT_SELECT_ONLY: the table of every segment becomes
 *     [ old[kept_0], .., old[kept_{K-1}], evicted entries ascending, rest as before ],
 * len becomes page_rows * (K - 1) + rows of the last kept page (short only when
 * that is the segment's last page), and the evicted pages are released (order
 * above).  No K/V byte is read or written. */
int ngc_paged_evict(const ngc_paged_cache *pc, int32_t layer, const float *logits,
                    int64_t logit_stride, const int32_t *keep, const ngc_evict_params *p,
                    int32_t max_keep, int32_t *kept_out, int32_t *sigma_out, float *logp_out,
                    void *ws, size_t ws_bytes, void *stream);

/* Append one row per (sequence, head) of `layer` (-1 = all layers), arguments as
 * in ngc_cache_append.  A segment whose len is a multiple of page_rows first
 * gets a page (order above; table entry -1 when the pool is empty).  A segment
 * at capacity (max_pages * page_rows rows) or without a page is skipped and
 * counted in NGC_STATUS_APPEND_FULL. */
int ngc_paged_append(const ngc_paged_cache *pc, int32_t layer, const void *k_new,
                     const void *v_new, const int32_t *new_pos,
                     void *ws, size_t ws_bytes, void *stream);

/* ngc_decode_attn over the paged layout: same arguments, same result as for a
 * contiguous cache holding the same logical rows. */
int ngc_paged_decode_attn(const ngc_paged_cache *pc, int32_t layer, const void *q, float scale,
                          int32_t max_len_hint, float *out, float *lse_out,
                          void *ws, size_t ws_bytes, void *stream);

/* ngc_score_keys over the paged layout.  scores_out: fp32
 * [L][B][Hkv][max_pages * page_rows]; with block == page_rows entry j of a
 * segment is the score of its logical page j (pass logit_stride = max_pages *
 * page_rows to ngc_paged_evict); block == 1 gives one score per row. */
int ngc_paged_score_keys(const ngc_paged_cache *pc, int32_t layer, const void *q_recent,
                         const float *lse_recent, int32_t w,
                         float scale, uint32_t flags, int32_t block, float *scores_out,
                         void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NGC_H */
