/*
 * ngc_oracle.c -- CPU oracle for the Neural Garbage Collection eviction step
 * and decode attention over the evicted caches.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded
 * statement of what the hot path computes, written from the paper.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it;
 * the product library never does and shares no code with it.
 *
 * Every function takes one *segment* (one independent top-K problem: one
 * layer, one sequence, one KV head) and works in fp64 unless the paper or the
 * exact-reproducibility requirement fixes something else.
 *
 * What each function follows:
 *   orc_philox4x32_10   the published Philox-4x32 generator with 10 rounds
 *                       (Salmon et al., SC'11); the paper (Sec. 4.3) only asks
 *                       for i.i.d. Gumbel noise, the counter generator is this
 *                       build's reading.
 *   orc_log             the logarithm *as defined for the noise*: a fixed
 *                       sequence of IEEE-754 double operations, so that a
 *                       second implementation reproduces every bit.
 *   orc_gumbel_u32      g = -log(-log u), u = (r + 1/2) 2^-32   (Sec. 4.3)
 *   orc_perturbed_keys  key_t = fl32(s_t + tau * g_t)           (Sec. 4.3;
 *                       tau = 0 is the greedy evaluation rule of Sec. 5.1)
 *   orc_select          keep the K largest perturbed values     (Sec. 4.3)
 *   orc_logprob_literal Eq. 2 evaluated term by term, K logsumexps
 *   orc_logprob_suffix  the same value by one reverse running sum (the
 *                       running-sum shortcut the paper mentions after
 *                       Eq. 2, in the cancellation-free arrangement)
 *   orc_logprob_grad_literal  d(Eq. 2)/d(logits), term by term (Eq. 4 needs it)
 *   orc_compact         permanent removal of evicted entries    (Sec. 4.1,
 *                       Eq. 7: next alive set = kept entries + new tokens)
 *   orc_decode_attn     softmax(q K^T / sqrt(d_h)) V over the surviving rows
 *                       (Sec. 4.2 for the scale, Sec. 4.1 for "conditioned on
 *                       the surviving entries")
 *   orc_replay_attn     attention of a whole trajectory under the replay mask:
 *                       query i sees key j iff j <= i and j had not been evicted
 *                       when token i was generated (Sec. 4.5, Appendix A.3)
 *   orc_score_keys      importance of every cached key: attention weights of
 *                       the w most recent queries, averaged over heads and
 *                       queries (Sec. 4.2, "Parameterizing eviction actions")
 *   orc_block_means     block-level scores: mean of the key scores over each
 *                       block of b contiguous keys (Sec. 4.2, "Coarsening")
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py
 * against published test vectors, closed forms, brute force or a library
 * routine.  Nothing is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ RNG -- */

/* One Philox-4x32 round: two 32x32->64 multiplies, the high halves are mixed
 * with the other counter words and the round key, the low halves pass. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                       uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)M0 * c0;
        uint64_t p1 = (uint64_t)M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The random word of item t of a segment.
 *   key     = (low, high) halves of the 64-bit seed
 *   counter = (t / 4, sequence b, layer l * 65536 + head selector, round)
 *   word    = output t mod 4
 * The head selector is the KV head index, or 0xFFFF when every head of a
 * layer shares one draw. */
uint32_t orc_item_word(uint64_t seed, uint32_t round, uint32_t l, uint32_t b,
                       uint32_t hsel, uint32_t t)
{
    uint32_t ctr[4] = { t >> 2, b, (l << 16) | (hsel & 0xFFFFu), round };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[t & 3u];
}

/* ------------------------------------------------------- defined log ---- */

/* log(x) for positive normal doubles, as a fixed operation sequence:
 *   x = 2^e * m, m in [1,2); if m > sqrt(2): m <- m/2, e <- e+1
 *   f = m - 1;  s = f / (2 + f);  z = s*s
 *   log m = 2s + s z (2/3 + 2/5 z + ... + 2/19 z^8)   (atanh series, Horner, fma)
 *   log x = fma(e, ln2, log m)
 * Every step is one correctly rounded IEEE operation. */
double orc_log(double x)
{
    uint64_t bits;
    memcpy(&bits, &x, 8);
    int e = (int)((bits >> 52) & 0x7FFu) - 1023;
    uint64_t mb = (bits & 0x000FFFFFFFFFFFFFull) | 0x3FF0000000000000ull;
    double m;
    memcpy(&m, &mb, 8);
    if (m > 1.4142135623730951) { m = m * 0.5; e += 1; }
    double f = m - 1.0;
    double s = f / (2.0 + f);
    double z = s * s;
    double p = 2.0 / 19.0;
    p = fma(p, z, 2.0 / 17.0);
    p = fma(p, z, 2.0 / 15.0);
    p = fma(p, z, 2.0 / 13.0);
    p = fma(p, z, 2.0 / 11.0);
    p = fma(p, z, 2.0 / 9.0);
    p = fma(p, z, 2.0 / 7.0);
    p = fma(p, z, 2.0 / 5.0);
    p = fma(p, z, 2.0 / 3.0);
    double t = s * z;
    double r = fma(t, p, 2.0 * s);
    return fma((double)e, 0.6931471805599453, r);
}

/* Standard Gumbel variate from one 32-bit word: u sits at the centre of its
 * 2^-32 cell, so it is never 0 or 1. */
double orc_gumbel_u32(uint32_t r)
{
    double u = ((double)r + 0.5) * 2.3283064365386963e-10; /* 2^-32, exact */
    double w = -orc_log(u);
    return -orc_log(w);
}

/* key_t = fl32( (double)s_t + (double)tau * g_t ); tau == 0 leaves s_t as is
 * and draws nothing. */
void orc_perturbed_keys(const float *logits, int32_t n_items, float tau,
                        uint64_t seed, uint32_t round, uint32_t l, uint32_t b,
                        uint32_t hsel, float *keys)
{
    for (int32_t t = 0; t < n_items; ++t) {
        if (tau == 0.0f) { keys[t] = logits[t]; continue; }
        double g = orc_gumbel_u32(orc_item_word(seed, round, l, b, hsel, (uint32_t)t));
        double noise = (double)tau * g;
        double k = (double)logits[t] + noise;
        keys[t] = (float)k;
    }
}

/* ------------------------------------------------------------ select ---- */

/* Total order on fp32 bit patterns that agrees with < on numbers and puts
 * -0 below +0: larger float <=> larger code. */
static uint32_t ordered_code(float x)
{
    uint32_t b;
    memcpy(&b, &x, 4);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

typedef struct { uint32_t code; int32_t idx; } orc_item;

static int cmp_key_desc_idx_asc(const void *pa, const void *pb)
{
    const orc_item *a = (const orc_item *)pa, *b = (const orc_item *)pb;
    if (a->code != b->code) return (a->code > b->code) ? -1 : 1;
    if (a->idx != b->idx) return (a->idx < b->idx) ? -1 : 1;
    return 0;
}

static int cmp_int32_asc(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/* sigma = the K items with the largest keys, in descending key order (equal
 * keys: lower index first); kept = the same items in ascending index order.
 * Returns 0, or -1 on bad arguments / NaN keys / allocation failure. */
int orc_select(const float *keys, int32_t n_items, int32_t K,
               int32_t *kept, int32_t *sigma)
{
    if (n_items < 0 || K < 0 || K > n_items) return -1;
    orc_item *it = (orc_item *)malloc(sizeof(orc_item) * (size_t)(n_items > 0 ? n_items : 1));
    if (!it) return -1;
    for (int32_t t = 0; t < n_items; ++t) {
        if (keys[t] != keys[t]) { free(it); return -1; }
        it[t].code = ordered_code(keys[t]);
        it[t].idx = t;
    }
    qsort(it, (size_t)n_items, sizeof(orc_item), cmp_key_desc_idx_asc);
    for (int32_t j = 0; j < K; ++j) { sigma[j] = it[j].idx; kept[j] = it[j].idx; }
    qsort(kept, (size_t)K, sizeof(int32_t), cmp_int32_asc);
    free(it);
    return 0;
}

/* ---------------------------------------------------------- log-prob ---- */

/* A pick of a masked entry (logit -inf: weight exp(-inf) = 0 in Eq. 2) has
 * probability zero, so the whole sequence has log-probability -inf.  This also
 * fixes the one case the formula leaves as 0/0: a masked pick at a step where
 * every entry still available is masked.  (Masked entries that are never picked
 * simply add nothing to any sum.) */
static int picks_a_masked_entry(const float *logits, const int32_t *sigma, int32_t K)
{
    for (int32_t j = 0; j < K; ++j)
        if (logits[sigma[j]] == -INFINITY) return 1;
    return 0;
}

/* Eq. 2, term by term: for j = 1..K the logit of the j-th pick minus the
 * logsumexp over every item not picked before it. O(nK). */
double orc_logprob_literal(const float *logits, int32_t n_items,
                           const int32_t *sigma, int32_t K)
{
    if (picks_a_masked_entry(logits, sigma, K)) return -INFINITY;
    unsigned char *gone = (unsigned char *)calloc((size_t)(n_items > 0 ? n_items : 1), 1);
    if (!gone) return NAN;
    double total = 0.0;
    for (int32_t j = 0; j < K; ++j) {
        double mx = -INFINITY;
        for (int32_t t = 0; t < n_items; ++t)
            if (!gone[t] && (double)logits[t] > mx) mx = (double)logits[t];
        double acc = 0.0;
        for (int32_t t = 0; t < n_items; ++t)
            if (!gone[t]) acc += exp((double)logits[t] - mx);
        double lse = mx + log(acc);
        total += (double)logits[sigma[j]] - lse;
        gone[sigma[j]] = 1;
    }
    free(gone);
    return total;
}

/* The same number in O(n + K): with m = max s and e_t = exp(s_t - m),
 * U = sum of e_t over items never picked, R_j = U + sum_{i >= j} e_{sigma_i}
 * (built from the last pick backwards, so only positive terms are added),
 * log p = sum_j (s_{sigma_j} - m) - sum_j log R_j. */
double orc_logprob_suffix(const float *logits, int32_t n_items,
                          const int32_t *sigma, int32_t K)
{
    if (picks_a_masked_entry(logits, sigma, K)) return -INFINITY;
    unsigned char *picked = (unsigned char *)calloc((size_t)(n_items > 0 ? n_items : 1), 1);
    if (!picked) return NAN;
    double mx = -INFINITY;
    for (int32_t t = 0; t < n_items; ++t)
        if ((double)logits[t] > mx) mx = (double)logits[t];
    for (int32_t j = 0; j < K; ++j) picked[sigma[j]] = 1;
    double U = 0.0;
    for (int32_t t = 0; t < n_items; ++t)
        if (!picked[t]) U += exp((double)logits[t] - mx);
    double total = 0.0, R = U;
    for (int32_t j = K - 1; j >= 0; --j) {
        double d = (double)logits[sigma[j]] - mx;
        R += exp(d);
        total += d - log(R);
    }
    free(picked);
    return total;
}

/* Gradient of Eq. 2 with respect to every logit, term by term: the j-th term
 * s_{sigma_j} - logsumexp(alive_j) contributes +1 at sigma_j and minus the
 * softmax over the items still alive at step j.  O(nK).  This is what the
 * eviction policy gradient of Eq. 4 multiplies by the advantage. */
void orc_logprob_grad_literal(const float *logits, int32_t n_items,
                              const int32_t *sigma, int32_t K, double *grad)
{
    unsigned char *gone = (unsigned char *)calloc((size_t)(n_items > 0 ? n_items : 1), 1);
    for (int32_t t = 0; t < n_items; ++t) grad[t] = 0.0;
    for (int32_t j = 0; j < K; ++j) {
        double mx = -INFINITY;
        for (int32_t t = 0; t < n_items; ++t)
            if (!gone[t] && (double)logits[t] > mx) mx = (double)logits[t];
        double den = 0.0;
        for (int32_t t = 0; t < n_items; ++t)
            if (!gone[t]) den += exp((double)logits[t] - mx);
        for (int32_t t = 0; t < n_items; ++t)
            if (!gone[t]) grad[t] -= exp((double)logits[t] - mx) / den;
        grad[sigma[j]] += 1.0;
        gone[sigma[j]] = 1;
    }
    free(gone);
}

/* -------------------------------------------------------- compaction ---- */

/* Rows are `row_elems` 16-bit words.  Items are blocks of `block` consecutive
 * rows (the last block of a segment of n rows may be short).  Kept items, in
 * ascending order, are packed to the front; returns the new row count.
 * dst may equal src (a sequential ascending copy never overtakes itself). */
int32_t orc_compact_rows(const uint16_t *src, uint16_t *dst, int32_t n_rows,
                         int32_t row_elems, int32_t block,
                         const int32_t *kept, int32_t K)
{
    int32_t out = 0;
    for (int32_t j = 0; j < K; ++j) {
        int32_t first = kept[j] * block;
        int32_t last = first + block;
        if (last > n_rows) last = n_rows;
        for (int32_t r = first; r < last; ++r, ++out)
            memmove(dst + (size_t)out * row_elems, src + (size_t)r * row_elems,
                    sizeof(uint16_t) * (size_t)row_elems);
    }
    return out;
}

int32_t orc_compact_i32(const int32_t *src, int32_t *dst, int32_t n_rows,
                        int32_t block, const int32_t *kept, int32_t K)
{
    int32_t out = 0;
    for (int32_t j = 0; j < K; ++j) {
        int32_t first = kept[j] * block;
        int32_t last = first + block;
        if (last > n_rows) last = n_rows;
        for (int32_t r = first; r < last; ++r, ++out) dst[out] = src[r];
    }
    return out;
}

/* Unordered variant ("fill the holes", single rows only): with K kept rows,
 * slots [0, K) that lose their row (holes, ascending) receive, in order, the
 * kept rows that sit at or beyond slot K (tails, ascending); kept rows already
 * below K stay where they are.  Same surviving set as orc_compact_rows, other
 * arrangement, far fewer rows moved.  Works on a copy: dst must not alias src.
 * Returns K. */
int32_t orc_compact_rows_unordered(const uint16_t *src, uint16_t *dst, int32_t n_rows,
                                   int32_t row_elems, const int32_t *kept, int32_t K)
{
    unsigned char *is_kept = (unsigned char *)calloc((size_t)(n_rows > 0 ? n_rows : 1), 1);
    if (!is_kept) return -1;
    for (int32_t j = 0; j < K; ++j) is_kept[kept[j]] = 1;
    /* rows that stay */
    for (int32_t r = 0; r < K && r < n_rows; ++r)
        if (is_kept[r])
            memcpy(dst + (size_t)r * row_elems, src + (size_t)r * row_elems,
                   sizeof(uint16_t) * (size_t)row_elems);
    /* i-th hole <- i-th tail */
    int32_t hole = 0;
    for (int32_t t = K; t < n_rows; ++t) {
        if (!is_kept[t]) continue;
        while (is_kept[hole]) ++hole;
        memcpy(dst + (size_t)hole * row_elems, src + (size_t)t * row_elems,
               sizeof(uint16_t) * (size_t)row_elems);
        ++hole;
    }
    free(is_kept);
    return K;
}

/* ---------------------------------------------------------- attention --- */

static double bf16_to_double(uint16_t h)
{
    uint32_t b = (uint32_t)h << 16;
    float f;
    memcpy(&f, &b, 4);
    return (double)f;
}

/* One KV head of one sequence: G query heads (rows of q) attend to the n
 * surviving rows of k and v.  x_j = scale * <q, k_j>; p = softmax(x);
 * o = sum_j p_j v_j.  n == 0 gives zeros.  Everything in fp64, the result is
 * rounded to fp32 once. */
void orc_decode_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                     int32_t n, int32_t G, int32_t D, double scale, float *out)
{
    double *x = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)D);
    for (int32_t g = 0; g < G; ++g) {
        double mx = -INFINITY;
        for (int32_t j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int32_t d = 0; d < D; ++d)
                acc += bf16_to_double(q[(size_t)g * D + d]) *
                       bf16_to_double(k[(size_t)j * D + d]);
            x[j] = acc * scale;
            if (x[j] > mx) mx = x[j];
        }
        double den = 0.0;
        for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
        for (int32_t j = 0; j < n; ++j) {
            double p = exp(x[j] - mx);
            den += p;
            for (int32_t d = 0; d < D; ++d)
                o[d] += p * bf16_to_double(v[(size_t)j * D + d]);
        }
        for (int32_t d = 0; d < D; ++d)
            out[(size_t)g * D + d] = (n > 0) ? (float)(o[d] / den) : 0.0f;
    }
    free(x);
    free(o);
}

/* log sum_j exp(scale * <q_g, k_j>) for every query head g (natural log,
 * -inf for n == 0): the normaliser of the attention above. */
void orc_decode_lse(const uint16_t *q, const uint16_t *k, int32_t n, int32_t G,
                    int32_t D, double scale, double *lse)
{
    for (int32_t g = 0; g < G; ++g) {
        double mx = -INFINITY, den = 0.0;
        double *x = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        for (int32_t j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int32_t d = 0; d < D; ++d)
                acc += bf16_to_double(q[(size_t)g * D + d]) * bf16_to_double(k[(size_t)j * D + d]);
            x[j] = acc * scale;
            if (x[j] > mx) mx = x[j];
        }
        for (int32_t j = 0; j < n; ++j) den += exp(x[j] - mx);
        lse[g] = (n > 0) ? mx + log(den) : -INFINITY;
        free(x);
    }
}

/* ------------------------------------------------------------ scoring --- */

/* Key importance for one KV head of one sequence (Sec. 4.2).
 *   q    [w][G][D]  queries of the w most recent tokens, G query heads each
 *   k    [n][D]     cached keys; the w most recent tokens are rows n-w .. n-1
 * For every query (j, g): a = softmax_t(scale * <q_{j,g}, k_t>) over the keys
 * it can see -- with causal != 0 query j (the token at row n-w+j) sees rows
 * t <= n-w+j, otherwise every query sees all n rows.  psi_t is the mean of
 * a_t over the w*G queries (0 where a query cannot see t). */
void orc_score_keys(const uint16_t *q, const uint16_t *k, int32_t n, int32_t w,
                    int32_t G, int32_t D, double scale, int32_t causal, double *psi)
{
    double *x = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    for (int32_t t = 0; t < n; ++t) psi[t] = 0.0;
    for (int32_t j = 0; j < w; ++j) {
        int32_t vis = causal ? (n - w + j + 1) : n;   /* number of visible rows */
        if (vis > n) vis = n;
        if (vis <= 0) continue;
        for (int32_t g = 0; g < G; ++g) {
            const uint16_t *qr = q + ((size_t)j * G + g) * D;
            double mx = -INFINITY;
            for (int32_t t = 0; t < vis; ++t) {
                double acc = 0.0;
                for (int32_t d = 0; d < D; ++d)
                    acc += bf16_to_double(qr[d]) * bf16_to_double(k[(size_t)t * D + d]);
                x[t] = acc * scale;
                if (x[t] > mx) mx = x[t];
            }
            double den = 0.0;
            for (int32_t t = 0; t < vis; ++t) den += exp(x[t] - mx);
            for (int32_t t = 0; t < vis; ++t) psi[t] += exp(x[t] - mx) / den;
        }
    }
    for (int32_t t = 0; t < n; ++t) psi[t] /= (double)(w * G);
    free(x);
}

/* s_j = mean of psi over block j (blocks of `block` consecutive keys, the
 * last one possibly short; every key is valid). */
void orc_block_means(const double *psi, int32_t n, int32_t block, double *s)
{
    int32_t N = (n + block - 1) / block;
    for (int32_t j = 0; j < N; ++j) {
        int32_t lo = j * block, hi = lo + block < n ? lo + block : n;
        double acc = 0.0;
        for (int32_t t = lo; t < hi; ++t) acc += psi[t];
        s[j] = acc / (double)(hi - lo);
    }
}

/* ------------------------------------------------------------- replay --- */

/* One KV head of one sequence, all T positions at once.  death[j] is the first
 * query position that can no longer see key j (T or more if j is never
 * evicted); visibility is  j <= i < death[j]  (Sec. 4.5: the mask replicates
 * the visibility pattern that the eviction decisions induced).
 *   q [T][G][D], k, v [T][D]  ->  out [T][G][D] (fp32). */
void orc_replay_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                     const int32_t *death, int32_t T, int32_t G, int32_t D,
                     double scale, float *out)
{
    double *x = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)D);
    for (int32_t i = 0; i < T; ++i)
        for (int32_t g = 0; g < G; ++g) {
            const uint16_t *qr = q + ((size_t)i * G + g) * D;
            double mx = -INFINITY;
            for (int32_t j = 0; j <= i; ++j) {
                if (death[j] <= i) continue;
                double acc = 0.0;
                for (int32_t d = 0; d < D; ++d)
                    acc += bf16_to_double(qr[d]) * bf16_to_double(k[(size_t)j * D + d]);
                x[j] = acc * scale;
                if (x[j] > mx) mx = x[j];
            }
            double den = 0.0;
            for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
            for (int32_t j = 0; j <= i; ++j) {
                if (death[j] <= i) continue;
                double p = exp(x[j] - mx);
                den += p;
                for (int32_t d = 0; d < D; ++d) o[d] += p * bf16_to_double(v[(size_t)j * D + d]);
            }
            for (int32_t d = 0; d < D; ++d)
                out[((size_t)i * G + g) * D + d] = (den > 0.0) ? (float)(o[d] / den) : 0.0f;
        }
    free(x);
    free(o);
}
