// Segmented Gumbel-top-k selection for gfx950, shared by the eviction kernels of
// the contiguous and of the paged cache layout: perturbed keys, radix select of
// the K-th largest, ascending kept list, sampled order (sigma) and its
// ordered-subset log-probability.
//
// Translation units that include this header are compiled with
// -ffp-contract=off: the noise arithmetic is an exact operation sequence (see
// ngc_noise.h).
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/ngc.h"
#include "ngc_device.h"
#include "ngc_noise.h"
#include "ngc_logsum.h"

namespace ngc {

// ------------------------------------------------------------ geometry ----

struct SegGeom {
    int B, Hkv, cap, block;
};

__device__ __forceinline__ void seg_coords(int seg, const SegGeom &g, int &l, int &b, int &h)
{
    h = seg % g.Hkv;
    const int lb = seg / g.Hkv;
    b = lb % g.B;
    l = lb / g.B;
}

// Rows in use of a segment, clamped to [0, cap]; counts a clamp.
__device__ __forceinline__ int seg_rows(const int32_t *len, int seg, int cap, int32_t *status)
{
    int n = len[seg];
    if (n < 0 || n > cap) {
        if (threadIdx.x == 0) atomicAdd(&status[NGC_STATUS_LEN_CLAMPED], 1);
        n = n < 0 ? 0 : cap;
    }
    return n;
}

// ------------------------------------------------------ perturbed keys ----

struct NoiseArgs {
    uint64_t seed;
    uint32_t round;
    float tau;
    int share_heads;
    int layer_base;   // global index of the view's layer 0 and sequence 0: the noise of an entry depends on
    int seq_base;     // where it sits in the model and the batch, not on how the caller sliced its buffers
};

// Keys of items 4*quad .. 4*quad+3 (those below n_items), one Philox call.
__device__ __forceinline__ void keys_of_quad(const float *row, int n_items, int quad,
                                             const NoiseArgs &na, int l, int b, int h,
                                             float s[4], float key[4])
{
    const int t0 = 4 * quad;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float x = (t0 + i < n_items) ? row[t0 + i] : -INFINITY;
        if (x != x) x = -INFINITY;   // NaN logits count as masked
        s[i] = x;
    }
    if (na.tau == 0.0f) {
#pragma unroll
        for (int i = 0; i < 4; ++i) key[i] = s[i];
        return;
    }
    uint32_t w[4];
    item_words(na.seed, na.round, (uint32_t)(l + na.layer_base), (uint32_t)(b + na.seq_base),
               na.share_heads ? 0xFFFFu : (uint32_t)h, (uint32_t)quad, w);
#pragma unroll
    for (int i = 0; i < 4; ++i) key[i] = perturb(s[i], na.tau, w[i]);
}

// ------------------------------------------------------------- select -----
//
// One workgroup works on one segment at a time.  LDS holds the order-preserving code of every
// perturbed key (4 B per item), two index buffers for the sort of the kept
// items (2 B per kept item each) and a histogram area.
//
//   1. keys:    4 items per thread per step, one Philox call per 4 items.
//   2. select:  the K-th largest code by a 3-pass radix select (11+11+10 bits)
//               over LDS histograms.
//   3. kept:    each wave owns a contiguous range of items; ballots and lane
//               prefix counts give every kept item its ascending output slot.
//               Items equal to the threshold are taken lowest index first.
//   4. sigma:   stable LSD radix sort (4 x 8 bits) of the kept indices by
//               descending code; stability plus the ascending start order is
//               the index tie-break.
//   5. logp:    Eq. 2 in the reverse-running-sum form: U = mass never picked,
//               R_j = U + sum_{i>=j} e_sigma_i built from the last pick
//               backwards; log p = sum_j (s_sigma_j - m) - sum_j log R_j.

constexpr int SEL_BINS = 2048;

struct SelectArgs {
    const float *logits;
    const int32_t *len;
    const int32_t *keep;
    int32_t *kept_out;
    int32_t *sigma_out;
    float *logp_out;
    int32_t *status;
    // compaction (skipped when k == nullptr)
    void *k;
    void *v;
    int32_t *pos;
    int32_t *len_out;
    int unordered;       // 1: fill the holes below K with the kept rows beyond K (block == 1 only)
    int seg0;
    int nseg;            // segments of the launch (the persistent eviction kernel hands them out one by one)
    int max_keep;
    int items_cap;       // ceil(cap / block): size of the code array in LDS
    int keep_cap;        // size of each index buffer in LDS
    int64_t logit_stride; // floats between the logit rows of consecutive segments
    uint32_t *pool_codes; // pooled mode: key codes of every item, Hkv * cap per (layer, sequence)
    SegGeom g;
    NoiseArgs na;
};

// The last two status words of the workspace are the library's own: a work counter and a count of finished
// workgroups of the eviction kernel, both zero between launches.
constexpr int WS_QUEUE_NEXT = NGC_STATUS_WORDS - 2;
constexpr int WS_QUEUE_DONE = NGC_STATUS_WORDS - 1;

constexpr int SMALL_ITEMS = 256;             // at most this many items: selection by ranking
constexpr int SORT_BITS = 9;                 // digit width of the sigma sort
constexpr int SORT_BINS = 1 << SORT_BITS;

// For each lane: the set of lanes of this wave whose SORT_BITS-bit digit equals
// its own, restricted to `valid` lanes.
__device__ __forceinline__ uint64_t match_digit(uint32_t d, uint64_t valid)
{
    uint64_t m = valid;
#pragma unroll
    for (int bit = 0; bit < SORT_BITS; ++bit) {
        const bool on = (d >> bit) & 1u;
        const uint64_t bal = __ballot(on);
        m &= on ? bal : ~bal;
    }
    return m;
}

// Unordered arrangement (single rows): kept rows below slot K stay; the i-th
// kept row at or beyond K moves into the i-th free slot below K.  Sources and
// destinations are disjoint, so there is no ordering to respect and no barrier.
// `kept` is the ascending kept list in LDS.  kept[0 .. jstar) are the kept rows
// below K; the i-th number missing from that list is i + #{p : kept[p] - p <= i}.
template <int ROW_BYTES, int THREADS, int UNROLL>
__device__ __forceinline__ void fill_holes_inplace(unsigned char *kbase, unsigned char *vbase, int32_t *pos,
                                                   const uint16_t *kept, int K)
{
    constexpr int PIECES = ROW_BYTES / 16;
    constexpr int ROWS_PER_STEP = THREADS / PIECES;
    int lo = 0, hi = K;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((int)kept[mid] < K) lo = mid + 1; else hi = mid;
    }
    const int jstar = lo, movers = K - jstar;
    auto hole_of = [&](int i) {
        int a = 0, b = jstar;
        while (a < b) {
            const int mid = (a + b) >> 1;
            if ((int)kept[mid] - mid <= i) a = mid + 1; else b = mid;
        }
        return i + a;
    };
    const int piece = threadIdx.x % PIECES, rsub = threadIdx.x / PIECES;
    for (int i0 = 0; i0 < movers; i0 += ROWS_PER_STEP * UNROLL) {
        u32x4 kb[UNROLL], vb[UNROLL];
        int dst[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int i = i0 + u * ROWS_PER_STEP + rsub;
            dst[u] = -1;
            kb[u] = u32x4{0u, 0u, 0u, 0u};
            vb[u] = u32x4{0u, 0u, 0u, 0u};
            if (i < movers) {
                const size_t off = (size_t)kept[jstar + i] * ROW_BYTES + piece * 16;
                kb[u] = *reinterpret_cast<const u32x4 *>(kbase + off);
                vb[u] = *reinterpret_cast<const u32x4 *>(vbase + off);
                dst[u] = hole_of(i);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            if (dst[u] >= 0) {
                const size_t off = (size_t)dst[u] * ROW_BYTES + piece * 16;
                *reinterpret_cast<u32x4 *>(kbase + off) = kb[u];
                *reinterpret_cast<u32x4 *>(vbase + off) = vb[u];
            }
    }
    if (pos)
        for (int i = threadIdx.x; i < movers; i += THREADS) pos[hole_of(i)] = pos[kept[jstar + i]];
}

// ------------------------------------------------- shared building blocks --
//
// The two steps every variant of the selection shares (segments of one head in
// LDS, pooled segments of all heads of a sequence with their codes in global
// memory, pages as items).  `code_at(i)` returns the key code of item i.

// K-th largest of the N codes by a 3-pass radix select (11 + 11 + 10 bits) over LDS histograms.  Returns that
// code; `need` = how many of the items equal to it are taken (lowest index first).  With `have_first` the caller
// has already accumulated the histogram of the top 11 bits in hist[0 .. SEL_BINS) (and passed a barrier).
// Whole workgroup; ends on a barrier.  Uses misc[0 .. 34).
template <int THREADS, class CodeAt>
__device__ __forceinline__ uint32_t radix_select_kth(CodeAt code_at, int N, int K, uint32_t *hist, int *misc,
                                                     int &need, bool have_first)
{
    const int tid = threadIdx.x;
    uint32_t prefix = 0, pmask = 0;
    need = K;   // how many of the items matching `prefix` are still to take
    const int shifts[3] = {21, 10, 0};
    const int widths[3] = {11, 11, 10};
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = shifts[pass], nb = 1 << widths[pass];
        if (pass > 0 || !have_first) {
            for (int i = tid; i < nb; i += THREADS) hist[i] = 0;
            __syncthreads();
            for (int t = tid; t < N; t += THREADS) {
                const uint32_t u = code_at(t);
                if ((u & pmask) == prefix) atomicAdd(&hist[(u >> shift) & (nb - 1)], 1u);
            }
        }
        __syncthreads();
        // bins in descending digit order; each thread owns `per` of them
        const int per = (nb + THREADS - 1) / THREADS;
        int mine = 0;
        for (int i = 0; i < per; ++i) {
            const int p = tid * per + i;
            if (p < nb) mine += (int)hist[nb - 1 - p];
        }
        int total;
        int above = block_excl_scan_i<THREADS>(mine, misc, &total);
        if (above < need && need <= above + mine) {
            for (int i = 0; i < per; ++i) {
                const int p = tid * per + i;
                const int c = (p < nb) ? (int)hist[nb - 1 - p] : 0;
                if (need <= above + c) {
                    misc[32] = nb - 1 - p;   // digit of the K-th largest
                    misc[33] = above;        // matching items with a larger digit
                    break;
                }
                above += c;
            }
        }
        __syncthreads();
        const uint32_t digit = (uint32_t)misc[32];
        need -= misc[33];
        prefix |= digit << shift;
        pmask |= (uint32_t)(nb - 1) << shift;
        __syncthreads();
    }
    return prefix;
}

// Sort of the K entries of idxA (u16 handles, ascending) by descending code, equal codes by ascending handle.
// The sort key is cmax - code_of(handle), which for kept items lies in [0, cmax - thr].
//
// Fast path: one counting pass into as many buckets as the histogram area holds, a prefix sum, an unordered scatter by bucket (LDS atomics hand out the positions), and then every entry finds
// its place inside its bucket by counting the entries of that bucket that precede it in the total order -- which
// makes the result independent of the order in which the atomics were served.  With thousands of buckets for
// thousands of kept items a bucket holds a few entries.  Whole workgroup; ends on a barrier.
//
// Fallback (a bucket above BUCKET_LIMIT entries: many equal or nearly equal keys): stable LSD radix sort, only
// the bits of the key range, SORT_BITS at a time; per-wave digit counts by LDS atomics, ranks inside a wave by
// match-any ballots -- stability plus the ascending start order is the index tie-break.
// Returns the buffer (idxA or idxB) that holds the sorted handles.  hist holds max(SEL_BINS, SORT_BINS * waves)
// entries.
constexpr int BUCKET_LIMIT = 64;

template <int THREADS, class CodeOf>
__device__ __forceinline__ uint16_t *sort_by_code_desc(CodeOf code_of, int K, uint32_t cmax, uint32_t thr,
                                                       uint16_t *idxA, uint16_t *idxB, uint32_t *hist, int *misc)
{
    constexpr int NW = THREADS / NGC_WAVE;
    constexpr int NB = (SEL_BINS > SORT_BINS * NW) ? SEL_BINS : SORT_BINS * NW;   // buckets = entries of hist
    static_assert(NB % THREADS == 0, "every thread owns the same number of buckets");
    const int tid = threadIdx.x, lane = lane_id(), wv = wave_id();
    const uint32_t range = cmax - thr;
    const int range_bits = range ? 32 - __clz(range) : 0;
    if (range_bits == 0) return idxA;   // all codes equal: the ascending start order is the answer
    // Buckets are equal slices of the VALUE range [key of thr, key of cmax] (not of the code range, which is
    // logarithmic in the value and nearly empty around zero): bucket = floor((kmax - key) * NB / width), a
    // non-increasing function of the key in IEEE arithmetic, so a larger key never lands in a later bucket.
    const float kmax = code_to_float(cmax), kthr = code_to_float(thr);
    const float width = kmax - kthr;
    if (width > 0.f && width < INFINITY) {
        const float per_value = (float)(NB - 1) / width;
        auto bucket_of = [&](uint32_t c) -> uint32_t {
            const float x = (kmax - code_to_float(c)) * per_value;     // >= 0; +inf for a masked key
            return (uint32_t)fminf(x, (float)(NB - 1));
        };
        for (int i = tid; i < NB; i += THREADS) hist[i] = 0;
        __syncthreads();
        for (int j = tid; j < K; j += THREADS) atomicAdd(&hist[bucket_of(code_of(idxA[j]))], 1u);
        __syncthreads();
        // bucket starts (exclusive prefix sum; every thread owns PER consecutive buckets) and the largest bucket
        constexpr int PER = NB / THREADS;
        int vals[PER], sum = 0;
        uint32_t biggest = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            vals[i] = (int)hist[tid * PER + i];
            sum += vals[i];
            biggest = (uint32_t)vals[i] > biggest ? (uint32_t)vals[i] : biggest;
        }
        biggest = block_max_u<THREADS>(biggest, reinterpret_cast<uint32_t *>(misc));
        if (biggest <= (uint32_t)BUCKET_LIMIT) {
            int total;
            int run = block_excl_scan_i<THREADS>(sum, misc, &total);
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                hist[tid * PER + i] = (uint32_t)run;
                run += vals[i];
            }
            __syncthreads();
            // unordered scatter: afterwards hist[b] is the END of bucket b (and the start of bucket b + 1)
            for (int j = tid; j < K; j += THREADS) {
                const uint16_t h = idxA[j];
                const uint32_t pos = atomicAdd(&hist[bucket_of(code_of(h))], 1u);
                idxB[pos] = h;
            }
            __syncthreads();
            // place inside the bucket: count the bucket's entries that come first (larger code, or the same code
            // and a smaller handle)
            for (int p = tid; p < K; p += THREADS) {
                const uint16_t h = idxB[p];
                const uint32_t c = code_of(h);
                const uint32_t b = bucket_of(c);
                const int start = b ? (int)hist[b - 1] : 0, end = (int)hist[b];
                int rank = 0;
                for (int q = start; q < end; ++q) {
                    const uint16_t h2 = idxB[q];
                    const uint32_t c2 = code_of(h2);
                    rank += (c2 > c || (c2 == c && h2 < h)) ? 1 : 0;
                }
                idxA[start + rank] = h;
            }
            __syncthreads();
            return idxA;
        }
    }
    // ---- fallback: stable LSD radix sort ---------------------------------------------------------------------
    const int per_wave_k = (((K + NW - 1) / NW) + NGC_WAVE - 1) & ~(NGC_WAVE - 1);
    const int k_begin = wv * per_wave_k;
    const int k_end = (k_begin + per_wave_k < K) ? (k_begin + per_wave_k) : K;
    uint16_t *cur = idxA, *dst = idxB;
    volatile uint32_t *vh = hist;
    const int passes = (range_bits + SORT_BITS - 1) / SORT_BITS;
#pragma unroll 1
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = SORT_BITS * pass;
        for (int i = tid; i < SORT_BINS * NW; i += THREADS) hist[i] = 0;
        __syncthreads();
        // per-wave digit counts over the wave's own contiguous range
        for (int j0 = k_begin; j0 < k_end; j0 += NGC_WAVE) {
            const int j = j0 + lane;
            if (j < k_end) {
                const uint32_t d = ((cmax - code_of(cur[j])) >> shift) & (SORT_BINS - 1);
                atomicAdd(&hist[wv * SORT_BINS + d], 1u);
            }
        }
        __syncthreads();
        // exclusive scan in (digit, wave) order; every thread owns PER consecutive entries
        {
            constexpr int PER = SORT_BINS * NW / THREADS;
            int vals[PER], sum = 0;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int e = tid * PER + i;
                vals[i] = (int)hist[(e % NW) * SORT_BINS + e / NW];
                sum += vals[i];
            }
            int total;
            int run = block_excl_scan_i<THREADS>(sum, misc, &total);
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int e = tid * PER + i;
                hist[(e % NW) * SORT_BINS + e / NW] = (uint32_t)run;
                run += vals[i];
            }
        }
        __syncthreads();
        // scatter in order: rank within the batch + running offset of (wave, digit)
        for (int j0 = k_begin; j0 < k_end; j0 += NGC_WAVE) {
            const int j = j0 + lane;
            const bool in = j < k_end;
            const uint16_t idx = in ? cur[j] : (uint16_t)0;
            const uint32_t d = in ? ((cmax - code_of(idx)) >> shift) & (SORT_BINS - 1) : 0u;
            const uint64_t peers = match_digit(d, __ballot(in));
            const int rank = popc_below(peers);
            uint32_t base = 0;
            if (in) base = vh[wv * SORT_BINS + d];
            __builtin_amdgcn_wave_barrier();
            if (in) {
                dst[base + rank] = idx;
                if (rank == 0) vh[wv * SORT_BINS + d] = base + (uint32_t)__popcll(peers);
            }
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
        uint16_t *tmp = cur; cur = dst; dst = tmp;
    }
    return cur;
}

// Slots of the small shared scratch array `misc` that outlive the selection.
constexpr int MISC_KEPT = 35;   // items kept in this segment
constexpr int MISC_ROWS = 36;   // rows in use after compaction
constexpr int MISC_FIRST = 37;  // first item that changes place

// Selection of one segment by the whole workgroup.  Leaves the kept count and
// the new row count in misc[MISC_KEPT], misc[MISC_ROWS] (valid after the next
// barrier).  Every thread of the workgroup returns at the same point.
template <int THREADS, int ROW_BYTES>
__device__ __forceinline__ void select_segment(const SelectArgs &a, int seg, unsigned char *smem_raw)
{
    constexpr int NW = THREADS / NGC_WAVE;
    constexpr int HIST = (SEL_BINS > SORT_BINS * NW) ? SEL_BINS : SORT_BINS * NW;
    uint32_t *code = reinterpret_cast<uint32_t *>(smem_raw);
    uint32_t *hist = code + a.items_cap;
    int *misc = reinterpret_cast<int *>(hist + HIST);            // 64 ints
    uint16_t *idxA = reinterpret_cast<uint16_t *>(misc + 64);
    uint16_t *idxB = idxA + a.keep_cap;
    float *fmisc = reinterpret_cast<float *>(misc);

    const int tid = threadIdx.x, lane = lane_id(), wv = wave_id();
    int l, b, h;
    seg_coords(seg, a.g, l, b, h);
    const int n = seg_rows(a.len, seg, a.g.cap, a.status);
    const int N = (n + a.g.block - 1) / a.g.block;
    int K = a.keep[seg];
    {
        int lim = N < a.max_keep ? N : a.max_keep;
        if (K < 0 || K > lim) {   // also when only max_keep (the row length of kept_out) is exceeded
            if (tid == 0) atomicAdd(&a.status[NGC_STATUS_KEEP_CLAMPED], 1);
            K = K < 0 ? 0 : lim;
        }
    }
    const float *row = a.logits + (size_t)seg * a.logit_stride;
    const bool want_logp = a.logp_out != nullptr;
    const bool want_sort = want_logp || a.sigma_out != nullptr;
    const bool fill_holes = a.unordered && a.k != nullptr;

    if (K == 0) {
        if (tid == 0) {
            misc[MISC_KEPT] = 0;
            misc[MISC_ROWS] = 0;
            if (want_logp) a.logp_out[seg] = 0.f;
        }
        return;
    }

    // ---- 1. keys ----------------------------------------------------------
    float smax = -INFINITY, neg_smin = -INFINITY;   // over the unmasked entries (a NaN compares false everywhere)
    uint32_t cmax = 0;
    for (int quad = tid; 4 * quad < N; quad += THREADS) {
        float s[4], key[4];
        keys_of_quad(row, N, quad, a.na, l, b, h, s, key);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * quad + i < N) {
                const uint32_t c = ordered_code(key[i]);
                code[4 * quad + i] = c;
                cmax = c > cmax ? c : cmax;
                smax = fmaxf(smax, s[i]);
                if (s[i] > -INFINITY) neg_smin = fmaxf(neg_smin, -s[i]);
            }
    }
    // Logits that span more than NGC_WIDE_SPREAD take the wide-range arithmetic of ngc_logsum.h for Eq. 2
    // (workgroup-uniform).
    bool wide = false;
    if (want_logp) {
        block_max2_f<THREADS>(smax, neg_smin, fmisc);   // has barriers
        wide = smax > -INFINITY && smax + neg_smin > NGC_WIDE_SPREAD;
        if (smax == -INFINITY) smax = 0.f;          // every entry masked: all weights are 0 (log p = -inf below)
    }
    if (want_sort) cmax = block_max_u<THREADS>(cmax, reinterpret_cast<uint32_t *>(misc));

    // Large segments: radix select, ballot compaction, radix sort (steps 2-4).  Segments of at most
    // SMALL_ITEMS items (blocks or pages as items, the paper's own sizes): ranking by counting instead.
    uint16_t *src = idxA;   // the kept items in sampled order, once known
    float unpicked = 0.f;   // sum of exp(s - smax) over items not kept (for logp)
    LogSum unpicked_w = ls_empty();   // the same sum on the wide-range route
    if (N > SMALL_ITEMS) {
        // ---- 2. radix select of the K-th largest code -------------------------
        int need;   // items equal to the threshold that are kept
        const uint32_t thr = radix_select_kth<THREADS>([&](int t) { return code[t]; }, N, K, hist, misc, need, false);

        // ---- 3. kept list, ascending ------------------------------------------
        const int per_wave = (((N + NW - 1) / NW) + NGC_WAVE - 1) & ~(NGC_WAVE - 1);
        const int w_begin = wv * per_wave;
        const int w_end = (w_begin + per_wave < N) ? (w_begin + per_wave) : N;
        {
            int gt = 0, eq = 0;
            for (int t0 = w_begin; t0 < w_end; t0 += NGC_WAVE) {
                const int t = t0 + lane;
                const uint32_t u = (t < w_end) ? code[t] : 0u;
                gt += __popcll(__ballot(t < w_end && u > thr));
                eq += __popcll(__ballot(t < w_end && u == thr));
            }
            if (lane == 0) { misc[wv] = gt; misc[16 + wv] = eq; }
        }
        __syncthreads();
        int gt_base = 0, eq_base = 0;
        for (int w = 0; w < wv; ++w) { gt_base += misc[w]; eq_base += misc[16 + w]; }
        unpicked = 0.f;
        int32_t *kept_row = a.kept_out + (size_t)seg * a.max_keep;
        for (int t0 = w_begin; t0 < w_end; t0 += NGC_WAVE) {
            const int t = t0 + lane;
            const bool in = t < w_end;
            const uint32_t u = in ? code[t] : 0u;
            const bool is_gt = in && u > thr, is_eq = in && u == thr;
            const uint64_t bgt = __ballot(is_gt), beq = __ballot(is_eq);
            const int gt_before = gt_base + popc_below(bgt);
            const int eq_before = eq_base + popc_below(beq);
            const bool sel = is_gt || (is_eq && eq_before < need);
            if (sel) {
                const int slot = gt_before + (eq_before < need ? eq_before : need);
                kept_row[slot] = t;
                if (want_sort || fill_holes) idxA[slot] = (uint16_t)t;
                if (slot == K - 1) misc[34] = t;   // highest kept index
            } else if (in && want_logp) {
                float x = row[t];
                if (x != x) x = -INFINITY;
                if (wide) unpicked_w = ls_add_term(unpicked_w, x);
                else unpicked += expf(x - smax);
            }
            gt_base += __popcll(bgt);
            eq_base += __popcll(beq);
        }
        __syncthreads();
        if (tid == 0) {
            const int last_item = misc[34];
            const int last_rows = (last_item == N - 1) ? (n - (N - 1) * a.g.block) : a.g.block;
            misc[MISC_KEPT] = K;
            misc[MISC_ROWS] = (K - 1) * a.g.block + last_rows;
        }
        if (fill_holes) {
            // idxA still holds the kept list in ascending order (the sort below permutes it)
            const size_t seg_off = (size_t)seg * a.g.cap * ROW_BYTES;
            fill_holes_inplace<ROW_BYTES, THREADS, 4>(reinterpret_cast<unsigned char *>(a.k) + seg_off,
                                                      reinterpret_cast<unsigned char *>(a.v) + seg_off,
                                                      a.pos ? a.pos + (size_t)seg * a.g.cap : nullptr, idxA, K);
        }
        if (want_sort) {

            // ---- 4. sigma: stable sort of the kept indices by descending code ------
            src = sort_by_code_desc<THREADS>([&](uint16_t t) { return code[t]; }, K, cmax, thr, idxA, idxB, hist, misc);
        }
    } else {
        // ---- 2'-4'. few items: rank every key by counting ---------------------
        // rank_t = number of keys that precede key t in the total order (larger code, or equal code and
        // smaller index).  rank < K <=> kept, and sigma[rank] = t directly: no select passes, no sort.
        // N * N / THREADS compares, each thread streaming the codes from LDS four at a time.
        for (int t = N + tid; t < ((N + 3) & ~3); t += THREADS) code[t] = 0;   // padding never outranks anything
        __syncthreads();
        int32_t *kept_row = a.kept_out + (size_t)seg * a.max_keep;
        int kept_so_far = 0;
        for (int t0 = 0; t0 < N; t0 += THREADS) {
            const int t = t0 + tid;
            const bool in = t < N;
            int rank = 0;
            if (in) {
                const uint32_t c = code[t];
                for (int u = 0; u < N; u += 4) {
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(&code[u]);
#pragma unroll
                    for (int i = 0; i < 4; ++i) rank += (v[i] > c || (v[i] == c && u + i < t)) ? 1 : 0;
                }
            }
            const bool sel = in && rank < K;
            const uint64_t bal = __ballot(sel);
            if (lane == 0) misc[wv] = __popcll(bal);
            __syncthreads();
            int before = kept_so_far, total = 0;
            for (int w = 0; w < NW; ++w) {
                const int c = misc[w];
                if (w < wv) before += c;
                total += c;
            }
            if (sel) {
                const int slot = before + popc_below(bal);
                kept_row[slot] = t;
                idxA[slot] = (uint16_t)t;        // ascending (the unordered arrangement reads it)
                idxB[rank] = (uint16_t)t;        // sampled order
                if (slot == K - 1) misc[34] = t; // highest kept index
            } else if (in && want_logp) {
                float x = row[t];
                if (x != x) x = -INFINITY;
                if (wide) unpicked_w = ls_add_term(unpicked_w, x);
                else unpicked += expf(x - smax);
            }
            kept_so_far += total;
            __syncthreads();
        }
        if (tid == 0) {
            const int last_item = misc[34];
            const int last_rows = (last_item == N - 1) ? (n - (N - 1) * a.g.block) : a.g.block;
            misc[MISC_KEPT] = K;
            misc[MISC_ROWS] = (K - 1) * a.g.block + last_rows;
        }
        if (fill_holes) {
            const size_t seg_off = (size_t)seg * a.g.cap * ROW_BYTES;
            fill_holes_inplace<ROW_BYTES, THREADS, 4>(reinterpret_cast<unsigned char *>(a.k) + seg_off,
                                                      reinterpret_cast<unsigned char *>(a.v) + seg_off,
                                                      a.pos ? a.pos + (size_t)seg * a.g.cap : nullptr, idxA, K);
        }
        src = idxB;
    }
    if (!want_sort) return;
    // the sorted list is in `src` (idxA or idxB, depending on the number of passes)
    if (a.sigma_out) {
        int32_t *sig_row = a.sigma_out + (size_t)seg * a.max_keep;
        for (int j = tid; j < K; j += THREADS) sig_row[j] = (int32_t)src[j];
    }
    if (!want_logp) return;

    // ---- 5. log-probability of sigma (Eq. 2) -------------------------------
    // The logits of the picked items, minus the maximum, are gathered into LDS first (over the key codes,
    // which are no longer needed), all loads in flight at once: the serial chunk loops below then never wait
    // for a gather.
    float *ds = reinterpret_cast<float *>(code);
    for (int j = tid; j < K; j += THREADS) {
        float x = row[src[j]];
        if (x != x) x = -INFINITY;
        ds[j] = wide ? x : x - smax;   // the wide-range route works on the logits as they came
    }
    __syncthreads();
    if (wide) {
        const LogSum Uw = block_sum_ls<THREADS>(unpicked_w, fmisc);
        const float lpw = sigma_logprob_wide<THREADS>([&](int j) { return ds[j]; }, K, Uw, fmisc);
        if (tid == 0) a.logp_out[seg] = lpw;
        return;
    }
    const float U = block_sum_f<THREADS>(unpicked, fmisc);
    const int chunk = (K + THREADS - 1) / THREADS;
    const int nchunks = (K + chunk - 1) / chunk;
    // thread 0 owns the LAST chunk, so an ordinary exclusive scan over threads
    // yields the mass of everything picked after a thread's chunk
    const int cidx = nchunks - 1 - tid;
    const int j_lo = cidx * chunk;
    const int j_hi = (cidx >= 0) ? ((j_lo + chunk < K) ? j_lo + chunk : K) : 0;
    float mass = 0.f;
    if (cidx >= 0)
        for (int j = j_lo; j < j_hi; ++j) mass += expf(ds[j]);
    float total_mass;
    const float after = block_excl_scan_f<THREADS>(mass, fmisc, &total_mass);
    float acc = 0.f;
    if (cidx >= 0) {
        float R = U + after;
        for (int j = j_hi - 1; j >= j_lo; --j) {
            const float d = ds[j];
            R += expf(d);
            // a masked pick (logit -inf) has probability 0: log p = -inf, also where nothing unmasked is left (R == 0)
            acc += (d == -INFINITY) ? -INFINITY : d - logf(R);
        }
    }
    const float lp = block_sum_f<THREADS>(acc, fmisc);
    if (tid == 0) a.logp_out[seg] = lp;
}

}  // namespace ngc
