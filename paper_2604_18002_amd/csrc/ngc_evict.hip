// Eviction step kernels for gfx950: perturbed keys, segmented Gumbel-top-k
// selection with its ordered-subset log-probability, in-place compaction of
// the surviving K/V rows, and the row append used between rounds.
//
// The selection itself lives in ngc_select.h.  Compiled with -ffp-contract=off:
// the noise arithmetic is an exact operation sequence (see ngc_noise.h).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <map>
#include <mutex>

#include "../../include/ngc.h"
#include "ngc_device.h"
#include "ngc_noise.h"
#include "ngc_select.h"
#include "ngc_logsum.h"

namespace ngc {

__global__ __launch_bounds__(256) void perturbed_keys_kernel(
    const float *__restrict__ logits, const int32_t *__restrict__ len, float *__restrict__ keys_out,
    int seg0, SegGeom g, NoiseArgs na, int32_t *status)
{
    const int seg = seg0 + blockIdx.x;
    int l, b, h;
    seg_coords(seg, g, l, b, h);
    const int n = seg_rows(len, seg, g.cap, status);
    const int n_items = (n + g.block - 1) / g.block;
    const float *row = logits + (size_t)seg * g.cap;
    float *out = keys_out + (size_t)seg * g.cap;
    for (int quad = threadIdx.x; 4 * quad < n_items; quad += 256) {
        float s[4], key[4];
        keys_of_quad(row, n_items, quad, na, l, b, h, s, key);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * quad + i < n_items) out[4 * quad + i] = key[i];
    }
}

// ------------------------------------------- log-prob of given actions ----

struct LogprobArgs {
    const float *logits;
    const int32_t *n_items;
    const int32_t *sigma;
    const int32_t *keep;
    float *logp_out;
    int32_t *status;
    int64_t logit_stride;
    int sigma_stride;
    int stage_cap;   // floats of dynamic LDS for the picked items' terms
};

// One workgroup per segment; LDS bitmap of picked items (65536 bits).
template <int THREADS>
__global__ __launch_bounds__(THREADS) void subset_logprob_kernel(LogprobArgs a)
{
    extern __shared__ float staged[];         // stage_cap floats
    __shared__ uint32_t picked[2048];
    __shared__ float fmisc[32];
    const int tid = threadIdx.x;
    const int seg = blockIdx.x;
    int N = a.n_items[seg];
    if (N < 0) N = 0;
    if (N > 65536) N = 65536;
    int K = a.keep[seg];
    if (K < 0 || K > N) {
        if (tid == 0) atomicAdd(&a.status[NGC_STATUS_KEEP_CLAMPED], 1);
        K = K < 0 ? 0 : N;
    }
    const float *row = a.logits + (size_t)seg * a.logit_stride;
    const int32_t *sig = a.sigma + (size_t)seg * a.sigma_stride;
    if (K == 0) {
        if (tid == 0) a.logp_out[seg] = 0.f;
        return;
    }
    for (int i = tid; i < 2048; i += THREADS) picked[i] = 0;
    __syncthreads();
    int bad = 0;
    for (int j = tid; j < K; j += THREADS) {
        const int t = sig[j];
        if (t < 0 || t >= N) { bad = 1; continue; }
        const uint32_t bit = 1u << (t & 31);
        if (atomicOr(&picked[t >> 5], bit) & bit) bad = 1;
    }
    if (bad) atomicAdd(&a.status[NGC_STATUS_BAD_SIGMA], 1);
    float smax = -INFINITY, neg_smin = -INFINITY;   // over the unmasked entries
    for (int t = tid; t < N; t += THREADS) {
        float x = row[t];
        if (x == x) smax = fmaxf(smax, x);
        if (x > -INFINITY) neg_smin = fmaxf(neg_smin, -x);
    }
    block_max2_f<THREADS>(smax, neg_smin, fmisc);   // barriers also publish `picked`
    // logits spanning more than NGC_WIDE_SPREAD: wide-range arithmetic (ngc_logsum.h); workgroup-uniform
    const bool wide = smax > -INFINITY && smax + neg_smin > NGC_WIDE_SPREAD;
    if (smax == -INFINITY) smax = 0.f;          // every entry masked: all weights are 0
    float unpicked = 0.f;
    LogSum unpicked_w = ls_empty();
    for (int t = tid; t < N; t += THREADS) {
        if (picked[t >> 5] & (1u << (t & 31))) continue;
        float x = row[t];
        if (x != x) x = -INFINITY;
        if (wide) unpicked_w = ls_add_term(unpicked_w, x);   // that route works on the logits as they came
        else unpicked += expf(x - smax);
    }
    const int chunk = (K + THREADS - 1) / THREADS;
    const int nchunks = (K + chunk - 1) / chunk;
    const int cidx = nchunks - 1 - tid;
    const int j_lo = cidx * chunk;
    const int j_hi = (cidx >= 0) ? ((j_lo + chunk < K) ? j_lo + chunk : K) : 0;
    auto logit_of = [&](int j) {
        int t = sig[j];
        t = t < 0 ? 0 : (t >= N ? N - 1 : t);
        float x = row[t];
        return (x != x) ? -INFINITY : x;
    };
    // When they fit, the picked items' terms are gathered into LDS first (all loads in flight at once), so
    // that the serial chunk loops do not wait for one gather after another.
    const bool use_stage = K <= a.stage_cap;
    const float shift = wide ? 0.f : smax;
    if (use_stage) {
        for (int j = tid; j < K; j += THREADS) staged[j] = logit_of(j) - shift;
        __syncthreads();
    }
    auto term = [&](int j) { return use_stage ? staged[j] : logit_of(j) - shift; };
    if (wide) {
        const LogSum Uw = block_sum_ls<THREADS>(unpicked_w, fmisc);
        const float lpw = sigma_logprob_wide<THREADS>(term, K, Uw, fmisc);
        if (tid == 0) a.logp_out[seg] = lpw;
        return;
    }
    const float U = block_sum_f<THREADS>(unpicked, fmisc);
    float mass = 0.f;
    if (cidx >= 0)
        for (int j = j_lo; j < j_hi; ++j) mass += expf(term(j));
    float total_mass;
    const float after = block_excl_scan_f<THREADS>(mass, fmisc, &total_mass);
    float acc = 0.f;
    if (cidx >= 0) {
        float R = U + after;
        for (int j = j_hi - 1; j >= j_lo; --j) {
            const float d = term(j);
            R += expf(d);
            acc += (d == -INFINITY) ? -INFINITY : d - logf(R);   // a masked pick: probability 0
        }
    }
    const float lp = block_sum_f<THREADS>(acc, fmisc);
    if (tid == 0) a.logp_out[seg] = lp;
}

// ------------------------------------------ gradient of the log-prob ------
//
// d log p / d s_t = 1[t in sigma] - e_t * C_{r(t)},  C_r = sum_{j <= r} 1 / R_j,
// r(t) = position of t in sigma (K if t was never picked), with e_t and R_j as
// in the forward form.  One reverse scan gives R_j, one forward scan of 1/R_j
// gives C_r; 1/R_j lives in LDS between the two.

struct LogprobBwdArgs {
    const float *logits;
    const int32_t *n_items;
    const int32_t *sigma;
    const int32_t *keep;
    const float *gout;     // upstream weight per segment, or nullptr for 1
    float *grad_out;
    int32_t *status;
    int64_t logit_stride;
    int sigma_stride;
    int keep_cap;
};

template <int THREADS>
__global__ __launch_bounds__(THREADS) void subset_logprob_backward_kernel(LogprobBwdArgs a)
{
    extern __shared__ float inv_r[];          // keep_cap floats
    __shared__ uint32_t picked[2048];
    __shared__ float fmisc[32];
    const int tid = threadIdx.x;
    const int seg = blockIdx.x;
    int N = a.n_items[seg];
    N = N < 0 ? 0 : (N > 65536 ? 65536 : N);
    int K = a.keep[seg];
    {
        const int lim = N < a.keep_cap ? N : a.keep_cap;
        if (K < 0 || K > lim) {
            if (tid == 0) atomicAdd(&a.status[NGC_STATUS_KEEP_CLAMPED], 1);
            K = K < 0 ? 0 : lim;
        }
    }
    const float *row = a.logits + (size_t)seg * a.logit_stride;
    float *grow = a.grad_out + (size_t)seg * a.logit_stride;
    const int32_t *sig = a.sigma + (size_t)seg * a.sigma_stride;
    const float g = a.gout ? a.gout[seg] : 1.0f;
    if (K == 0) {
        for (int t = tid; t < N; t += THREADS) grow[t] = 0.f;
        return;
    }
    for (int i = tid; i < 2048; i += THREADS) picked[i] = 0;
    __syncthreads();
    int bad = 0;
    for (int j = tid; j < K; j += THREADS) {
        const int t = sig[j];
        if (t < 0 || t >= N) { bad = 1; continue; }
        const uint32_t bit = 1u << (t & 31);
        if (atomicOr(&picked[t >> 5], bit) & bit) bad = 1;
    }
    if (bad) atomicAdd(&a.status[NGC_STATUS_BAD_SIGMA], 1);
    float smax = -INFINITY, neg_smin = -INFINITY;   // over the unmasked entries
    for (int t = tid; t < N; t += THREADS) {
        const float x = row[t];
        if (x == x) smax = fmaxf(smax, x);
        if (x > -INFINITY) neg_smin = fmaxf(neg_smin, -x);
    }
    block_max2_f<THREADS>(smax, neg_smin, fmisc);
    const int chunk = (K + THREADS - 1) / THREADS;
    const int nchunks = (K + chunk - 1) / chunk;
    if (smax > -INFINITY && smax + neg_smin > NGC_WIDE_SPREAD) {
        // Logits spanning more than NGC_WIDE_SPREAD (workgroup-uniform): the same two scans in the wide-range
        // arithmetic of ngc_logsum.h.  LDS holds, per pick, first d_j = s_j - max, then -log R_j, then log C_j;
        // e_t C_r = exp(d_t + log C_r) is a sum of ratios e_t / R_j <= 1 and never leaves fp32's range.
        auto d_of = [&](int t) {
            const float x = row[t];
            return (x != x) ? -INFINITY : x - smax;
        };
        LogSum uw = ls_empty();
        for (int t = tid; t < N; t += THREADS)
            if (!(picked[t >> 5] & (1u << (t & 31)))) uw = ls_add_term(uw, d_of(t));
        const LogSum Uw = block_sum_ls<THREADS>(uw, fmisc);
        for (int j = tid; j < K; j += THREADS) {
            int t = sig[j];
            t = t < 0 ? 0 : (t >= N ? N - 1 : t);
            inv_r[j] = d_of(t);
        }
        __syncthreads();
        {   // reverse pass: thread 0 owns the last chunk; d -> -log R in place
            const int cidx = nchunks - 1 - tid;
            const int j_lo = cidx * chunk;
            const int j_hi = (cidx >= 0) ? ((j_lo + chunk < K) ? j_lo + chunk : K) : 0;
            LogSum mass = ls_empty();
            if (cidx >= 0)
                for (int j = j_lo; j < j_hi; ++j) mass = ls_add_term(mass, inv_r[j]);
            LogSum total;
            const LogSum after = block_excl_scan_ls<THREADS>(mass, fmisc, &total);
            if (cidx >= 0) {
                LogSum R = ls_add(Uw, after);
                for (int j = j_hi - 1; j >= j_lo; --j) {
                    R = ls_add_term(R, inv_r[j]);
                    inv_r[j] = -ls_log(R);
                }
            }
        }
        __syncthreads();
        LogSum c_all;
        {   // forward pass: thread i owns chunk i; -log R -> log C in place
            const int j_lo = tid * chunk;
            const int j_hi = (tid < nchunks) ? ((j_lo + chunk < K) ? j_lo + chunk : K) : j_lo;
            LogSum part = ls_empty();
            for (int j = j_lo; j < j_hi; ++j) part = ls_add_term(part, inv_r[j]);
            LogSum C = block_excl_scan_ls<THREADS>(part, fmisc, &c_all);
            for (int j = j_lo; j < j_hi; ++j) {
                C = ls_add_term(C, inv_r[j]);
                inv_r[j] = ls_log(C);
            }
        }
        __syncthreads();
        const float log_c_all = ls_log(c_all);
        for (int j = tid; j < K; j += THREADS) {
            const int t = sig[j];
            if (t >= 0 && t < N) grow[t] = g * (1.0f - expf(d_of(t) + inv_r[j]));
        }
        for (int t = tid; t < N; t += THREADS)
            if (!(picked[t >> 5] & (1u << (t & 31)))) grow[t] = -g * expf(d_of(t) + log_c_all);
        return;
    }
    float unpicked = 0.f;
    for (int t = tid; t < N; t += THREADS) {
        if (picked[t >> 5] & (1u << (t & 31))) continue;
        float x = row[t];
        if (x != x) x = -INFINITY;
        unpicked += expf(x - smax);
    }
    const float U = block_sum_f<THREADS>(unpicked, fmisc);
    auto mass_of = [&](int j) {
        int t = sig[j];
        t = t < 0 ? 0 : (t >= N ? N - 1 : t);
        const float x = row[t];
        return (x != x) ? 0.f : expf(x - smax);
    };
    // The masses of the picked items are gathered into LDS first, all loads in flight at once; the two
    // scans then run on LDS and never wait for a gather inside their serial chunk loops.
    for (int j = tid; j < K; j += THREADS) inv_r[j] = mass_of(j);
    __syncthreads();
    // reverse pass: thread 0 owns the last chunk; mass -> 1 / R in place
    {
        const int cidx = nchunks - 1 - tid;
        const int j_lo = cidx * chunk;
        const int j_hi = (cidx >= 0) ? ((j_lo + chunk < K) ? j_lo + chunk : K) : 0;
        float mass = 0.f;
        if (cidx >= 0)
            for (int j = j_lo; j < j_hi; ++j) mass += inv_r[j];
        float total;
        const float after = block_excl_scan_f<THREADS>(mass, fmisc, &total);
        if (cidx >= 0) {
            float R = U + after;
            for (int j = j_hi - 1; j >= j_lo; --j) {
                R += inv_r[j];
                inv_r[j] = 1.0f / R;
            }
        }
    }
    __syncthreads();
    // forward pass: thread i owns chunk i; 1 / R -> C in place
    float c_all;
    {
        const int j_lo = tid * chunk;
        const int j_hi = (tid < nchunks) ? ((j_lo + chunk < K) ? j_lo + chunk : K) : j_lo;
        float part = 0.f;
        for (int j = j_lo; j < j_hi; ++j) part += inv_r[j];
        const float before = block_excl_scan_f<THREADS>(part, fmisc, &c_all);
        float C = before;
        for (int j = j_lo; j < j_hi; ++j) {
            C += inv_r[j];
            inv_r[j] = C;
        }
    }
    __syncthreads();
    for (int j = tid; j < K; j += THREADS) {
        const int t = sig[j];
        if (t >= 0 && t < N) grow[t] = g * (1.0f - mass_of(j) * inv_r[j]);
    }
    for (int t = tid; t < N; t += THREADS) {
        if (picked[t >> 5] & (1u << (t & 31))) continue;
        float x = row[t];
        const float e = (x != x) ? 0.f : expf(x - smax);
        grow[t] = -g * e * c_all;
    }
}

// ------------------------------------------- eviction loss (Eq. 4) --------
//
// L^l = -(1/P) sum_prompts (1/G) sum_{i in prompt} A_i (1/n_i) sum_{t < n_i} sum_h logp[t][l][i][h],
// A_i = r_i - mean of r over the G rollouts of the prompt, n_i = rounds that fired for rollout i.
// One workgroup per layer; advantages and 1/n_i in LDS; fp64 accumulation in a fixed order (the
// advantages of a prompt sum to zero, so the terms cancel heavily).  Also writes d loss / d logp,
// the upstream weights of subset_logprob_backward_kernel.

struct LmemArgs {
    const float *logp;     // [R][L][B][H]
    const int32_t *rounds; // [B]
    const float *reward;   // [B]
    float *adv_out;        // [B] or nullptr
    float *loss_layer;     // [L]
    float *gout;           // [R][L][B][H] or nullptr
    int R, L, B, H, group;
};

constexpr int LMEM_THREADS = 256;
constexpr int LMEM_MAX_B = 8192;

__global__ __launch_bounds__(LMEM_THREADS) void lmem_layer_kernel(LmemArgs a)
{
    __shared__ float weight[LMEM_MAX_B];      // A_i / n_i (0 when no round fired)
    __shared__ int nrounds[LMEM_MAX_B];
    __shared__ double red[LMEM_THREADS];
    const int l = blockIdx.x, tid = threadIdx.x;
    for (int i = tid; i < a.B; i += LMEM_THREADS) {
        const int g0 = (i / a.group) * a.group;
        double mean = 0.0;
        for (int j = 0; j < a.group; ++j) mean += (double)a.reward[g0 + j];
        mean /= (double)a.group;
        const double adv = (double)a.reward[i] - mean;
        int n = a.rounds[i];
        n = n < 0 ? 0 : (n > a.R ? a.R : n);
        nrounds[i] = n;
        weight[i] = n > 0 ? (float)(adv / (double)n) : 0.f;
        if (l == 0 && a.adv_out) a.adv_out[i] = (float)adv;
    }
    __syncthreads();
    const int BH = a.B * a.H;
    double acc = 0.0;
    for (int t = 0; t < a.R; ++t) {
        const size_t base = ((size_t)t * a.L + l) * BH;
        for (int e = tid; e < BH; e += LMEM_THREADS) {
            const int i = e / a.H;
            const bool live = t < nrounds[i];
            if (live) acc += (double)a.logp[base + e] * (double)weight[i];
            if (a.gout) a.gout[base + e] = live ? -weight[i] / (float)a.B : 0.f;
        }
    }
    red[tid] = acc;
    __syncthreads();
    for (int s = LMEM_THREADS / 2; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) a.loss_layer[l] = (float)(-red[0] / (double)a.B);
}

__global__ void lmem_total_kernel(const float *loss_layer, int L, float *loss)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        double s = 0.0;
        for (int l = 0; l < L; ++l) s += (double)loss_layer[l];
        *loss = (float)s;
    }
}

// --------------------------------------------------------- compaction -----
//
// In place: the row that ends at slot j comes from a slot >= j, and once one
// kept row has moved every later one moves too (the kept list is ascending).
// A workgroup walks the rows from the first one that moves (row_start) to the
// end in tiles of TILE_ROWS destination rows.  The stores of a tile may only
// follow a workgroup barrier that every wave reached after issuing its loads of
// that tile (a row of the tile can be the source of another row of the same
// tile); they never touch a row that a later tile still has to read (the
// sources of tile i+1 lie at or beyond its first row), and earlier tiles are
// done with their reads.  So the loop is software-pipelined over two register
// buffers: after the barrier of tile i the loads of tile i+1 are issued, then
// the index fetches of tile i+2, then the stores of tile i.  Every memory
// operation inside the loop is unconditional (indices are clamped to the last
// row, so a tile past the end re-reads rows that exist; full tiles store all
// their rows), which lets the wait before the stores leave the younger loads in
// flight: loads, index fetches and stores of three tiles overlap.  Only the
// last, partial tile is stored under a row test.  16-byte accesses, one full
// row per ROW_BYTES/16 consecutive lanes, K and V together; all of them carry
// the nontemporal hint (every row is touched once).  Offsets inside a segment
// are 32-bit (the host checks cap * ROW_BYTES < 2^31).

template <int ROW_BYTES, int THREADS, int UNROLL>
__device__ __forceinline__ void compact_kv_inplace(unsigned char *kbase, unsigned char *vbase,
                                                   const int32_t *kept, int rows_new, int row_start, int block)
{
    constexpr int PIECES = ROW_BYTES / 16;           // 16-byte pieces per row
    constexpr int ROWS_PER_STEP = THREADS / PIECES;  // rows covered by one load per thread
    constexpr int TILE_ROWS = ROWS_PER_STEP * UNROLL;
    const int rsub = threadIdx.x / PIECES;
    const uint32_t col = (uint32_t)(threadIdx.x % PIECES) * 16u;
    const int last = rows_new - 1;
    if (row_start >= rows_new) return;   // workgroup-uniform

    // source rows of this thread's rows of a tile; rows past the end take the last row's source
    auto sources = [&](int tile, int (&src)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            int r = tile + u * ROWS_PER_STEP + rsub;
            r = r < last ? r : last;
            const int item = r / block;
            src[u] = kept[item] * block + (r - item * block);
        }
    };
    auto load = [&](const int (&src)[UNROLL], u32x4 (&kb)[UNROLL], u32x4 (&vb)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t off = (uint32_t)src[u] * ROW_BYTES + col;
            kb[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kbase + off));
            vb[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vbase + off));
        }
    };
    auto store_full = [&](int tile, const u32x4 (&kb)[UNROLL], const u32x4 (&vb)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t off = (uint32_t)(tile + u * ROWS_PER_STEP + rsub) * ROW_BYTES + col;
            __builtin_nontemporal_store(kb[u], reinterpret_cast<u32x4 *>(kbase + off));
            __builtin_nontemporal_store(vb[u], reinterpret_cast<u32x4 *>(vbase + off));
        }
    };
    auto store_tail = [&](int tile, const u32x4 (&kb)[UNROLL], const u32x4 (&vb)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int r = tile + u * ROWS_PER_STEP + rsub;
            if (r < rows_new) {
                const uint32_t off = (uint32_t)r * ROW_BYTES + col;
                __builtin_nontemporal_store(kb[u], reinterpret_cast<u32x4 *>(kbase + off));
                __builtin_nontemporal_store(vb[u], reinterpret_cast<u32x4 *>(vbase + off));
            }
        }
    };

    int src[UNROLL];
    int tile = row_start;
    u32x4 ka[UNROLL], va[UNROLL], kb[UNROLL], vb[UNROLL];
    sources(tile, src);
    load(src, ka, va);
    sources(tile + TILE_ROWS, src);
    // one copy of the step per buffer, so that each buffer is named by constants and stays in registers
    while (true) {
        __syncthreads();                       // every wave has issued its loads of `tile`
        if (tile + TILE_ROWS > rows_new) { store_tail(tile, ka, va); break; }
        load(src, kb, vb);                     // tile + 1
        sources(tile + 2 * TILE_ROWS, src);    // tile + 2
        store_full(tile, ka, va);
        tile += TILE_ROWS;
        __syncthreads();
        if (tile + TILE_ROWS > rows_new) { store_tail(tile, kb, vb); break; }
        load(src, ka, va);
        sources(tile + 2 * TILE_ROWS, src);
        store_full(tile, kb, vb);
        tile += TILE_ROWS;
    }
}

__device__ __forceinline__ int source_row(const int32_t *kept, int r, int block)
{
    if (block == 1) return kept[r];
    const int item = r / block;
    return kept[item] * block + (r - item * block);
}

template <int THREADS>
__device__ __forceinline__ void compact_pos_inplace(int32_t *pos, const int32_t *kept, int rows_new,
                                                    int row_start, int block)
{
    constexpr int TILE = 4 * THREADS;
    for (int tile = (row_start / TILE) * TILE; tile < rows_new; tile += TILE) {
        int32_t val[4];
        bool moves[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = tile + u * THREADS + threadIdx.x;
            const int s = (r < rows_new) ? source_row(kept, r, block) : r;
            moves[u] = (s != r);
            val[u] = 0;
            if (moves[u]) val[u] = pos[s];
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (moves[u]) pos[tile + u * THREADS + threadIdx.x] = val[u];
    }
}

// ------------------------------------------------- pooled-heads mode ------
//
// One selection problem per (layer, sequence): the items of all its KV heads
// compete for one budget, so heads whose logits are larger keep more rows.
// Item order (for ties and for the sampled sequence) is (head, row); the noise
// of item (head, row) is the one the per-head mode draws for it.  Up to
// Hkv * cap = 65536 items: their key codes live in a workspace in global
// memory (read in order by the select passes), the kept items' codes, logits
// and item indices in three dense arrays next to them (K entries each, served
// by the L2 cache to the sort and to the log-probability), the index buffers
// of the sort in LDS.  Select and sort are the
// shared routines of ngc_select.h.

constexpr int POOL_THREADS = 1024;
constexpr int POOL_MAX_HEADS = 16;
// misc slots of the pooled kernel
constexpr int PM_N = 40;      // rows per head        [40, 56)
constexpr int PM_OFF = 56;    // item offset per head [56, 73)
constexpr int PM_BASE = 73;   // kept slots before each head [73, 90)

template <int ROW_BYTES>
__global__ __launch_bounds__(POOL_THREADS) void evict_pooled_kernel(SelectArgs a)
{
    constexpr int THREADS = POOL_THREADS;
    constexpr int NW = THREADS / NGC_WAVE;
    constexpr int HIST = (SEL_BINS > SORT_BINS * NW) ? SEL_BINS : SORT_BINS * NW;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint32_t *hist = reinterpret_cast<uint32_t *>(smem_raw);
    int *misc = reinterpret_cast<int *>(hist + HIST);   // 128 ints
    uint16_t *idxA = reinterpret_cast<uint16_t *>(misc + 128);
    uint16_t *idxB = idxA + a.keep_cap;
    float *fmisc = reinterpret_cast<float *>(misc);

    const int tid = threadIdx.x, lane = lane_id(), wv = wave_id();
    const int Hkv = a.g.Hkv, cap = a.g.cap;
    const int lb = a.seg0 / Hkv + blockIdx.x;     // layer * B + sequence
    const int l = lb / a.g.B, b = lb - l * a.g.B;
    const int seg_first = lb * Hkv;
    // per (layer, sequence): [codes of all items][codes | logits | item indices of the kept items]
    uint32_t *code = a.pool_codes + (size_t)lb * Hkv * cap * 4;
    uint32_t *kcode = code + (size_t)Hkv * cap;
    float *klogit = reinterpret_cast<float *>(kcode + (size_t)Hkv * cap);
    uint16_t *items = reinterpret_cast<uint16_t *>(klogit + (size_t)Hkv * cap);

    // ---- 0. geometry of the pooled item space ------------------------------
    if (tid == 0) {
        int off = 0, ktot = 0;
        for (int h = 0; h < Hkv; ++h) {
            int n = a.len[seg_first + h];
            if (n < 0 || n > cap) {
                atomicAdd(&a.status[NGC_STATUS_LEN_CLAMPED], 1);
                n = n < 0 ? 0 : cap;
            }
            int kh = a.keep[seg_first + h];
            if (kh < 0) { atomicAdd(&a.status[NGC_STATUS_KEEP_CLAMPED], 1); kh = 0; }
            misc[PM_N + h] = n;
            misc[PM_OFF + h] = off;
            off += n;
            ktot += kh;
        }
        misc[PM_OFF + Hkv] = off;
        int lim = off < a.keep_cap ? off : a.keep_cap;
        if (ktot > lim) {
            atomicAdd(&a.status[NGC_STATUS_KEEP_CLAMPED], 1);
            ktot = lim;
        }
        misc[MISC_KEPT] = ktot;
    }
    __syncthreads();
    const int N = misc[PM_OFF + Hkv];
    const int K = misc[MISC_KEPT];
    const bool want_logp = a.logp_out != nullptr;
    const bool want_sort = want_logp || a.sigma_out != nullptr;
    auto head_of = [&](int i) {
        int h = 0;
        while (h + 1 < Hkv && i >= misc[PM_OFF + h + 1]) ++h;
        return h;
    };
    if (K == 0) {
        if (tid < Hkv) {
            if (a.k) a.len_out[seg_first + tid] = 0;
            if (want_logp) a.logp_out[seg_first + tid] = 0.f;
        }
        return;
    }

    // ---- 1. keys (and the first histogram of the radix select) -------------
    for (int i = tid; i < SEL_BINS; i += THREADS) hist[i] = 0;
    __syncthreads();
    float smax = -INFINITY, neg_smin = -INFINITY;   // over the unmasked entries
    uint32_t cmax = 0;
    for (int h = 0; h < Hkv; ++h) {
        const int n = misc[PM_N + h], off = misc[PM_OFF + h];
        const float *row = a.logits + (size_t)(seg_first + h) * cap;
        for (int quad = tid; 4 * quad < n; quad += THREADS) {
            float s[4], key[4];
            keys_of_quad(row, n, quad, a.na, l, b, h, s, key);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (4 * quad + i < n) {
                    const uint32_t c = ordered_code(key[i]);
                    code[off + 4 * quad + i] = c;
                    atomicAdd(&hist[c >> 21], 1u);
                    cmax = c > cmax ? c : cmax;
                    smax = fmaxf(smax, s[i]);
                    if (s[i] > -INFINITY) neg_smin = fmaxf(neg_smin, -s[i]);
                }
        }
    }
    bool wide = false;   // logits spanning more than NGC_WIDE_SPREAD: wide-range arithmetic for Eq. 2
    if (want_logp) {
        block_max2_f<THREADS>(smax, neg_smin, fmisc);
        wide = smax > -INFINITY && smax + neg_smin > NGC_WIDE_SPREAD;
        if (smax == -INFINITY) smax = 0.f;
    }
    if (want_sort) cmax = block_max_u<THREADS>(cmax, reinterpret_cast<uint32_t *>(misc));

    // ---- 2. radix select (the first histogram was accumulated with the keys) --
    int need;
    __syncthreads();   // publishes the codes and the histogram of step 1
    const uint32_t thr = radix_select_kth<THREADS>([&](int t) { return code[t]; }, N, K, hist, misc, need, true);

    // ---- 3. kept items, ascending in (head, row) order ----------------------
    // Slot j of the kept list gets its item index (items[j]) and its code (kcode[j]) in two dense arrays next to
    // the codes, so that everything after this step works on K entries read in order or from the L2 cache
    // instead of gathering from the N codes.
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
    float unpicked = 0.f;
    LogSum unpicked_w = ls_empty();
    for (int t0 = w_begin; t0 < w_end; t0 += NGC_WAVE) {
        const int t = t0 + lane;
        const bool in = t < w_end;
        const uint32_t u = in ? code[t] : 0u;
        const bool is_gt = in && u > thr, is_eq = in && u == thr;
        const uint64_t bgt = __ballot(is_gt), beq = __ballot(is_eq);
        const int gt_before = gt_base + popc_below(bgt);
        const int eq_before = eq_base + popc_below(beq);
        const bool sel = is_gt || (is_eq && eq_before < need);
        if (in && (want_logp || sel)) {
            float x = 0.f;
            if (want_logp) {
                const int h = head_of(t);
                x = a.logits[(size_t)(seg_first + h) * cap + (t - misc[PM_OFF + h])];
                if (x != x) x = -INFINITY;
            }
            if (sel) {
                const int slot = gt_before + (eq_before < need ? eq_before : need);
                items[slot] = (uint16_t)t;
                kcode[slot] = u;
                klogit[slot] = x;
                idxA[slot] = (uint16_t)slot;
            } else if (wide) {
                unpicked_w = ls_add_term(unpicked_w, x);
            } else {
                unpicked += expf(x - smax);
            }
        }
        gt_base += __popcll(bgt);
        eq_base += __popcll(beq);
    }
    __syncthreads();   // items, kcode (global, this workgroup's own) and idxA are complete
    // kept slots before each head: first slot whose item lies at or beyond the head's offset
    if (tid <= Hkv) {
        const int target = misc[PM_OFF + tid];
        int lo = 0, hi = K;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if ((int)items[mid] < target) lo = mid + 1; else hi = mid;
        }
        misc[PM_BASE + tid] = lo;
    }
    __syncthreads();
    auto head_of_slot = [&](int j) {
        int h = 0;
        while (h + 1 < Hkv && j >= misc[PM_BASE + h + 1]) ++h;
        return h;
    };
    for (int j = tid; j < K; j += THREADS) {
        const int h = head_of_slot(j);
        const int slot = j - misc[PM_BASE + h];
        if (slot < a.max_keep) a.kept_out[(size_t)(seg_first + h) * a.max_keep + slot] = (int)items[j] - misc[PM_OFF + h];
    }
    if (tid < Hkv && misc[PM_BASE + tid + 1] - misc[PM_BASE + tid] > a.max_keep)
        atomicAdd(&a.status[NGC_STATUS_KEEP_CLAMPED], 1);

    if (want_sort) {
        // ---- 4. sigma: the slots sorted by descending code ---------------------
        const uint16_t *src = sort_by_code_desc<THREADS>([&](uint16_t j) { return kcode[j]; }, K, cmax, thr, idxA, idxB,
                                                         hist, misc);
        auto logit_of_slot = [&](int j) { return klogit[j]; };
        if (a.sigma_out) {
            // the pooled sequence occupies the Hkv rows of this (layer, sequence) back to back
            int32_t *sig_row = a.sigma_out + (size_t)seg_first * a.max_keep;
            const int room = Hkv * a.max_keep;
            for (int j = tid; j < K && j < room; j += THREADS) {
                const int slot = src[j], h = head_of_slot(slot);
                sig_row[j] = h * cap + ((int)items[slot] - misc[PM_OFF + h]);
            }
        }
        if (want_logp) {
            // ---- 5. log-probability of the pooled sequence -------------------
            if (wide) {
                const LogSum Uw = block_sum_ls<THREADS>(unpicked_w, fmisc);
                const float lpw = sigma_logprob_wide<THREADS>([&](int j) { return logit_of_slot(src[j]); }, K, Uw,
                                                              fmisc);
                if (tid < Hkv) a.logp_out[seg_first + tid] = (tid == 0) ? lpw : 0.f;
            } else {
                const float U = block_sum_f<THREADS>(unpicked, fmisc);
                const int chunk = (K + THREADS - 1) / THREADS;
                const int nchunks = (K + chunk - 1) / chunk;
                const int cidx = nchunks - 1 - tid;
                const int j_lo = cidx * chunk;
                const int j_hi = (cidx >= 0) ? ((j_lo + chunk < K) ? j_lo + chunk : K) : 0;
                float mass = 0.f;
                if (cidx >= 0)
                    for (int j = j_lo; j < j_hi; ++j) mass += expf(logit_of_slot(src[j]) - smax);
                float total_mass;
                const float after = block_excl_scan_f<THREADS>(mass, fmisc, &total_mass);
                float acc = 0.f;
                if (cidx >= 0) {
                    float R = U + after;
                    for (int j = j_hi - 1; j >= j_lo; --j) {
                        const float d = logit_of_slot(src[j]) - smax;
                        R += expf(d);
                        acc += (d == -INFINITY) ? -INFINITY : d - logf(R);
                    }
                }
                const float lp = block_sum_f<THREADS>(acc, fmisc);
                if (tid < Hkv) a.logp_out[seg_first + tid] = (tid == 0) ? lp : 0.f;
            }
        }
    }
    if (a.k == nullptr) return;

    // ---- 6. per-head compaction ---------------------------------------------
    __syncthreads();   // kept_out of this workgroup is complete and visible
    for (int h = 0; h < Hkv; ++h) {
        int Kh = misc[PM_BASE + h + 1] - misc[PM_BASE + h];
        Kh = Kh < a.max_keep ? Kh : a.max_keep;
        const size_t seg_off = (size_t)(seg_first + h) * cap * ROW_BYTES;
        const int32_t *kept = a.kept_out + (size_t)(seg_first + h) * a.max_keep;
        compact_kv_inplace<ROW_BYTES, THREADS, 4>(reinterpret_cast<unsigned char *>(a.k) + seg_off,
                                                  reinterpret_cast<unsigned char *>(a.v) + seg_off,
                                                  kept, Kh, 0, 1);
        if (a.pos) compact_pos_inplace<THREADS>(a.pos + (size_t)(seg_first + h) * cap, kept, Kh, 0, 1);
        if (tid == 0) a.len_out[seg_first + h] = Kh;
    }
}

// One segment at a time per workgroup: sample, score, then move the survivors.  While a workgroup is in its
// (ALU/LDS bound) selection phase, the other workgroups of the grid keep the memory system busy with their
// compaction phase.
template <int THREADS, int ROW_BYTES, int UNROLL>
__device__ __forceinline__ void evict_segment(const SelectArgs &a, int seg, unsigned char *smem_raw, int *misc)
{
    select_segment<THREADS, ROW_BYTES>(a, seg, smem_raw);
    if (a.k == nullptr) return;   // selection only

    if (threadIdx.x == 0) misc[MISC_FIRST] = 0x7FFFFFFF;
    __syncthreads();   // publishes misc[] and this workgroup's kept_out writes
    const int K = misc[MISC_KEPT];
    const int rows_new = misc[MISC_ROWS];
    const int32_t *kept = a.kept_out + (size_t)seg * a.max_keep;
    if (a.unordered) {   // rows were moved right after the kept list was known
        if (threadIdx.x == 0) a.len_out[seg] = rows_new;
        return;
    }
    // first item that changes place (kept is ascending and kept[j] >= j)
    {
        int mine = K;
        for (int j = threadIdx.x; j < K; j += THREADS)
            if (kept[j] != j) { mine = j; break; }
        if (mine < K) atomicMin(&misc[MISC_FIRST], mine);
    }
    __syncthreads();
    const int first = misc[MISC_FIRST];
    if (first < K) {
        const int row_start = first * a.g.block;
        const size_t seg_off = (size_t)seg * a.g.cap * ROW_BYTES;
        compact_kv_inplace<ROW_BYTES, THREADS, UNROLL>(reinterpret_cast<unsigned char *>(a.k) + seg_off,
                                                       reinterpret_cast<unsigned char *>(a.v) + seg_off,
                                                       kept, rows_new, row_start, a.g.block);
        if (a.pos)
            compact_pos_inplace<THREADS>(a.pos + (size_t)seg * a.g.cap, kept, rows_new, row_start, a.g.block);
    }
    if (threadIdx.x == 0) a.len_out[seg] = rows_new;
}

// The 1024-thread kernel (the host picks it for large segments, see ngc_evict) is persistent: one workgroup fills a CU, the grid
// holds as many workgroups as the chip keeps resident, and each takes the next segment from a counter in the
// workspace until none is left.  (With one workgroup per segment, a CU waited 7 us on average -- 20 us in one
// case out of ten -- between the end of one 1024-thread workgroup and the start of the next, with nothing else
// resident to cover the gap: 6 % of a round at 14336 segments of ~110 us each.)  The last workgroup to finish
// puts the two counters back to zero.  The smaller workgroups keep one workgroup per segment: two to four of
// them share a CU and cover each other's turnaround, and the loop costs them registers (values that do not
// change between segments stay live across the whole body: 69 -> 117 and 101 -> 171 vector registers, one
// workgroup fewer per CU, 6 % slower at 3584 segments of 4096 rows).
//
// Shape of the loop: the fetch by thread 0 sits between two barriers of its own, and the item index is made a
// scalar (it is the same in every lane).  Without the barrier in front of it the compiler merges the
// "thread 0 only" tail of one segment (the store of the new length) with the "thread 0 only" fetch of the
// next into one path, and the lanes that skip it are sent round an inner loop -- back to the barrier and the
// stale item -- that thread 0 never leaves: the grid never ends.
constexpr int PERSISTENT_THREADS = 1024;

template <int THREADS>
__device__ __forceinline__ int next_segment(const SelectArgs &a, int *slot)
{
    __syncthreads();   // every wave is done with the previous segment (its LDS, and the last read of *slot)
    if (threadIdx.x == 0) *slot = atomicAdd(&a.status[WS_QUEUE_NEXT], 1);
    __syncthreads();
    return __builtin_amdgcn_readfirstlane(*slot);
}

template <int THREADS, int ROW_BYTES, int UNROLL>
__global__ __launch_bounds__(THREADS) void evict_kernel(SelectArgs a)
{
    constexpr int NW = THREADS / NGC_WAVE;
    constexpr int HIST = (SEL_BINS > SORT_BINS * NW) ? SEL_BINS : SORT_BINS * NW;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    int *misc = reinterpret_cast<int *>(reinterpret_cast<uint32_t *>(smem_raw) + a.items_cap + HIST);
    if constexpr (THREADS != PERSISTENT_THREADS) {
        evict_segment<THREADS, ROW_BYTES, UNROLL>(a, a.seg0 + (int)blockIdx.x, smem_raw, misc);
    } else {
        __shared__ int next_item;
        for (int item = next_segment<THREADS>(a, &next_item); item < a.nseg;
             item = next_segment<THREADS>(a, &next_item))
            evict_segment<THREADS, ROW_BYTES, UNROLL>(a, a.seg0 + item, smem_raw, misc);
        if (threadIdx.x == 0) {
            const int done = atomicAdd(&a.status[WS_QUEUE_DONE], 1);
            if (done == (int)gridDim.x - 1) {   // every workgroup has taken its last item: nobody reads the counters any more
                __hip_atomic_store(&a.status[WS_QUEUE_NEXT], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&a.status[WS_QUEUE_DONE], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// --------------------------------------------------------- keep counts ----
//
// The fraction rule of Sec. 4.1 evaluated where the lengths live: K = ceil(N * num / den) items of the
// N = ceil(len / block) a segment has, in exact integer arithmetic, at least `min_keep` (and at least 1
// for a non-empty segment), at most N.  Saves the host a read-back of the ragged lengths per round.
__global__ __launch_bounds__(256) void keep_counts_kernel(const int32_t *__restrict__ len, int32_t *__restrict__ keep,
                                                          int seg0, int nseg, int cap, int block,
                                                          int64_t num, int64_t den, int min_keep)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= nseg) return;
    int n = len[seg0 + i];
    n = n < 0 ? 0 : (n > cap ? cap : n);
    const int64_t N = (n + block - 1) / block;
    int64_t K = (N * num + den - 1) / den;
    if (K < min_keep) K = min_keep;
    if (K < 1) K = 1;
    if (K > N) K = N;
    keep[seg0 + i] = (int32_t)K;
}

// -------------------------------------------------------------- append ----

struct AppendArgs {
    void *k;
    void *v;
    int32_t *pos;
    int32_t *len;
    const void *k_new;
    const void *v_new;
    const int32_t *new_pos;
    int32_t *status;
    int seg0;       // first segment of the launch
    int src_seg0;   // segment index that k_new[0] belongs to
    int B, Hkv, cap;
};

// One wave per segment: lanes [0, PIECES) copy the K row, the next PIECES the V row.
template <int ROW_BYTES>
__global__ __launch_bounds__(64) void append_kernel(AppendArgs a)
{
    constexpr int PIECES = ROW_BYTES / 16;
    const int seg = a.seg0 + blockIdx.x;
    const int lane = threadIdx.x;
    const int n = a.len[seg];
    if (n < 0 || n >= a.cap) {
        if (lane == 0) atomicAdd(&a.status[NGC_STATUS_APPEND_FULL], 1);
        return;
    }
    const size_t src_off = (size_t)(seg - a.src_seg0) * ROW_BYTES;
    const size_t dst_off = ((size_t)seg * a.cap + n) * ROW_BYTES;
    if (lane < 2 * PIECES) {
        const bool is_v = lane >= PIECES;
        const int piece = is_v ? lane - PIECES : lane;
        const unsigned char *s = reinterpret_cast<const unsigned char *>(is_v ? a.v_new : a.k_new) + src_off;
        unsigned char *d = reinterpret_cast<unsigned char *>(is_v ? a.v : a.k) + dst_off;
        *reinterpret_cast<uint4 *>(d + piece * 16) = *reinterpret_cast<const uint4 *>(s + piece * 16);
    }
    __syncthreads();
    if (lane == 0) {
        if (a.pos && a.new_pos) a.pos[(size_t)seg * a.cap + n] = a.new_pos[(seg / a.Hkv) % a.B];
        a.len[seg] = n + 1;
    }
}

}  // namespace ngc

// ============================================================ host side ====

using namespace ngc;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_cache(const ngc_cache *c)
{
    if (!c || !c->k || !c->v || !c->len) return NGC_EINVAL;
    if (!aligned16(c->k) || !aligned16(c->v)) return NGC_EINVAL;
    if (c->L <= 0 || c->B <= 0 || c->Hkv <= 0 || c->Hq <= 0 || c->cap <= 0) return NGC_EINVAL;
    if (c->D != 64 && c->D != 128) return NGC_EINVAL;
    if (c->Hq % c->Hkv != 0 || c->Hq / c->Hkv > 16) return NGC_EINVAL;
    if (c->L > 65535 || c->Hkv > 65534) return NGC_EINVAL;   // noise counter packs layer and head in 16 bits each
    return NGC_OK;
}

// The noise counter packs the global layer index into 16 bits.
int check_bases(const ngc_cache *c, const ngc_evict_params *p)
{
    if (p->layer_base < 0 || p->seq_base < 0) return NGC_EINVAL;
    if ((long long)p->layer_base + c->L > 65535) return NGC_EINVAL;
    if ((long long)p->seq_base + c->B > 0x7FFFFFFFLL) return NGC_EINVAL;
    return NGC_OK;
}

int layer_range(const ngc_cache *c, int layer, int *seg0, int *nseg)
{
    if (layer < -1 || layer >= c->L) return NGC_EINVAL;
    const int per_layer = c->B * c->Hkv;
    *seg0 = layer < 0 ? 0 : layer * per_layer;
    *nseg = layer < 0 ? c->L * per_layer : per_layer;
    return NGC_OK;
}

constexpr size_t STATUS_BYTES = NGC_STATUS_WORDS * sizeof(int32_t);

// Grid of a persistent kernel: as many workgroups as the device keeps resident at this workgroup size and LDS
// use (asked of the runtime once per device, kernel and LDS size, then remembered: the query costs tens of
// microseconds of host time; one per CU if the runtime does not say), but no more than there are items.
int resident_workgroups(const void *fn, int threads, size_t lds, int items)
{
    struct Key {
        int dev;
        const void *fn;
        size_t lds;
        bool operator<(const Key &o) const
        {
            return dev != o.dev ? dev < o.dev : (fn != o.fn ? fn < o.fn : lds < o.lds);
        }
    };
    static std::mutex lock;
    static std::map<Key, long long> known;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) dev = 0;
    long long slots;
    {
        std::lock_guard<std::mutex> g(lock);
        const Key key{dev, fn, lds};
        auto it = known.find(key);
        if (it == known.end()) {
            int cus = 0, per_cu = 0;
            if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
                cus = 256;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, threads, lds) != hipSuccess || per_cu <= 0) {
                (void)hipGetLastError();
                per_cu = 1;
            }
            it = known.emplace(key, (long long)cus * per_cu).first;
        }
        slots = it->second;
    }
    return (int)(slots < items ? slots : items);
}

size_t select_lds_bytes(int threads, int items_cap, int keep_cap)
{
    const int nw = threads / 64;
    const int hist = (SEL_BINS > SORT_BINS * nw) ? SEL_BINS : SORT_BINS * nw;
    return (size_t)items_cap * 4 + (size_t)hist * 4 + 64 * 4 + (size_t)keep_cap * 2 * 2;
}

}  // namespace

extern "C" int ngc_perturbed_keys(const ngc_cache *c, int32_t layer, const float *logits,
                                  const ngc_evict_params *p, float *keys_out,
                                  void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_cache(c);
    if (rc) return rc;
    if (!logits || !keys_out || !p || !ws || p->block < 1) return NGC_EINVAL;
    if ((rc = check_bases(c, p)) != NGC_OK) return rc;
    if (ws_bytes < STATUS_BYTES) return NGC_ENOSPC;
    int seg0, nseg;
    rc = layer_range(c, layer, &seg0, &nseg);
    if (rc) return rc;
    SegGeom g{c->B, c->Hkv, c->cap, p->block};
    NoiseArgs na{p->seed, p->round, p->noise_scale, p->share_heads, p->layer_base, p->seq_base};
    hipLaunchKernelGGL(perturbed_keys_kernel, dim3(nseg), dim3(256), 0, (hipStream_t)stream,
                       logits, c->len, keys_out, seg0, g, na, reinterpret_cast<int32_t *>(ws));
    NGC_HIP_CHECK(hipGetLastError());
    return NGC_OK;
}

extern "C" int ngc_evict(const ngc_cache *c, int32_t layer, const float *logits,
                         const int32_t *keep, const ngc_evict_params *p, int32_t max_keep,
                         int32_t *kept_out, int32_t *sigma_out, float *logp_out,
                         void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_cache(c);
    if (rc) return rc;
    if (!logits || !keep || !p || !kept_out || !ws || p->block < 1 || max_keep < 1) return NGC_EINVAL;
    if ((rc = check_bases(c, p)) != NGC_OK) return rc;
    if ((p->flags & NGC_EVICT_UNORDERED) && p->block != 1) return NGC_EUNSUPPORTED;
    if ((long long)c->cap * c->D * 2 > 0x7FFFFFFFLL) return NGC_EUNSUPPORTED;   // 32-bit byte offsets inside a segment
    int seg0, nseg;
    rc = layer_range(c, layer, &seg0, &nseg);
    if (rc) return rc;
    const int nseg_total = c->L * c->B * c->Hkv;
    if (ws_bytes < STATUS_BYTES + (size_t)nseg_total * 8) return NGC_ENOSPC;
    if (!aligned16(ws)) return NGC_EINVAL;

    if (p->flags & NGC_EVICT_POOL_HEADS) {
        // one selection per (layer, sequence) over the items of all its heads
        if (p->block != 1 || (p->flags & NGC_EVICT_UNORDERED)) return NGC_EUNSUPPORTED;
        if (c->Hkv > POOL_MAX_HEADS || (long long)c->Hkv * c->cap > 65536) return NGC_EUNSUPPORTED;
        const size_t codes_off = ngc_workspace_bytes(c, max_keep);
        const size_t codes_bytes = (size_t)c->L * c->B * c->Hkv * c->cap * sizeof(uint32_t) * 4;
        if (ws_bytes < codes_off + codes_bytes) return NGC_ENOSPC;
        long long kc = (long long)c->Hkv * max_keep;
        if (kc > (long long)c->Hkv * c->cap) kc = (long long)c->Hkv * c->cap;
        int keep_cap = (int)((kc + 7) & ~7LL);
        const int hist = (SEL_BINS > SORT_BINS * (POOL_THREADS / 64)) ? SEL_BINS : SORT_BINS * (POOL_THREADS / 64);
        size_t lds = (size_t)hist * 4 + 128 * 4 + (size_t)keep_cap * 2 * 2;
        if (lds > 160 * 1024) {
            // Hkv * max_keep is only an upper bound of what a (layer, sequence) keeps (max_keep has to cover the
            // largest single head); the budget itself is on the device.  The index buffers take what LDS holds;
            // a budget above that is clamped by the kernel and counted in NGC_STATUS_KEEP_CLAMPED.
            keep_cap = (int)(((160 * 1024 - (size_t)hist * 4 - 128 * 4) / 4) & ~7u);
            lds = (size_t)hist * 4 + 128 * 4 + (size_t)keep_cap * 2 * 2;
        }
        SelectArgs sa;
        sa.logits = logits; sa.len = c->len; sa.keep = keep;
        sa.kept_out = kept_out; sa.sigma_out = sigma_out; sa.logp_out = logp_out;
        sa.status = reinterpret_cast<int32_t *>(ws);
        const bool move = !(p->flags & NGC_EVICT_SELECT_ONLY);
        sa.k = move ? c->k : nullptr; sa.v = c->v; sa.pos = c->pos; sa.len_out = c->len;
        sa.unordered = 0;
        sa.seg0 = seg0; sa.max_keep = max_keep; sa.items_cap = 0; sa.keep_cap = keep_cap;
        sa.pool_codes = reinterpret_cast<uint32_t *>(reinterpret_cast<unsigned char *>(ws) + codes_off);
        sa.g = SegGeom{c->B, c->Hkv, c->cap, 1};
        sa.logit_stride = c->cap;
        sa.na = NoiseArgs{p->seed, p->round, p->noise_scale, p->share_heads, p->layer_base, p->seq_base};
        const void *fn = (c->D == 128) ? reinterpret_cast<const void *>(&evict_pooled_kernel<256>)
                                       : reinterpret_cast<const void *>(&evict_pooled_kernel<128>);
        if (lds > 64 * 1024)
            NGC_HIP_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        void *kargs[] = {&sa};
        NGC_HIP_CHECK(hipLaunchKernel(fn, dim3(nseg / c->Hkv), dim3(POOL_THREADS), kargs, lds,
                                      (hipStream_t)stream));
        return NGC_OK;
    }

    const int items_cap = (c->cap + p->block - 1) / p->block;
    if (items_cap > 16384) return NGC_EUNSUPPORTED;
    int keep_cap = max_keep < items_cap ? max_keep : items_cap;
    keep_cap = (keep_cap + 7) & ~7;
    const int items_cap_al = (items_cap + 3) & ~3;
    // Workgroup size and rows in flight per thread, measured on configs 2-4.  A round that moves rows in order
    // is a copy with a selection in front: the copy wants as many bytes in flight per compute unit as registers
    // allow, which is one 1024-thread workgroup per CU from 4097 rows per segment up (the size follows the rows
    // of a segment, not its items: with blocks of rows as items the selection is small and the copy is all there
    // is).  A round that only selects, or fills holes (few rows move), is bound by the selection's ~45 workgroup
    // barriers; two 512-thread workgroups per CU then cover each other's waits, up to the 8192 rows at which two
    // of them still fit in LDS (config 3, selection only: 1.79 -> 1.14 ms, steady-state 1.46 -> 0.84 ms;
    // unordered: 4.54 -> 4.18 and 2.17 -> 1.53 ms).
    const bool move_rows = !(p->flags & NGC_EVICT_SELECT_ONLY);
    const bool copy_bound = move_rows && !(p->flags & NGC_EVICT_UNORDERED);
    const int threads = c->cap > (copy_bound ? 4096 : 8192) ? 1024 : (c->cap > 2048 ? 512 : 256);
    const size_t lds = select_lds_bytes(threads, items_cap_al, keep_cap);
    if (lds > 160 * 1024) return NGC_EUNSUPPORTED;

    int32_t *status = reinterpret_cast<int32_t *>(ws);

    SelectArgs sa;
    sa.logits = logits; sa.len = c->len; sa.keep = keep;
    sa.kept_out = kept_out; sa.sigma_out = sigma_out; sa.logp_out = logp_out;
    sa.status = status;
    sa.k = move_rows ? c->k : nullptr; sa.v = c->v; sa.pos = c->pos; sa.len_out = c->len;
    sa.unordered = (p->flags & NGC_EVICT_UNORDERED) ? 1 : 0;
    sa.pool_codes = nullptr;
    sa.seg0 = seg0; sa.max_keep = max_keep; sa.items_cap = items_cap_al; sa.keep_cap = keep_cap;
    sa.g = SegGeom{c->B, c->Hkv, c->cap, p->block};
    sa.logit_stride = c->cap;
    sa.na = NoiseArgs{p->seed, p->round, p->noise_scale, p->share_heads, p->layer_base, p->seq_base};

    hipStream_t st = (hipStream_t)stream;
    const void *fn;
#define NGC_PICK(T, U) ((c->D == 128) ? reinterpret_cast<const void *>(&evict_kernel<T, 256, U>) \
                                      : reinterpret_cast<const void *>(&evict_kernel<T, 128, U>))
    if (threads == 1024) fn = NGC_PICK(1024, 4);
    else if (threads == 512) fn = NGC_PICK(512, 2);
    else fn = NGC_PICK(256, 4);
#undef NGC_PICK
    if (lds > 64 * 1024)
        NGC_HIP_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    sa.nseg = nseg;
    const int grid = threads == PERSISTENT_THREADS ? resident_workgroups(fn, threads, lds, nseg) : nseg;
    void *kargs[] = {&sa};
    NGC_HIP_CHECK(hipLaunchKernel(fn, dim3(grid), dim3(threads), kargs, lds, st));
    return NGC_OK;
}

extern "C" int ngc_subset_logprob(const float *logits, const int32_t *n_items,
                                  const int32_t *sigma, const int32_t *keep, int32_t nseg,
                                  int64_t logit_stride, int32_t sigma_stride,
                                  float *logp_out, void *ws, size_t ws_bytes, void *stream)
{
    if (!logits || !n_items || !sigma || !keep || !logp_out || !ws) return NGC_EINVAL;
    if (nseg < 0 || logit_stride < 0 || sigma_stride < 0) return NGC_EINVAL;
    if (ws_bytes < STATUS_BYTES) return NGC_ENOSPC;
    if (nseg == 0) return NGC_OK;
    const int stage_cap = sigma_stride < 16384 ? sigma_stride : 16384;     // at most 64 KB of LDS
    LogprobArgs la{logits, n_items, sigma, keep, logp_out, reinterpret_cast<int32_t *>(ws),
                   logit_stride, sigma_stride, stage_cap};
    const size_t lds = (size_t)stage_cap * sizeof(float);
    const void *fn = reinterpret_cast<const void *>(&subset_logprob_kernel<512>);
    if (lds > 48 * 1024)
        NGC_HIP_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    void *kargs[] = {&la};
    NGC_HIP_CHECK(hipLaunchKernel(fn, dim3(nseg), dim3(512), kargs, lds, (hipStream_t)stream));
    return NGC_OK;
}

extern "C" int ngc_subset_logprob_backward(const float *logits, const int32_t *n_items,
                                           const int32_t *sigma, const int32_t *keep, int32_t nseg,
                                           int64_t logit_stride, int32_t sigma_stride, int32_t max_keep,
                                           const float *gout, float *grad_out,
                                           void *ws, size_t ws_bytes, void *stream)
{
    if (!logits || !n_items || !sigma || !keep || !grad_out || !ws) return NGC_EINVAL;
    if (nseg < 0 || logit_stride < 0 || sigma_stride < 0 || max_keep < 1) return NGC_EINVAL;
    if (ws_bytes < STATUS_BYTES) return NGC_ENOSPC;
    if (max_keep > 32768) return NGC_EUNSUPPORTED;
    if (nseg == 0) return NGC_OK;
    LogprobBwdArgs la{logits, n_items, sigma, keep, gout, grad_out, reinterpret_cast<int32_t *>(ws),
                      logit_stride, sigma_stride, max_keep};
    const size_t lds = (size_t)max_keep * sizeof(float);
    const void *fn = reinterpret_cast<const void *>(&subset_logprob_backward_kernel<512>);
    if (lds > 48 * 1024)
        NGC_HIP_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    void *kargs[] = {&la};
    NGC_HIP_CHECK(hipLaunchKernel(fn, dim3(nseg), dim3(512), kargs, lds, (hipStream_t)stream));
    return NGC_OK;
}

extern "C" int ngc_cache_append(const ngc_cache *c, int32_t layer, const void *k_new,
                                const void *v_new, const int32_t *new_pos,
                                void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_cache(c);
    if (rc) return rc;
    if (!k_new || !v_new || !ws || !aligned16(k_new) || !aligned16(v_new)) return NGC_EINVAL;
    if (ws_bytes < STATUS_BYTES) return NGC_ENOSPC;
    int seg0, nseg;
    rc = layer_range(c, layer, &seg0, &nseg);
    if (rc) return rc;
    AppendArgs aa{c->k, c->v, c->pos, c->len, k_new, v_new, new_pos,
                  reinterpret_cast<int32_t *>(ws), seg0, seg0, c->B, c->Hkv, c->cap};
    if (c->D == 128)
        hipLaunchKernelGGL(append_kernel<256>, dim3(nseg), dim3(64), 0, (hipStream_t)stream, aa);
    else
        hipLaunchKernelGGL(append_kernel<128>, dim3(nseg), dim3(64), 0, (hipStream_t)stream, aa);
    NGC_HIP_CHECK(hipGetLastError());
    return NGC_OK;
}

extern "C" int ngc_lmem(const float *logp, const int32_t *rounds, const float *reward,
                        int32_t R, int32_t L, int32_t B, int32_t Hkv, int32_t group,
                        float *adv_out, float *loss_layer, float *loss, float *gout, void *stream)
{
    if (!logp || !rounds || !reward || !loss_layer || !loss) return NGC_EINVAL;
    if (R < 1 || L < 1 || B < 1 || Hkv < 1 || group < 1 || B % group != 0) return NGC_EINVAL;
    if (B > LMEM_MAX_B) return NGC_EUNSUPPORTED;
    LmemArgs la{logp, rounds, reward, adv_out, loss_layer, gout, R, L, B, Hkv, group};
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(lmem_layer_kernel, dim3(L), dim3(LMEM_THREADS), 0, st, la);
    NGC_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(lmem_total_kernel, dim3(1), dim3(64), 0, st, (const float *)loss_layer, (int)L, loss);
    NGC_HIP_CHECK(hipGetLastError());
    return NGC_OK;
}

extern "C" int ngc_keep_counts(const int32_t *len, int32_t seg0, int32_t nseg, int32_t cap, int32_t block,
                               int32_t num, int32_t den, int32_t min_keep, int32_t *keep_out, void *stream)
{
    if (!len || !keep_out) return NGC_EINVAL;
    if (seg0 < 0 || nseg < 0 || cap < 1 || block < 1 || num < 0 || den < 1 || num > den || min_keep < 0) return NGC_EINVAL;
    if (nseg == 0) return NGC_OK;
    hipLaunchKernelGGL(keep_counts_kernel, dim3((nseg + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                       len, keep_out, (int)seg0, (int)nseg, (int)cap, (int)block, (int64_t)num, (int64_t)den, (int)min_keep);
    NGC_HIP_CHECK(hipGetLastError());
    return NGC_OK;
}
