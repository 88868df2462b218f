// Key scoring for the eviction policy on gfx950 (Sec. 4.2 of the paper): the
// attention weights that the w most recent queries put on every cached key,
// averaged over the query heads of a KV head and over the w queries, then
// (optionally) averaged over KV heads and over blocks of consecutive keys.
//
// One workgroup of 4 waves per (layer, sequence, KV head).  The w*G query rows
// are padded to QT tiles of 16 and both passes run on the matrix cores:
//   pass 1  S^T = K Q^T   (queries on lane%16): running max / sum per query row
//   pass 2  S   = Q K^T   (keys on lane%16):    p = 2^(x - m) / l, summed over
//                                               the query rows of each key
// The two orientations use the same operand registers with the MFMA arguments
// swapped.  K is read twice (once per pass); nothing else touches HBM except
// the one fp32 score per key that is written.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/ngc.h"
#include "ngc_device.h"

namespace ngc {

constexpr int SC_WAVES = 4;
constexpr int SC_TILE = 32;

struct ScoreArgs {
    const unsigned char *k;
    const int32_t *len;
    const unsigned char *q;   // bf16 [lb][w][Hq][D]
    const float *lse;         // optional fp32 [lb][w][Hq]: log-sum-exp of every query's scaled scores
    float *psi_out;           // fp32 [seg][cap], one value per key
    int32_t *status;
    int seg0, lb0;
    int w, G, Hkv, cap, causal;
    float scale_log2e;
    // paged layout: k is the pool and a tile's base comes from the page table
    const int32_t *table;   // [seg][max_pages] or nullptr (contiguous layout)
    int max_pages, num_pages, tpp_shift;
};

// Up to three query tiles the kernel fits 168 registers per thread without spilling, i.e. three waves per SIMD
// (three workgroups per CU) instead of the two the compiler settles for by itself; with four tiles it does not.
template <int D, int QT>
__global__ __launch_bounds__(SC_WAVES * 64) __attribute__((amdgpu_waves_per_eu(QT <= 3 ? 3 : 2)))
void score_keys_kernel(ScoreArgs a)
{
    constexpr int ROW_BYTES = D * 2;
    constexpr int KCH = D / 32;
    constexpr int LROW = ROW_BYTES + 16;
    constexpr int K_LOADS = SC_TILE * ROW_BYTES / (64 * 16);
    constexpr int K_PIECES = ROW_BYTES / 16;
    constexpr int K_ROWS_PER_LOAD = 64 / K_PIECES;
    constexpr int WAVE_LDS = SC_TILE * LROW;

    __shared__ __align__(16) unsigned char lds[SC_WAVES * WAVE_LDS];
    __shared__ float red_m[SC_WAVES][QT * 16];
    __shared__ float red_l[SC_WAVES][QT * 16];
    __shared__ float fin_m[QT * 16];
    __shared__ float fin_il[QT * 16];

    const int lane = lane_id(), wv = wave_id();
    const int li = lane & 15, kg = lane >> 4;
    const int seg = a.seg0 + blockIdx.x;
    const int G = a.G, w = a.w, R = w * G;
    int n = a.len[seg];
    if (n < 0 || n > a.cap) {
        if (threadIdx.x == 0) atomicAdd(&a.status[NGC_STATUS_LEN_CLAMPED], 1);
        n = n < 0 ? 0 : a.cap;
    }
    if (n == 0) return;
    const int h = seg % a.Hkv;
    const int lb = seg / a.Hkv - a.lb0;
    const int Hq = a.Hkv * G;
    const unsigned char *kseg = a.table ? a.k : a.k + (size_t)seg * a.cap * ROW_BYTES;
    const int32_t *tab = a.table ? a.table + (size_t)seg * a.max_pages : nullptr;
    float *psi = a.psi_out + (size_t)seg * a.cap;
    const int tiles = (n + SC_TILE - 1) / SC_TILE;
    const int last_row = n - 1;

    // query operands: row r = qt*16 + li  ->  (recent query j = r / G, head g = r % G)
    bf16x8 qop[QT][KCH];
    int vis_q[QT];   // number of rows the query row of this lane can see
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int r = qt * 16 + li;
        const int j = r / G, g = r - j * G;
        const bool ok = r < R;
        int vis = a.causal ? (n - w + j + 1) : n;
        vis = vis > n ? n : vis;
        vis_q[qt] = ok ? (vis > 0 ? vis : 0) : 0;
        const unsigned char *qrow = a.q + (((size_t)lb * w + j) * Hq + (size_t)h * G + g) * ROW_BYTES;
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (ok) v = *reinterpret_cast<const u32x4 *>(qrow + c * 64 + kg * 16);
            qop[qt][c] = __builtin_bit_cast(bf16x8, v);
        }
    }

    unsigned char *wlds = lds + wv * WAVE_LDS;
    u32x4 kbuf[K_LOADS];
    // Unconditional: a tile past the end re-reads the last tile, so that the number of loads in flight is
    // the same on every path and the wait for the current tile never also waits for the prefetch.
    auto load_tile = [&](int tile_raw) {
        const int tile = tile_raw < tiles ? tile_raw : tiles - 1;
        const int row0 = tile * SC_TILE;
        const unsigned char *kt = kseg;
        int first = 0;   // row number at offset 0 of kt
        if (tab) {       // a tile lies inside one page
            int page = tab[tile >> a.tpp_shift];
            page = (page < 0 || page >= a.num_pages) ? 0 : page;
            kt = kseg + (((size_t)page << a.tpp_shift) + (size_t)(tile & ((1 << a.tpp_shift) - 1))) *
                            (SC_TILE * ROW_BYTES);
            first = row0;
        }
#pragma unroll
        for (int r = 0; r < K_LOADS; ++r) {
            int row = row0 + r * K_ROWS_PER_LOAD + lane / K_PIECES;
            row = row < last_row ? row : last_row;
            kbuf[r] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4 *>(kt + (size_t)(row - first) * ROW_BYTES + (lane % K_PIECES) * 16));
        }
    };
    auto stage_tile = [&]() {
#pragma unroll
        for (int r = 0; r < K_LOADS; ++r) {
            const int rl = r * K_ROWS_PER_LOAD + lane / K_PIECES;
            *reinterpret_cast<u32x4 *>(wlds + rl * LROW + (lane % K_PIECES) * 16) = kbuf[r];
        }
    };

    // ------------------------------------------------ pass 1: max and sum ---
    // (skipped when the caller hands over the log-sum-exp that decode attention
    // already computed for these very queries: then K is read only once)
    if (a.lse != nullptr) {
        for (int r = threadIdx.x; r < QT * 16; r += SC_WAVES * 64) {
            float m2 = -INFINITY;
            if (r < R) {
                const int j = r / G, g = r - j * G;
                m2 = a.lse[((size_t)lb * w + j) * Hq + (size_t)h * G + g] * 1.4426950408889634f;
            }
            fin_m[r] = m2;
            fin_il[r] = (m2 > -INFINITY) ? 1.0f : 0.f;
        }
        __syncthreads();
    } else {
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) { m_run[qt] = -INFINITY; l_run[qt] = 0.f; }
    {
        int tile = wv;
        load_tile(tile);
        for (; tile < tiles; tile += SC_WAVES) {
            stage_tile();
            const int row0 = tile * SC_TILE;
            load_tile(tile + SC_WAVES);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_wave_barrier();
            bf16x8 kop[2][KCH];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int c = 0; c < KCH; ++c)
                    kop[mt][c] = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const u32x4 *>(wlds + (mt * 16 + li) * LROW + c * 64 + kg * 16));
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < KCH; ++c) {
                    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[0][c], qop[qt][c], s0, 0, 0, 0);
                    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[1][c], qop[qt][c], s1, 0, 0, 0);
                }
                // lane (q = li, kg): keys row0 + 4kg + r (s0) and row0 + 16 + 4kg + r (s1)
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int t = row0 + ((e < 4) ? (4 * kg + e) : (16 + 4 * kg + e - 4));
                    const float sc = (e < 4) ? s0[e] : s1[e - 4];
                    x[e] = (t < vis_q[qt]) ? sc * a.scale_log2e : -INFINITY;
                }
                float tmax = x[0];
#pragma unroll
                for (int e = 1; e < 8; ++e) tmax = fmaxf(tmax, x[e]);
                tmax = quad_rows_max(tmax);
                const float m_new = fmaxf(m_run[qt], tmax);
                if (m_new > -INFINITY) {
                    float psum = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) psum += fast_exp2(x[e] - m_new);
                    l_run[qt] = l_run[qt] * fast_exp2(m_run[qt] - m_new) + psum;
                    m_run[qt] = m_new;
                }
            }
        }
    }
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        float l = l_run[qt];
        l = quad_rows_sum(l);
        if (kg == 0) { red_m[wv][qt * 16 + li] = m_run[qt]; red_l[wv][qt * 16 + li] = l; }
    }
    __syncthreads();
    for (int r = threadIdx.x; r < QT * 16; r += SC_WAVES * 64) {
        float M = red_m[0][r];
#pragma unroll
        for (int x = 1; x < SC_WAVES; ++x) M = fmaxf(M, red_m[x][r]);
        float L = 0.f;
#pragma unroll
        for (int x = 0; x < SC_WAVES; ++x) {
            const float mw = red_m[x][r];
            L += (mw == -INFINITY) ? 0.f : red_l[x][r] * fast_exp2(mw - M);
        }
        fin_m[r] = M;
        fin_il[r] = (L > 0.f) ? 1.0f / L : 0.f;
    }
    __syncthreads();
    }

    // ------------------------------------- pass 2: probabilities per key ---
    // lane (key = li, kg) holds query rows qt*16 + 4kg + r
    float m_row[QT][4], il_row[QT][4];
    int vis_row[QT][4];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = qt * 16 + 4 * kg + r;
            m_row[qt][r] = fin_m[row];
            il_row[qt][r] = fin_il[row];
            const int j = row / G;
            int vis = a.causal ? (n - w + j + 1) : n;
            vis = vis > n ? n : vis;
            vis_row[qt][r] = (row < R && vis > 0) ? vis : 0;
        }
    const float inv_rows = 1.0f / (float)R;
    {
        int tile = wv;
        load_tile(tile);
        for (; tile < tiles; tile += SC_WAVES) {
            stage_tile();
            const int row0 = tile * SC_TILE;
            load_tile(tile + SC_WAVES);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_wave_barrier();
            bf16x8 kop[2][KCH];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int c = 0; c < KCH; ++c)
                    kop[nt][c] = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const u32x4 *>(wlds + (nt * 16 + li) * LROW + c * 64 + kg * 16));
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const int t = row0 + nt * 16 + li;   // the key of this lane
                float acc = 0.f;
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int c = 0; c < KCH; ++c)
                        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qop[qt][c], kop[nt][c], s, 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (t < vis_row[qt][r])
                            acc += fast_exp2(s[r] * a.scale_log2e - m_row[qt][r]) * il_row[qt][r];
                }
                acc = quad_rows_sum(acc);
                if (kg == 0 && t < n) psi[t] = acc * inv_rows;
            }
        }
    }
}

// Block means and head pooling, in place over the per-key scores: item j of a
// segment becomes the mean of the scores of its rows; with pooling, the mean of
// that over the KV heads of the (layer, sequence) that have item j.  One
// workgroup per (layer, sequence); items are processed in ascending tiles and
// an item only reads rows at or beyond its own index, so reading a tile,
// waiting, then writing it never clobbers what a later tile still reads.
struct ReduceArgs {
    float *scores;      // [lb][Hkv][cap]
    const int32_t *len;
    int lb0_seg;        // first (layer*B + sequence) of the launch
    int Hkv, cap, block, pool;
};

__global__ __launch_bounds__(256) void score_reduce_kernel(ReduceArgs a)
{
    const int lb = a.lb0_seg + blockIdx.x;
    const int Hkv = a.Hkv, block = a.block;
    int max_items = 0;
    for (int h = 0; h < Hkv; ++h) {
        int n = a.len[lb * Hkv + h];
        n = n < 0 ? 0 : (n > a.cap ? a.cap : n);
        const int N = (n + block - 1) / block;
        max_items = N > max_items ? N : max_items;
    }
    float *base = a.scores + (size_t)lb * Hkv * a.cap;
    auto rows_of = [&](int h) {
        int n = a.len[lb * Hkv + h];
        return n < 0 ? 0 : (n > a.cap ? a.cap : n);
    };
    auto block_mean = [&](int h, int j, int n) {
        const int lo = j * block;
        const int hi = (lo + block < n) ? lo + block : n;
        float acc = 0.f;
        for (int t = lo; t < hi; ++t) acc += base[(size_t)h * a.cap + t];
        return acc / (float)(hi - lo);
    };
    for (int tile = 0; tile < max_items; tile += 256) {
        const int j = tile + threadIdx.x;
        if (a.pool) {
            float pooled = 0.f;
            int heads = 0;
            for (int h = 0; h < Hkv; ++h) {
                const int n = rows_of(h);
                if (j * block < n) { pooled += block_mean(h, j, n); ++heads; }
            }
            __syncthreads();
            for (int h = 0; h < Hkv; ++h)
                if (j * block < rows_of(h)) base[(size_t)h * a.cap + j] = pooled / (float)heads;
            __syncthreads();
        } else {
            for (int h = 0; h < Hkv; ++h) {
                const int n = rows_of(h);
                const bool have = j * block < n;
                const float v = have ? block_mean(h, j, n) : 0.f;
                __syncthreads();
                if (have) base[(size_t)h * a.cap + j] = v;
                __syncthreads();
            }
        }
    }
}

}  // namespace ngc

using namespace ngc;

namespace {
int launch_score(const ngc_cache *c, const ngc_paged_cache *pc, int32_t layer, const void *q_recent,
                 const float *lse_recent, int32_t w, float scale, uint32_t flags, int32_t block,
                 float *scores_out, void *ws, size_t ws_bytes, void *stream)
{
    if (!c->k || !c->len || !q_recent || !scores_out || !ws) return NGC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(c->k) | reinterpret_cast<uintptr_t>(q_recent)) & 15u) return NGC_EINVAL;
    if (c->L <= 0 || c->B <= 0 || c->Hkv <= 0 || c->Hq <= 0 || c->cap <= 0) return NGC_EINVAL;
    if (c->D != 64 && c->D != 128) return NGC_EINVAL;
    if ((long long)c->cap * c->D * 2 > 0x7FFFFFFFLL) return NGC_EUNSUPPORTED;   // 32-bit byte offsets inside a segment
    if (c->Hq % c->Hkv != 0 || w < 1 || block < 1 || !(scale == scale)) return NGC_EINVAL;
    if (layer < -1 || layer >= c->L) return NGC_EINVAL;
    if (ws_bytes < NGC_STATUS_WORDS * sizeof(int32_t)) return NGC_ENOSPC;
    if (lse_recent && (flags & NGC_SCORE_NO_CAUSAL)) return NGC_EINVAL;   // decode's lse is the causal one
    const int G = c->Hq / c->Hkv;
    const int R = w * G;
    if (R > 64) return NGC_EUNSUPPORTED;
    const bool pool = (flags & NGC_SCORE_POOL_HEADS) != 0;
    const int per_layer = c->B * c->Hkv;
    const int seg0 = layer < 0 ? 0 : layer * per_layer;
    const int nseg = layer < 0 ? c->L * per_layer : per_layer;

    ScoreArgs sa;
    sa.k = reinterpret_cast<const unsigned char *>(c->k);
    sa.len = c->len;
    sa.q = reinterpret_cast<const unsigned char *>(q_recent);
    sa.lse = lse_recent;
    sa.psi_out = scores_out;
    sa.status = reinterpret_cast<int32_t *>(ws);
    sa.seg0 = seg0;
    sa.lb0 = layer < 0 ? 0 : layer * c->B;
    sa.w = w; sa.G = G; sa.Hkv = c->Hkv; sa.cap = c->cap;
    sa.causal = (flags & NGC_SCORE_NO_CAUSAL) ? 0 : 1;
    sa.scale_log2e = scale * 1.4426950408889634f;
    sa.table = nullptr; sa.max_pages = 0; sa.num_pages = 0; sa.tpp_shift = 0;
    if (pc) {
        sa.table = pc->table; sa.max_pages = pc->max_pages; sa.num_pages = pc->num_pages;
        int tpp = pc->page_rows / SC_TILE, sh = 0;
        while ((1 << sh) < tpp) ++sh;
        sa.tpp_shift = sh;
    }
    hipStream_t st = (hipStream_t)stream;
    const int qt = (R + 15) / 16;
#define NGC_LAUNCH_SCORE(DD, QQ) \
    hipLaunchKernelGGL((score_keys_kernel<DD, QQ>), dim3(nseg), dim3(SC_WAVES * 64), 0, st, sa)
    if (c->D == 128) {
        if (qt == 1) NGC_LAUNCH_SCORE(128, 1); else if (qt == 2) NGC_LAUNCH_SCORE(128, 2);
        else if (qt == 3) NGC_LAUNCH_SCORE(128, 3); else NGC_LAUNCH_SCORE(128, 4);
    } else {
        if (qt == 1) NGC_LAUNCH_SCORE(64, 1); else if (qt == 2) NGC_LAUNCH_SCORE(64, 2);
        else if (qt == 3) NGC_LAUNCH_SCORE(64, 3); else NGC_LAUNCH_SCORE(64, 4);
    }
#undef NGC_LAUNCH_SCORE
    NGC_HIP_CHECK(hipGetLastError());
    if (pool || block > 1) {
        // scores_out is indexed by the global segment; the reduce kernel gets the global base
        ReduceArgs ra{scores_out, c->len, seg0 / c->Hkv, c->Hkv, c->cap, block, pool ? 1 : 0};
        hipLaunchKernelGGL(score_reduce_kernel, dim3(nseg / c->Hkv), dim3(256), 0, st, ra);
        NGC_HIP_CHECK(hipGetLastError());
    }
    return NGC_OK;
}
}  // namespace

extern "C" int ngc_score_keys(const ngc_cache *c, int32_t layer, const void *q_recent,
                              const float *lse_recent, int32_t w,
                              float scale, uint32_t flags, int32_t block, float *scores_out,
                              void *ws, size_t ws_bytes, void *stream)
{
    if (!c) return NGC_EINVAL;
    return launch_score(c, nullptr, layer, q_recent, lse_recent, w, scale, flags, block, scores_out,
                        ws, ws_bytes, stream);
}

extern "C" int ngc_paged_score_keys(const ngc_paged_cache *pc, int32_t layer, const void *q_recent,
                                    const float *lse_recent, int32_t w,
                                    float scale, uint32_t flags, int32_t block, float *scores_out,
                                    void *ws, size_t ws_bytes, void *stream)
{
    if (!pc || !pc->table) return NGC_EINVAL;
    if (pc->page_rows < SC_TILE || (pc->page_rows & (pc->page_rows - 1)) != 0) return NGC_EINVAL;
    if (pc->max_pages <= 0 || pc->num_pages <= 0) return NGC_EINVAL;
    if ((long long)pc->max_pages * pc->page_rows > 0x7FFFFFFFLL / 256) return NGC_EUNSUPPORTED;
    ngc_cache c{};
    c.k = pc->k_pool; c.v = pc->v_pool; c.len = pc->len; c.pos = nullptr;
    c.L = pc->L; c.B = pc->B; c.Hkv = pc->Hkv; c.Hq = pc->Hq; c.D = pc->D;
    c.cap = pc->max_pages * pc->page_rows;
    return launch_score(&c, pc, layer, q_recent, lse_recent, w, scale, flags, block, scores_out,
                        ws, ws_bytes, stream);
}
