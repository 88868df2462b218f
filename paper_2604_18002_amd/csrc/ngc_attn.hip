// Decode attention over the surviving (compacted, ragged) cache rows on gfx950.
//
// One query token per sequence; every KV head serves G = Hq / Hkv query heads.
// The work is memory bound (each K and V row is read once and used by G
// queries), so the kernel is built around full-row 16-byte loads and keeps the
// vector ALU free by running both contractions on the matrix cores with the G
// query heads padded to a 16-wide tile:
//
//   S^T[row][q] = sum_d K[row][d] Q[q][d]     mfma 16x16x32 bf16, A = K rows
//   O^T[d][q]   = sum_row V[row][d] P[q][row] mfma 16x16x32 bf16, A = V^T
//
// Both products put the query head on the lane index (lane % 16), so all
// soft-max state (running max, running sum, rescale factor) is lane local.
//
// Data movement per 32-row tile and wave:
//   K: 8 (D=128) loads of 16 B per lane, one full row per 16 lanes -> wave
//      private LDS -> read back in the A-operand layout.
//   V: loaded straight into the registers that feed the second product.  Lane
//      (i, kg) loads, for each of the 8 rows that its lane group kg contracts
//      over, the 16 B holding d = 8i .. 8i+7; eight 2x2 16-bit transposes turn
//      them into the eight A operands for the d-tiles {8i + c}.  No LDS.
//   K and V rows are read exactly once, so their loads carry the nontemporal
//      hint (measured on MI355X: 7.1 TB/s streaming reads with it, 6.35 without).
//   P is split into a bf16 head and a bf16 remainder (two MFMAs) so the second
//      product is accurate to ~2^-16 relative, not bf16's 2^-8.
//
// Long segments are split over several workgroups (flash-decode); each writes
// an unnormalised partial (max, sum, O) and takes a ticket of its segment; the
// workgroup that takes the last ticket merges the partials.  One launch per
// call.  The partials and tickets cross workgroups (and the L2 caches of
// different XCDs) through device-scope stores and loads, which go to memory
// (16-byte buffer accesses for the O rows, relaxed atomics for the rest); the
// only wait is each writer's own wait for its stores before the workgroup's
// ticket -- no cache-wide write-back or invalidate is involved.
//
// The same kernel can first append the new token's K/V row (Sec. 4.1: the cache
// grows by one entry per token): the wave that owns the last tile writes the
// row before it loads that tile, and the length is stored by whichever
// workgroup of the segment finishes last, after every other one has read it.
//
// Paged layout (PAGED = true): a 32-row tile never straddles a page (pages hold
// a power-of-two number of rows >= 32), so only the tile's base address changes:
// it comes from the segment's page table.  Table entries are fetched two tiles
// ahead of their use so that the lookup never sits in front of the K/V loads.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "../../include/ngc.h"
#include "ngc_device.h"

namespace ngc {

constexpr int ATT_WAVES = 4;
constexpr int ATT_TILE = 32;   // rows per wave step
constexpr int MAX_SPLITS = 64;  // workgroups per segment at most

struct AttnArgs {
    const unsigned char *k;
    const unsigned char *v;
    const int32_t *len;
    const unsigned char *q;
    float *out;
    float *lse_out;   // optional: log-sum-exp of the scaled scores per query head, natural log
    float *part_o;    // [nseg_launch][S][G][D]
    float *part_ml;   // [nseg_launch][S][G][2]
    int32_t *status;
    int seg0;         // first segment of the launch
    int nseg;         // segments of the launch
    int lb0;          // (layer * B + sequence) that q[0] / out[0] belong to
    int S;            // splits per segment
    int G, Hkv, cap;
    float scale_log2e;
    // paged layout only: k, v are the pools
    const int32_t *table;   // [seg][max_pages]
    int max_pages;
    int num_pages;
    int tpp_shift;          // log2(tiles per page)
    int32_t *ticket;        // [segments of the launch] workgroups of a segment that are done; 0 between launches
    // fused append (APPEND kernels only)
    unsigned char *k_rw;    // the cache again, writable
    unsigned char *v_rw;
    int32_t *len_rw;
    int32_t *pos;           // or nullptr
    const unsigned char *k_new;   // [launch segments][D] bf16
    const unsigned char *v_new;
    const int32_t *new_pos;       // [B] or nullptr
    int B;
};

// Loads and stores that other workgroups' data travels through: relaxed, device scope (served by memory, not by
// an XCD's own L2).
__device__ __forceinline__ void st_device(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_device(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16-byte versions for the partial O rows (a wave's stores land as whole cache lines instead of one 4-byte
// write-through per lane): raw buffer accesses with the device-scope bit, bounds-checked by the hardware against
// `bytes` (a load past the end returns 0, a store past the end is dropped).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t device_span(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
constexpr int AUX_DEVICE_SCOPE = 16;   // sc1
__device__ __forceinline__ void st_device16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, f32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, byte_off, 0, AUX_DEVICE_SCOPE);
}
__device__ __forceinline__ f32x4 ld_device16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, AUX_DEVICE_SCOPE));
}

// Tiles [t_lo, t_hi) of split s when `tiles` tiles are cut into at most S
// nearly equal runs; s_eff = number of non-empty splits.
__device__ __forceinline__ void split_range(int tiles, int S, int s, int &t_lo, int &t_hi, int &s_eff)
{
    const int per = (tiles + S - 1) / S;
    s_eff = per > 0 ? (tiles + per - 1) / per : 0;
    t_lo = s * per;
    t_hi = t_lo + per < tiles ? t_lo + per : tiles;
}

template <int D, bool PAGED, bool APPEND>
__global__ __launch_bounds__(ATT_WAVES * 64) void decode_kernel(AttnArgs a)
{
    constexpr int ROW_BYTES = D * 2;
    constexpr int DPL = D / 16;                 // bf16 per lane in a V row (8 or 4)
    constexpr int KCH = D / 32;                 // 32-wide d chunks of the first product
    constexpr int LROW = ROW_BYTES + 16;        // padded LDS row
    constexpr int K_LOADS = ATT_TILE * ROW_BYTES / (64 * 16);   // 16-B loads per lane per K tile
    constexpr int K_PIECES = ROW_BYTES / 16;    // lanes per K row
    constexpr int K_ROWS_PER_LOAD = 64 / K_PIECES;
    constexpr int WAVE_LDS = ATT_TILE * LROW;

    __shared__ __align__(16) unsigned char lds[ATT_WAVES * WAVE_LDS];
    __shared__ float red_m[ATT_WAVES][16];
    __shared__ float red_l[ATT_WAVES][16];
    __shared__ float fin_l[16];
    __shared__ int is_last;

    const int lane = lane_id(), wv = wave_id();
    const int li = lane & 15, kg = lane >> 4;
    // Workgroup -> (segment, run): run-major, i.e. the first runs of all segments come first, then the second runs,
    // ...  Consecutive workgroups go round-robin to the 8 XCDs: this way every XCD gets the same share of each
    // run index (with the run as the fastest coordinate and S = 2, all first runs land on four of the XCDs and all
    // second runs on the other four: measured 15 % slower at 1024 segments of 16K rows).
    const int split = (int)(blockIdx.x / a.nseg);
    const int seg_local = (int)(blockIdx.x - split * a.nseg);
    const int seg = a.seg0 + seg_local;
    const int G = a.G;

    int n = a.len[seg];
    if (n < 0 || n > a.cap) {
        if (threadIdx.x == 0 && split == 0) atomicAdd(&a.status[NGC_STATUS_LEN_CLAMPED], 1);
        n = n < 0 ? 0 : a.cap;
    }
    // fused append: this call's row goes to slot n and takes part in the attention
    bool grew = false;
    if constexpr (APPEND) {
        if (n < a.cap) {
            grew = true;
            n += 1;
        } else if (threadIdx.x == 0 && split == 0) {
            atomicAdd(&a.status[NGC_STATUS_APPEND_FULL], 1);
        }
    }
    const int h = seg % a.Hkv;
    const int lb = seg / a.Hkv - a.lb0;   // (layer * B + sequence) relative to q / out
    float *out_seg = a.out + ((size_t)lb * a.Hkv + h) * G * D;   // [G][D] of this KV head

    // Every workgroup of a split segment takes a ticket when it is done (right away if its split is empty); the
    // one that takes the last ticket returns true here, all others false.  Whole workgroup calls it.
    auto took_last_ticket = [&]() -> bool {
        __syncthreads();   // this workgroup's partial stores have been waited for by their threads
        if (threadIdx.x == 0) {
            const int old = __hip_atomic_fetch_add(&a.ticket[seg_local], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = (old == a.S - 1) ? 1 : 0;
        }
        __syncthreads();
        return is_last != 0;
    };
    // What the last workgroup of a segment does besides merging: the tickets return to 0 for the next launch and
    // the appended row becomes part of the segment.
    auto close_segment = [&]() {
        if (threadIdx.x == 0) {
            if (a.S > 1) __hip_atomic_store(&a.ticket[seg_local], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (APPEND && grew) a.len_rw[seg] = n;
        }
    };

    if (n == 0) {
        if (split == 0) {
            if (a.lse_out && (int)threadIdx.x < G) a.lse_out[((size_t)lb * a.Hkv + h) * G + threadIdx.x] = -INFINITY;
            for (int i = threadIdx.x; i < G * D; i += ATT_WAVES * 64) out_seg[i] = 0.f;
            if (threadIdx.x == 0) atomicAdd(&a.status[NGC_STATUS_EMPTY_ATTN], 1);
        }
        return;
    }
    const int tiles = (n + ATT_TILE - 1) / ATT_TILE;
    int t_lo, t_hi, s_eff;
    split_range(tiles, a.S, split, t_lo, t_hi, s_eff);
    const float *seg_po = a.part_o + (size_t)seg_local * a.S * G * D;
    const float *seg_pml = a.part_ml + (size_t)seg_local * a.S * G * 2;
    // Merge of the s_eff partials of this segment: out = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M).  Three
    // rounds of loads in all (the partials' (max, sum) pairs, then the O values four splits at a time), each round
    // issued as one batch.  Uses the K staging area, which no wave needs any more.
    auto merge_partials = [&]() {
        __asm__ volatile("" ::: "memory");
        float *ml_s = reinterpret_cast<float *>(lds);          // [s_eff][G][2] -> (weight, sum)
        float *den_s = ml_s + MAX_SPLITS * 16 * 2;             // [G]
        const int n_ml = s_eff * G * 2;
        for (int i = threadIdx.x; i < n_ml; i += ATT_WAVES * 64) ml_s[i] = ld_device(&seg_pml[i]);
        __syncthreads();
        if ((int)threadIdx.x < G) {
            const int qi = threadIdx.x;
            float M = -INFINITY;
            for (int sp = 0; sp < s_eff; ++sp) M = fmaxf(M, ml_s[(sp * G + qi) * 2]);
            float den = 0.f;
            for (int sp = 0; sp < s_eff; ++sp) {
                const float wgt = fast_exp2(ml_s[(sp * G + qi) * 2] - M);
                den += ml_s[(sp * G + qi) * 2 + 1] * wgt;
                ml_s[(sp * G + qi) * 2] = wgt;
            }
            den_s[qi] = den;
            if (a.lse_out) a.lse_out[((size_t)lb * a.Hkv + h) * G + qi] = (M + __log2f(den)) * 0.6931471805599453f;
        }
        __syncthreads();
        const __amdgpu_buffer_rsrc_t po = device_span(seg_po, (uint32_t)(s_eff * G * D * sizeof(float)));
        for (int i4 = threadIdx.x; i4 < G * D / 4; i4 += ATT_WAVES * 64) {
            const int qi = (i4 * 4) / D;
            f32x4 num = {0.f, 0.f, 0.f, 0.f};
            for (int sp0 = 0; sp0 < s_eff; sp0 += 4) {
                f32x4 o[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int sp = (sp0 + u < s_eff) ? sp0 + u : s_eff - 1;
                    o[u] = ld_device16(po, (uint32_t)((sp * G * D + i4 * 4) * sizeof(float)));
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (sp0 + u < s_eff) num += o[u] * ml_s[((sp0 + u) * G + qi) * 2];
            }
            const float inv = 1.0f / den_s[qi];
            *reinterpret_cast<f32x4 *>(&out_seg[i4 * 4]) = num * inv;
        }
    };
    if (t_lo >= t_hi) {   // whole workgroup: no rows for this split
        if (took_last_ticket()) {
            close_segment();
            if (s_eff > 1) merge_partials();
        }
        return;
    }

    const unsigned char *kseg = PAGED ? a.k : a.k + (size_t)seg * a.cap * ROW_BYTES;
    const unsigned char *vseg = PAGED ? a.v : a.v + (size_t)seg * a.cap * ROW_BYTES;
    // paged: byte offset of a tile inside the pools (wave-uniform)
    const int32_t *tab = PAGED ? a.table + (size_t)seg * a.max_pages : nullptr;
    const int wv_u = __builtin_amdgcn_readfirstlane(wv);
    auto tile_base = [&](int tile) -> size_t {
        const int tc = tile < tiles ? tile : tiles - 1;   // a prefetch past the end re-reads the last tile
        int page = tab[tc >> a.tpp_shift];
        page = (page < 0 || page >= a.num_pages) ? 0 : page;   // never leave the pool
        return ((size_t)page << a.tpp_shift) * (ATT_TILE * ROW_BYTES) +
               (size_t)(tc & ((1 << a.tpp_shift) - 1)) * (ATT_TILE * ROW_BYTES);
    };

    // B operand of the first product: Q[q = li][32c + 8kg .. +7], zero for q >= G
    bf16x8 qop[KCH];
    {
        const unsigned char *qrow = a.q + ((size_t)lb * a.Hkv * G + (size_t)h * G + li) * ROW_BYTES;
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            u32x4 w = {0u, 0u, 0u, 0u};
            if (li < G) w = *reinterpret_cast<const u32x4 *>(qrow + c * 64 + kg * 16);
            qop[c] = __builtin_bit_cast(bf16x8, w);
        }
    }

    f32x4 oacc[DPL];
#pragma unroll
    for (int c = 0; c < DPL; ++c) oacc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;

    unsigned char *wlds = lds + wv * WAVE_LDS;
    const int last_row = n - 1;

    // rows this lane loads, relative to the tile: K in full-row order, V in the
    // order its lane group contracts over (matches the layout of the scores)
    int vrow_rel[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) vrow_rel[e] = (e < 4) ? (4 * kg + e) : (16 + 4 * kg + (e - 4));

    // 32-bit byte offsets inside the segment (a segment is at most cap * ROW_BYTES <= 2^31 bytes)
    const uint32_t k_col = (uint32_t)(lane % K_PIECES) * 16u;
    const uint32_t v_col = (uint32_t)li * (DPL * 2);
    u32x4 kbuf[K_LOADS];
    // `base`: paged layout only, tile_base() of the tile
    auto issue_loads = [&](int tile, size_t base, u32x4 (&vb)[8]) {
        const int row0 = tile * ATT_TILE;
        const unsigned char *kt = kseg, *vt = vseg;
        int first = 0;            // row number that offset 0 of kt / vt holds
        if constexpr (PAGED) {
            kt = kseg + base;
            vt = vseg + base;
            first = (tile < tiles ? tile : tiles - 1) * ATT_TILE;
        }
#pragma unroll
        for (int r = 0; r < K_LOADS; ++r) {
            int row = row0 + r * K_ROWS_PER_LOAD + lane / K_PIECES;
            row = row < last_row ? row : last_row;
            kbuf[r] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4 *>(kt + ((uint32_t)(row - first) * ROW_BYTES + k_col)));
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int row = row0 + vrow_rel[e];
            row = row < last_row ? row : last_row;
            const unsigned char *p = vt + ((uint32_t)(row - first) * ROW_BYTES + v_col);
            if constexpr (DPL == 8) {
                vb[e] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
            } else {
                const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
                vb[e] = u32x4{t[0], t[1], 0u, 0u};
            }
        }
    };
    auto stage_k = [&]() {
#pragma unroll
        for (int r = 0; r < K_LOADS; ++r) {
            const int rl = r * K_ROWS_PER_LOAD + lane / K_PIECES;
            *reinterpret_cast<u32x4 *>(wlds + rl * LROW + k_col) = kbuf[r];
        }
    };
    // one 32-row tile: K from the wave's LDS area, V from registers
    auto compute_tile = [&](int tile, const u32x4 (&vcur)[8]) {
        const int row0 = tile * ATT_TILE;
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
            const u32x4 a0 = *reinterpret_cast<const u32x4 *>(wlds + li * LROW + c * 64 + kg * 16);
            const u32x4 a1 = *reinterpret_cast<const u32x4 *>(wlds + (16 + li) * LROW + c * 64 + kg * 16);
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a0), qop[c], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a1), qop[c], s1, 0, 0, 0);
        }
        // lane (q = li, kg) now holds rows 4kg+r (s0[r]) and 16+4kg+r (s1[r])
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float sc = (e < 4) ? s0[e] : s1[e - 4];
            x[e] = (row0 + vrow_rel[e] < n) ? sc * a.scale_log2e : -INFINITY;
        }
        float tmax = x[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) tmax = fmaxf(tmax, x[e]);
        tmax = quad_rows_max(tmax);
        const float m_new = fmaxf(m_run, tmax);           // finite: a tile has a valid row
        if (__ballot(m_new != m_run)) {                   // wave-uniform: the running max moved somewhere
            const float alpha = fast_exp2(m_run - m_new); // 0 on the first tile, 1 where nothing changed
            l_run *= alpha;
#pragma unroll
            for (int c = 0; c < DPL; ++c) oacc[c] *= alpha;
            m_run = m_new;
        }
        float p[8], psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            p[e] = fast_exp2(x[e] - m_run);
            psum += p[e];
        }
        l_run += psum;   // lane-local part; lane groups are summed at the end

        // P as bf16 head + bf16 remainder (B operands)
        uint32_t ph[4], pl[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const uint32_t b0 = __float_as_uint(p[2 * e2]), b1 = __float_as_uint(p[2 * e2 + 1]);
            const float r0 = p[2 * e2] - __uint_as_float(b0 & 0xFFFF0000u);
            const float r1 = p[2 * e2 + 1] - __uint_as_float(b1 & 0xFFFF0000u);
            ph[e2] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);                     // upper halves of b0, b1
            pl[e2] = __builtin_amdgcn_perm(__float_as_uint(r1), __float_as_uint(r0), 0x07060302u);
        }
        const bf16x8 p_hi = __builtin_bit_cast(bf16x8, u32x4{ph[0], ph[1], ph[2], ph[3]});
        const bf16x8 p_lo = __builtin_bit_cast(bf16x8, u32x4{pl[0], pl[1], pl[2], pl[3]});

        // O^T += V^T P
#pragma unroll
        for (int c = 0; c < DPL; ++c) {
            uint32_t va[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const uint32_t w0 = vcur[2 * e2][c >> 1];       // row e = 2*e2,   d pair c/2
                const uint32_t w1 = vcur[2 * e2 + 1][c >> 1];   // row e = 2*e2+1
                // 2x2 transpose of 16-bit elements: one byte permute per output word
                va[e2] = (c & 1) ? __builtin_amdgcn_perm(w1, w0, 0x07060302u)
                                 : __builtin_amdgcn_perm(w1, w0, 0x05040100u);
            }
            const bf16x8 vop = __builtin_bit_cast(bf16x8, u32x4{va[0], va[1], va[2], va[3]});
            oacc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, p_hi, oacc[c], 0, 0, 0);
            oacc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, p_lo, oacc[c], 0, 0, 0);
        }
    };

    // Software pipeline, unrolled by two so that the V registers of the tile in
    // flight and of the tile being computed are distinct (no copies): the loads
    // of the next tile are issued before the current tile's math and are only
    // waited for at the top of the next step.  The prefetch is unconditional (a
    // tile past the end only re-reads the last row, which every load clamps to)
    // so that the number of loads in flight is the same on every path and the
    // wait for the current tile's data does not also wait for the prefetch.
    if constexpr (APPEND) {
        // The wave that owns the last tile stores the new row before anything else.  No other wave or workgroup
        // uses that row (prefetches past a split's end are never computed on).  The wave's loads of that tile
        // come after the store in program order; they are issued at once only when the last tile is also the
        // wave's first one -- then the wave waits for the store first.  Otherwise the loads of the last tile are
        // issued after the wave has waited for an earlier tile's data, and memory operations of a wave complete
        // in issue order, so the store is done by then.
        const int last_tile = tiles - 1;
        if (grew && last_tile >= t_lo && last_tile < t_hi && ((last_tile - t_lo) % ATT_WAVES) == wv) {
            if (lane < 2 * K_PIECES) {
                const bool is_v = lane >= K_PIECES;
                const int piece = is_v ? lane - K_PIECES : lane;
                const size_t src_off = (size_t)seg_local * ROW_BYTES + piece * 16;
                const size_t dst_off = ((size_t)seg * a.cap + (n - 1)) * ROW_BYTES + piece * 16;
                const u32x4 row = *reinterpret_cast<const u32x4 *>((is_v ? a.v_new : a.k_new) + src_off);
                *reinterpret_cast<u32x4 *>((is_v ? a.v_rw : a.k_rw) + dst_off) = row;
            }
            if (lane == 0 && a.pos && a.new_pos) a.pos[(size_t)seg * a.cap + (n - 1)] = a.new_pos[(seg / a.Hkv) % a.B];
            if (last_tile - t_lo < 2 * ATT_WAVES) __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    }

    u32x4 v_a[8], v_b[8];
    int tile = t_lo + (PAGED ? wv_u : wv);
    size_t base1 = 0, base2 = 0;   // paged: bases of the next tile and of the one after it
    if constexpr (PAGED) {
        base1 = tile_base(tile + ATT_WAVES);
        base2 = tile_base(tile + 2 * ATT_WAVES);
        issue_loads(tile, tile_base(tile), v_a);
    } else {
        issue_loads(tile, 0, v_a);
    }
    while (tile < t_hi) {
        stage_k();
        issue_loads(tile + ATT_WAVES, base1, v_b);
        if constexpr (PAGED) { base1 = base2; base2 = tile_base(tile + 3 * ATT_WAVES); }
        __builtin_amdgcn_sched_barrier(0);
        compute_tile(tile, v_a);
        __builtin_amdgcn_sched_barrier(0);
        tile += ATT_WAVES;
        if (tile >= t_hi) break;
        stage_k();
        issue_loads(tile + ATT_WAVES, base1, v_a);
        if constexpr (PAGED) { base1 = base2; base2 = tile_base(tile + 3 * ATT_WAVES); }
        __builtin_amdgcn_sched_barrier(0);
        compute_tile(tile, v_b);
        __builtin_amdgcn_sched_barrier(0);
        tile += ATT_WAVES;
    }

    // ---- merge the waves of this workgroup ----------------------------------
    l_run = quad_rows_sum(l_run);
    if (kg == 0) { red_m[wv][li] = m_run; red_l[wv][li] = l_run; }
    __syncthreads();   // also: every wave is done with its K staging area
    float m_all = red_m[0][li];
#pragma unroll
    for (int w = 1; w < ATT_WAVES; ++w) m_all = fmaxf(m_all, red_m[w][li]);
    float l_all = 0.f;
#pragma unroll
    for (int w = 0; w < ATT_WAVES; ++w) {
        const float mw = red_m[w][li];
        l_all += (mw == -INFINITY) ? 0.f : red_l[w][li] * fast_exp2(mw - m_all);
    }
    const float f = (m_run == -INFINITY) ? 0.f : fast_exp2(m_run - m_all);
    if (wv == 0 && kg == 0) fin_l[li] = l_all;
    // O of every wave, scaled to the common max, into LDS as [wave][q][D] fp32
    // (the K staging area is free now and large enough)
    static_assert(ATT_WAVES * 16 * D * 4 <= ATT_WAVES * WAVE_LDS, "staging area too small");
    float *ost = reinterpret_cast<float *>(lds);
    // lane (q = li, kg), register (c, r) holds d = DPL * (4kg + r) + c
    if (li < G) {
#pragma unroll
        for (int c = 0; c < DPL; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                ost[(wv * 16 + li) * D + DPL * (4 * kg + r) + c] = oacc[c][r] * f;
    }
    __syncthreads();
    const bool direct = (s_eff == 1);   // the only split of its segment with rows: finish here
    if (direct) {
        for (int i = threadIdx.x; i < G * D; i += ATT_WAVES * 64) {
            const int qi = i / D, d = i - qi * D;
            float acc = 0.f;
#pragma unroll
            for (int w = 0; w < ATT_WAVES; ++w) acc += ost[(w * 16 + qi) * D + d];
            out_seg[i] = acc / fin_l[qi];
        }
        if (a.lse_out && wv == 0 && kg == 0 && li < G)
            a.lse_out[((size_t)lb * a.Hkv + h) * G + li] = (m_all + __log2f(l_all)) * 0.6931471805599453f;
        if (a.S == 1 || took_last_ticket()) close_segment();
        return;
    }
    float *dst_o = a.part_o + ((size_t)seg_local * a.S + split) * G * D;
    const __amdgpu_buffer_rsrc_t po = device_span(dst_o, (uint32_t)(G * D * sizeof(float)));
    for (int i4 = threadIdx.x; i4 < G * D / 4; i4 += ATT_WAVES * 64) {
        const int qi = (i4 * 4) / D, d = i4 * 4 - qi * D;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) acc += *reinterpret_cast<const f32x4 *>(&ost[(w * 16 + qi) * D + d]);
        st_device16(po, (uint32_t)(i4 * 4 * sizeof(float)), acc);
    }
    if (wv == 0 && kg == 0 && li < G) {
        float *ml = a.part_ml + (((size_t)seg_local * a.S + split) * G + li) * 2;
        st_device(&ml[0], m_all);
        st_device(&ml[1], l_all);
    }
    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's partial stores have reached memory
    if (took_last_ticket()) {
        close_segment();
        merge_partials();
    }
}

}  // namespace ngc

// ============================================================ host side ====

using namespace ngc;

namespace {
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
constexpr size_t STATUS_BYTES = NGC_STATUS_WORDS * sizeof(int32_t);
// How many workgroups share a segment.  Two measured limits (MI355X, one launch per layer, microseconds per
// launch against S, best in brackets):
//     segments x rows      S=1    2     3     4     6     8    12    16    24    32    64
//         4 x  3-10K                          23.1        16.3  14.8 [14.3] 15.0  16.0  22.0
//        16 x  3-10K                          26.3        19.7 [18.0] 18.8  23.8  25.1  36.4
//        32 x  3-10K       80.3  46.3  35.1  29.4  25.7 [25.6] 31.7  30.8
//        64 x  3-10K       88.7  54.8  44.9 [42.8] 51.0  46.9  50.6  52.2
//       128 x  3-10K      101.1 [77.6] 91.6  82.1  82.6  84.6  89.2  94.0
//       256 x  3-10K     [142.1] 149.9 145.5 148.3 151.9 156.3 166.9 178.0
//         8 x  1.9-2.5K                       12.5       [11.2] 11.5  12.4  14.3  15.7  24.3
//        32 x  1.9-3.5K    33.2  22.6  19.7  17.0 [16.7] 17.3  20.8  20.8
//       128 x  1.9-3.5K    40.7 [36.2] 41.7  39.4  43.8  43.7  48.9  52.9
//       256 x  1.9-3.5K   [60.9] 67.5  71.3  73.2  77.4  81.4  93.2 103.5
//         8 x  1.5K                           10.5       [10.1] 10.4  11.1  13.7  13.7  20.8
//        32 x  1.5K        18.0  14.7  13.6  12.3 [12.2] 12.5  15.0  15.4
//        64 x  1.5K        20.5  16.0 [15.3] 15.5  18.2  17.9  20.9  22.0
//       128 x  1.5K       [22.1] 22.2  25.6  25.0  27.8  29.5  33.9  36.7
// (a) the launch should not have more workgroups than the chip has CUs: beyond one workgroup per CU a further cut
// only adds workgroups, each paying its first-tile wait, its epilogue and the partial -> ticket -> merge chain;
// (b) with few segments, a run should stay long enough that streaming it (~68 GB/s per workgroup) costs more than
// what one more partial adds to the merge (~0.16 us): S ~ sqrt(80 x megabytes of the longest segment).
constexpr int COMPUTE_UNITS = 256;
constexpr int MIN_TILES_PER_SPLIT = 4;

int splits_for(int nseg_launch, int max_len, int row_bytes)
{
    const int tiles = (max_len + ATT_TILE - 1) / ATT_TILE;
    const double seg_mb = 2.0 * row_bytes * max_len * 1e-6;          // K and V
    int s = COMPUTE_UNITS / (nseg_launch > 0 ? nseg_launch : 1);
    const int by_merge = (int)sqrt(80.0 * seg_mb);
    const int by_length = tiles / MIN_TILES_PER_SPLIT;
    s = s < by_merge ? s : by_merge;
    s = s < by_length ? s : by_length;
    s = s < MAX_SPLITS ? s : MAX_SPLITS;
    return s > 1 ? s : 1;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// workspace layout: [status][per segment of the cache: 2 int32 of the paged layout's pool bookkeeping]
//                   [per segment of the cache: ticket][partial O][partial (max, sum)]
size_t ticket_offset(const ngc_cache *c)
{
    return STATUS_BYTES + (size_t)c->L * c->B * c->Hkv * 2 * sizeof(int32_t);
}
size_t attn_offset(const ngc_cache *c)
{
    return align256(ticket_offset(c) + (size_t)c->L * c->B * c->Hkv * sizeof(int32_t));
}
size_t partial_o_bytes(const ngc_cache *c, int nseg_launch, int S)
{
    return align256((size_t)nseg_launch * S * (c->Hq / c->Hkv) * c->D * sizeof(float));
}
size_t partial_ml_bytes(const ngc_cache *c, int nseg_launch, int S)
{
    return align256((size_t)nseg_launch * S * (c->Hq / c->Hkv) * 2 * sizeof(float));
}
size_t attn_partial_bytes(const ngc_cache *c, int nseg_launch, int S)
{
    return S > 1 ? partial_o_bytes(c, nseg_launch, S) + partial_ml_bytes(c, nseg_launch, S) : 0;
}
}  // namespace

extern "C" int ngc_version(void) { return 220; }

extern "C" const char *ngc_strerror(int code)
{
    switch (code) {
    case NGC_OK: return "ok";
    case NGC_EINVAL: return "invalid argument (null or misaligned pointer, bad shape or parameter)";
    case NGC_ENOSPC: return "workspace too small (ngc_decode_attn_static: the call needs more than its fixed scratch array)";
    case NGC_EHIP: return "a HIP runtime call failed";
    case NGC_EUNSUPPORTED: return "request outside the limits of this entry point";
    default: return "unknown error code";
    }
}

extern "C" size_t ngc_workspace_bytes(const ngc_cache *c, int32_t max_keep)
{
    (void)max_keep;
    if (!c || c->L <= 0 || c->B <= 0 || c->Hkv <= 0 || c->Hq <= 0 || c->cap <= 0) return 0;
    const int per_layer = c->B * c->Hkv;
    // the most any launch can ask for: one layer or all layers, any length hint (a launch that finds less
    // workspace than its preferred split needs falls back to fewer splits, so this is a guarantee, not a limit)
    size_t most = 0;
    for (int hint = c->cap; hint >= 1; hint = hint / 2) {
        const size_t one = attn_partial_bytes(c, per_layer, splits_for(per_layer, hint, c->D * 2));
        const size_t all = attn_partial_bytes(c, per_layer * c->L, splits_for(per_layer * c->L, hint, c->D * 2));
        most = one > most ? one : most;
        most = all > most ? all : most;
    }
    return attn_offset(c) + most;
}

namespace {
// Shared by both layouts.  `c` carries the logical geometry (for the paged
// layout: cap = max_pages * page_rows, k / v = the pools).
struct NewRows {            // fused append: the new token's rows, or all null
    const void *k_new;
    const void *v_new;
    const int32_t *new_pos;
};

// `fixed_layout`: the scratch is not a workspace sized for this cache but the library's own fixed array, which
// serves caches of any geometry one after the other: tickets and partials then sit at offsets that do not depend
// on the geometry (a ticket region that moved with the geometry would land on an earlier call's partials).
constexpr size_t FIXED_TICKET_OFFSET = STATUS_BYTES;      // COMPUTE_UNITS tickets: only launches of at most
constexpr size_t FIXED_PARTIAL_OFFSET = 4096;             // COMPUTE_UNITS / 2 segments are ever split

int launch_decode(const ngc_cache *c, const ngc_paged_cache *pc, int32_t layer, const NewRows *nr, const void *q,
                  float scale, int32_t max_len_hint, float *out, float *lse_out, int32_t *status, void *ws,
                  size_t ws_bytes, void *stream, bool fixed_layout = false)
{
    if (nr && (!nr->k_new || !nr->v_new || !aligned16(nr->k_new) || !aligned16(nr->v_new) || pc)) return NGC_EINVAL;
    if (!c->k || !c->v || !c->len || !q || !out || !ws) return NGC_EINVAL;
    if (!aligned16(c->k) || !aligned16(c->v) || !aligned16(q) || !aligned16(out) || !aligned16(ws)) return NGC_EINVAL;
    if (c->L <= 0 || c->B <= 0 || c->Hkv <= 0 || c->Hq <= 0 || c->cap <= 0) return NGC_EINVAL;
    if (c->D != 64 && c->D != 128) return NGC_EINVAL;
    if ((long long)c->cap * c->D * 2 > 0x7FFFFFFFLL) return NGC_EUNSUPPORTED;   // 32-bit byte offsets inside a segment
    if (c->Hq % c->Hkv != 0 || c->Hq / c->Hkv > 16) return NGC_EINVAL;
    if (layer < -1 || layer >= c->L || max_len_hint < 0) return NGC_EINVAL;
    if (!(scale == scale)) return NGC_EINVAL;
    const int per_layer = c->B * c->Hkv;
    const int seg0 = layer < 0 ? 0 : layer * per_layer;
    const int nseg = layer < 0 ? c->L * per_layer : per_layer;
    const int max_len = (max_len_hint > 0 && max_len_hint < c->cap) ? max_len_hint : c->cap;
    int S = splits_for(nseg, max_len, c->D * 2);
    if (nseg > COMPUTE_UNITS) S = 1;   // (what splits_for() returns anyway: the fixed ticket region relies on it)
    const size_t off = fixed_layout ? FIXED_PARTIAL_OFFSET : attn_offset(c);
    if (ws_bytes < off) return NGC_ENOSPC;
    if (fixed_layout) {   // the fixed array either holds what the launch wants or the call is refused
        if (ws_bytes < off + attn_partial_bytes(c, nseg, S)) return NGC_ENOSPC;
    } else {
        while (S > 1 && ws_bytes < off + attn_partial_bytes(c, nseg, S)) --S;   // fewer splits: same result, less scratch
    }
    if ((long long)nseg * S > 0x7FFFFFFFLL) return NGC_EUNSUPPORTED;

    AttnArgs aa;
    aa.k = reinterpret_cast<const unsigned char *>(c->k);
    aa.v = reinterpret_cast<const unsigned char *>(c->v);
    aa.len = c->len;
    aa.q = reinterpret_cast<const unsigned char *>(q);
    aa.out = out;
    aa.lse_out = lse_out;
    aa.part_o = reinterpret_cast<float *>(reinterpret_cast<unsigned char *>(ws) + off);
    aa.part_ml = reinterpret_cast<float *>(reinterpret_cast<unsigned char *>(ws) + off +
                                           partial_o_bytes(c, nseg, S));
    aa.status = status ? status : reinterpret_cast<int32_t *>(ws);
    aa.seg0 = seg0;
    aa.nseg = nseg;
    aa.lb0 = layer < 0 ? 0 : layer * c->B;
    aa.S = S; aa.G = c->Hq / c->Hkv; aa.Hkv = c->Hkv; aa.cap = c->cap;
    aa.scale_log2e = scale * 1.4426950408889634f;
    aa.ticket = reinterpret_cast<int32_t *>(reinterpret_cast<unsigned char *>(ws) +
                                            (fixed_layout ? FIXED_TICKET_OFFSET : ticket_offset(c)));
    aa.k_rw = reinterpret_cast<unsigned char *>(c->k);
    aa.v_rw = reinterpret_cast<unsigned char *>(c->v);
    aa.len_rw = c->len;
    aa.pos = c->pos;
    aa.k_new = nr ? reinterpret_cast<const unsigned char *>(nr->k_new) : nullptr;
    aa.v_new = nr ? reinterpret_cast<const unsigned char *>(nr->v_new) : nullptr;
    aa.new_pos = nr ? nr->new_pos : nullptr;
    aa.B = c->B;
    aa.table = nullptr; aa.max_pages = 0; aa.num_pages = 0; aa.tpp_shift = 0;
    if (pc) {
        aa.table = pc->table; aa.max_pages = pc->max_pages; aa.num_pages = pc->num_pages;
        int tpp = pc->page_rows / ATT_TILE, sh = 0;
        while ((1 << sh) < tpp) ++sh;
        aa.tpp_shift = sh;
    }
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid(nseg * S), block(ATT_WAVES * 64);
    if (pc) {
        if (c->D == 128) hipLaunchKernelGGL((decode_kernel<128, true, false>), grid, block, 0, st, aa);
        else             hipLaunchKernelGGL((decode_kernel<64, true, false>), grid, block, 0, st, aa);
    } else if (nr) {
        if (c->D == 128) hipLaunchKernelGGL((decode_kernel<128, false, true>), grid, block, 0, st, aa);
        else             hipLaunchKernelGGL((decode_kernel<64, false, true>), grid, block, 0, st, aa);
    } else {
        if (c->D == 128) hipLaunchKernelGGL((decode_kernel<128, false, false>), grid, block, 0, st, aa);
        else             hipLaunchKernelGGL((decode_kernel<64, false, false>), grid, block, 0, st, aa);
    }
    NGC_HIP_CHECK(hipGetLastError());
    return NGC_OK;
}
}  // namespace

extern "C" int ngc_decode_attn(const ngc_cache *c, int32_t layer, const void *q, float scale,
                               int32_t max_len_hint, float *out, float *lse_out,
                               void *ws, size_t ws_bytes, void *stream)
{
    if (!c) return NGC_EINVAL;
    return launch_decode(c, nullptr, layer, nullptr, q, scale, max_len_hint, out, lse_out, nullptr, ws, ws_bytes,
                         stream);
}

extern "C" int ngc_decode_step(const ngc_cache *c, int32_t layer, const void *k_new, const void *v_new,
                               const int32_t *new_pos, const void *q, float scale, int32_t max_len_hint,
                               float *out, float *lse_out, void *ws, size_t ws_bytes, void *stream)
{
    if (!c) return NGC_EINVAL;
    const NewRows nr{k_new, v_new, new_pos};
    return launch_decode(c, nullptr, layer, &nr, q, scale, max_len_hint, out, lse_out, nullptr, ws, ws_bytes, stream);
}

// ---- the same call for callers that cannot allocate ------------------------
//
// The split partials and tickets (and, when the caller passes no status buffer,
// the status words) live in a fixed array inside the library's device image
// instead of a caller-provided workspace.  The array starts out zeroed when the
// image is loaded and every launch leaves the tickets at zero again.  Every GPU holds its own copy of the array; its
// address on a device is looked up once, with that device current, and kept.
constexpr size_t STATIC_SCRATCH_BYTES = NGC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES];      // device address of `scratch` per device, nullptr until looked up

int static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return NGC_EHIP;
    if (dev < 0 || dev >= MAX_DEVICES) return NGC_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return NGC_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return NGC_OK;
}
}  // namespace

extern "C" int ngc_decode_attn_static(const ngc_cache *c, int32_t layer, const void *q, float scale,
                                      int32_t max_len_hint, float *out, float *lse_out,
                                      int32_t *status, void *stream)
{
    if (!c) return NGC_EINVAL;
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc) return rc;
    return launch_decode(c, nullptr, layer, nullptr, q, scale, max_len_hint, out, lse_out, status, ws,
                         STATIC_SCRATCH_BYTES, stream, true);
}

extern "C" int ngc_paged_decode_attn(const ngc_paged_cache *pc, int32_t layer, const void *q, float scale,
                                     int32_t max_len_hint, float *out, float *lse_out,
                                     void *ws, size_t ws_bytes, void *stream)
{
    if (!pc || !pc->table) return NGC_EINVAL;
    if (pc->page_rows < ATT_TILE || (pc->page_rows & (pc->page_rows - 1)) != 0) return NGC_EINVAL;
    if (pc->max_pages <= 0 || pc->num_pages <= 0) return NGC_EINVAL;
    if ((long long)pc->max_pages * pc->page_rows > 0x7FFFFFFFLL / 256) return NGC_EUNSUPPORTED;
    ngc_cache c{};
    c.k = pc->k_pool; c.v = pc->v_pool; c.len = pc->len; c.pos = nullptr;
    c.L = pc->L; c.B = pc->B; c.Hkv = pc->Hkv; c.Hq = pc->Hq; c.D = pc->D;
    c.cap = pc->max_pages * pc->page_rows;
    return launch_decode(&c, pc, layer, nullptr, q, scale, max_len_hint, out, lse_out, nullptr, ws, ws_bytes, stream);
}
