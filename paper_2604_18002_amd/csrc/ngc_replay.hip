// Replay attention for the training forward pass (Sec. 4.5 and Appendix A.3 of
// the paper): all T positions of a trajectory at once, query i seeing key j iff
// j <= i and j had not been evicted when token i was generated.
//
// Instead of the paper's dense T x T boolean mask per layer, visibility is one
// int per key: death[j] = first query position that no longer sees key j, so
// visible(i, j) = (j <= i < death[j]).  A small first kernel compacts, for every
// tile of 128 query positions, the list of keys that at least one of its
// queries can see (j not after its last query, death[j] after its first); the
// attention kernel then only ever loads those rows: the work follows the
// retained cache, not the T x T triangle.  The lists are shared by all query
// heads that share the decisions.
//
// Flash-attention forward on the matrix cores, same operand scheme as the
// decode kernel (S^T = K Q^T, O^T = V^T P, query on lane%16, P as bf16 head +
// remainder).  A workgroup = 4 waves x 32 query positions of one query head;
// K/V tiles of 32 keys are loaded cooperatively into double-buffered LDS and
// shared by the 4 waves.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/ngc.h"
#include "ngc_device.h"

namespace ngc {

constexpr int RP_WAVES = 4;
constexpr int RP_QW = 32;                    // query positions per wave
constexpr int RP_QT = RP_WAVES * RP_QW;      // query positions per workgroup
constexpr int RP_KT = 64;                    // keys per LDS tile (one barrier per tile)
constexpr int RP_MT = 32;                    // keys per step of the math (and per entry of tile_death)
// Start of the running max: finite and below every real score, so that 2^(x - m) is 0 for a masked
// x = -inf without a special case, and the first rescale factor 2^(m_init - m_new) is 0.
constexpr float RP_M_INIT = -1.0e30f;

struct ReplayArgs {
    const unsigned char *q;    // bf16 [B][T][Hq][D]
    const unsigned char *k;    // bf16 [B][T][Hkv][D]
    const unsigned char *v;
    const int32_t *death;      // [B][Hd][T]
    uint16_t *klist;           // [B*Hd][nqt][T] visible keys per query tile, ascending
    int32_t *kcount;           // [B*Hd][nqt]
    int32_t *tile_death;       // [B*Hd][nqt][ceil(T/32)] smallest death among each RP_MT keys of a list
    float *out;                // fp32 [B][T][Hq][D]
    int B, T, Hq, Hkv, Hd;     // Hd = Hkv (a death row per KV head) or 1 (shared by the heads)
    float scale_log2e;
};

// Ordered compaction (ballot + prefix over the 4 waves), 256 keys per step.
__global__ __launch_bounds__(RP_WAVES * 64) void replay_lists_kernel(ReplayArgs a)
{
    __shared__ int wave_cnt[RP_WAVES];
    const int tid = threadIdx.x, lane = lane_id(), wv = wave_id();
    const int T = a.T;
    const int nqt = (T + RP_QT - 1) / RP_QT;
    const int qt = blockIdx.x, row = blockIdx.y;          // row = b * Hd + hd
    const int i0 = qt * RP_QT;
    const int last_pos = (i0 + RP_QT - 1 < T - 1) ? i0 + RP_QT - 1 : T - 1;
    const int32_t *death = a.death + (size_t)row * T;
    uint16_t *klist = a.klist + ((size_t)row * nqt + qt) * T;
    int n_list = 0;
    for (int j0 = 0; j0 <= last_pos; j0 += RP_WAVES * 64) {
        const int j = j0 + tid;
        const bool pred = j <= last_pos && death[j] > i0;
        const uint64_t bal = __ballot(pred);
        if (lane == 0) wave_cnt[wv] = __popcll(bal);
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int x = 0; x < RP_WAVES; ++x) {
            const int c = wave_cnt[x];
            if (x < wv) before += c;
            total += c;
        }
        if (pred) klist[n_list + before + popc_below(bal)] = (uint16_t)j;
        n_list += total;
        __syncthreads();
    }
    if (tid == 0) a.kcount[(size_t)row * nqt + qt] = n_list;
    // smallest death per list tile: a tile whose keys all outlive a wave's queries needs no per-element mask
    // (the list writes above are this workgroup's own and the loop ended on a barrier)
    const int tiles_max = (T + RP_MT - 1) / RP_MT;
    int32_t *tmin = a.tile_death + ((size_t)row * nqt + qt) * tiles_max;
    for (int t = tid; t * RP_MT < n_list; t += RP_WAVES * 64) {
        const int s1 = (t + 1) * RP_MT < n_list ? (t + 1) * RP_MT : n_list;
        int m = 0x7FFFFFFF;
        for (int s = t * RP_MT; s < s1; ++s) {
            const int d = death[klist[s]];
            m = d < m ? d : m;
        }
        tmin[t] = m;
    }
}

template <int D>
__global__ __launch_bounds__(RP_WAVES * 64) __attribute__((amdgpu_waves_per_eu(2)))
void replay_attn_kernel(ReplayArgs a)
{
    constexpr int ROW_BYTES = D * 2;
    constexpr int DPL = D / 16;
    constexpr int KCH = D / 32;
    constexpr int LROW = ROW_BYTES + 16;
    constexpr int TILE_LDS = RP_KT * LROW;
    constexpr int PIECES = ROW_BYTES / 16;                 // 16-byte pieces per row
    constexpr int LOADS = RP_KT * PIECES / (RP_WAVES * 64); // per thread, per tensor

    __shared__ __align__(16) unsigned char lds_k[2][TILE_LDS];
    __shared__ __align__(16) unsigned char lds_v[2][TILE_LDS];
    __shared__ __align__(16) int32_t lds_death[2][RP_KT];
    __shared__ __align__(16) int32_t lds_kidx[2][RP_KT];
    __shared__ int32_t lds_tmin[2][RP_KT / RP_MT];

    const int tid = threadIdx.x, lane = lane_id(), wv = wave_id();
    const int li = lane & 15, kg = lane >> 4;
    const int T = a.T;
    const int nqt = (T + RP_QT - 1) / RP_QT;
    // Workgroup -> (query tile, head, trajectory).  The hardware deals consecutive workgroups round-robin to the
    // 8 XCDs, and a query tile's work grows with its position, so the tile index is the slowest coordinate,
    // heaviest first: every XCD gets the same mix of tiles at every moment.  Within one tile index the KV group
    // (trajectory, KV head) is the fastest coordinate: with a multiple of 8 groups an XCD always works on the
    // same groups, whose K/V rows then stay in its own L2 for all their query heads and tiles.
    const int G = a.Hq / a.Hkv;
    const int nkv = a.B * a.Hkv;
    const int per_tile = G * nkv;
    const int qt = nqt - 1 - (int)(blockIdx.x / per_tile);
    const int rem = (int)(blockIdx.x % per_tile);
    const int kvp = rem % nkv;
    const int b = kvp / a.Hkv, hkv = kvp % a.Hkv;
    const int head = hkv * G + rem / nkv;
    const int hd = a.Hd == 1 ? 0 : hkv;
    const int i0 = qt * RP_QT;
    const int32_t *death = a.death + ((size_t)b * a.Hd + hd) * T;
    // bytes between consecutive tokens; a sequence's K (or V) spans less than 2^32 bytes (checked on the host),
    // so a row's offset from the sequence's first row fits 32 bits
    const uint32_t kv_row = (uint32_t)a.Hkv * ROW_BYTES;
    const unsigned char *kbase = a.k + ((size_t)b * T * a.Hkv + hkv) * ROW_BYTES;
    const unsigned char *vbase = a.v + ((size_t)b * T * a.Hkv + hkv) * ROW_BYTES;

    // ---- query operands: two tiles of 16 positions per wave ------------------
    int qpos[2];
    bf16x8 qop[2][KCH];
#pragma unroll
    for (int qa = 0; qa < 2; ++qa) {
        qpos[qa] = i0 + wv * RP_QW + qa * 16 + li;
        const int p = qpos[qa] < T ? qpos[qa] : T - 1;
        const unsigned char *qrow = a.q + (((size_t)b * T + p) * a.Hq + head) * ROW_BYTES;
#pragma unroll
        for (int c = 0; c < KCH; ++c)
            qop[qa][c] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(qrow + c * 64 + kg * 16));
    }

    f32x4 oacc[2][DPL];
    float m_run[2], l_run[2];
#pragma unroll
    for (int qa = 0; qa < 2; ++qa) {
        m_run[qa] = RP_M_INIT;
        l_run[qa] = 0.f;
#pragma unroll
        for (int c = 0; c < DPL; ++c) oacc[qa][c] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    int vrow_rel[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) vrow_rel[e] = (e < 4) ? (4 * kg + e) : (16 + 4 * kg + (e - 4));

    // keys this workgroup needs (list built by replay_lists_kernel)
    const uint16_t *klist = a.klist + (((size_t)b * a.Hd + hd) * nqt + qt) * T;
    int n_list = 0;   // length of the list; read after the first list entries have been requested
    const int32_t *tmin = a.tile_death + (((size_t)b * a.Hd + hd) * nqt + qt) * ((T + RP_MT - 1) / RP_MT);
    const int wave_q0 = i0 + wv * RP_QW;                               // first query position of this wave
    const int wave_q1 = (wave_q0 + RP_QW - 1 < T - 1) ? wave_q0 + RP_QW - 1 : T - 1;   // last real one

    // One tile on its way from global memory to LDS, in two steps so that no load waits for another
    // inside one step: first the list entries (which keys), one step later the rows they name.
    struct IdxStage {
        int key[LOADS];   // key index of the rows this thread copies
        int mine;         // the entry of list slot s0 + tid % RP_KT, as stored
    };
    struct Stage {
        u32x4 k[LOADS], v[LOADS];
        int d, i;
        int tmin;   // threads < RP_KT / RP_MT only
    };
    // List entries are fetched without looking at the list's length (slots past its end hold whatever the
    // workspace held: any value is clamped to a valid key, and such slots are switched off when the tile is
    // stored), so the first of these loads does not have to wait for the length to arrive.
    auto load_idx = [&](int t, IdxStage &ix) {
        const int s0 = t * RP_KT;
#pragma unroll
        for (int r = 0; r < LOADS; ++r) {
            const int piece_id = r * (RP_WAVES * 64) + tid;
            int slot = s0 + piece_id / PIECES;
            slot = slot < T ? slot : T - 1;             // a list row has T slots
            const int key = (int)klist[slot];
            ix.key[r] = key < T ? key : T - 1;          // whatever the list holds, stay inside k / v
        }
        // every thread fetches the key of list slot s0 + tid % RP_KT: no branch around a load, so the loads in
        // flight are the same on every path
        int sl = s0 + (tid & (RP_KT - 1));
        sl = sl < T ? sl : T - 1;
        ix.mine = (int)klist[sl];
    };
    auto load_rows = [&](int t, const IdxStage &ix, Stage &st) {
#pragma unroll
        for (int r = 0; r < LOADS; ++r) {
            const int piece_id = r * (RP_WAVES * 64) + tid;
            const uint32_t off = (uint32_t)ix.key[r] * kv_row + (uint32_t)(piece_id % PIECES) * 16u;
            st.k[r] = *reinterpret_cast<const u32x4 *>(kbase + off);
            st.v[r] = *reinterpret_cast<const u32x4 *>(vbase + off);
        }
        int ti = t * (RP_KT / RP_MT) + (tid & (RP_KT / RP_MT - 1));
        const bool t_inside = ti * RP_MT < n_list;
        ti = t_inside ? ti : 0;
        const int tm = tmin[ti];
        st.tmin = t_inside ? tm : 0;
        // 0x7FFFFFFF = a key no query comes after: slots past the end of the list
        const bool inside = t * RP_KT + (tid & (RP_KT - 1)) < n_list;
        const int dkey = ix.mine < T ? ix.mine : T - 1;
        const int dv = death[dkey];
        st.i = inside ? ix.mine : 0x7FFFFFFF;
        st.d = inside ? dv : 0;
    };
    auto store_tile = [&](int buf, const Stage &st) {
#pragma unroll
        for (int r = 0; r < LOADS; ++r) {
            const int piece_id = r * (RP_WAVES * 64) + tid;
            const int off = (piece_id / PIECES) * LROW + (piece_id % PIECES) * 16;
            *reinterpret_cast<u32x4 *>(lds_k[buf] + off) = st.k[r];
            *reinterpret_cast<u32x4 *>(lds_v[buf] + off) = st.v[r];
        }
        if (tid < RP_KT) { lds_death[buf][tid] = st.d; lds_kidx[buf][tid] = st.i; }
        if (tid < RP_KT / RP_MT) lds_tmin[buf][tid] = st.tmin;
    };

    auto compute_tile = [&](int buf) {
#pragma unroll
      for (int half = 0; half < RP_KT / RP_MT; ++half) {
        // ---- RP_MT keys of this tile, from LDS --------------------------------
        const unsigned char *lk = lds_k[buf] + half * RP_MT * LROW, *lv = lds_v[buf] + half * RP_MT * LROW;
        const int32_t *ldeath = &lds_death[buf][half * RP_MT], *lkidx = &lds_kidx[buf][half * RP_MT];
        // the list ascends: if the first of these keys is after this wave's last query, so are all
        const bool wave_needs = (lkidx[0] <= i0 + wv * RP_QW + RP_QW - 1);
        if (wave_needs) {
            bf16x8 kop[2][KCH];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int c = 0; c < KCH; ++c)
                    kop[mt][c] = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const u32x4 *>(lk + (mt * 16 + li) * LROW + c * 64 + kg * 16));
            // A tile whose keys all precede this wave's first query and all outlive its last one needs no
            // mask (wave-uniform, so the branches below do not diverge).
            const bool full = __builtin_amdgcn_readfirstlane(
                (lkidx[RP_MT - 1] <= wave_q0 && lds_tmin[buf][half] > wave_q1) ? 1 : 0) != 0;
            bf16x8 p_hi[2], p_lo[2];
            f32x4 sc0[2], sc1[2];
#pragma unroll
            for (int qa = 0; qa < 2; ++qa) {
                sc0[qa] = f32x4{0.f, 0.f, 0.f, 0.f};
                sc1[qa] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int c = 0; c < KCH; ++c)
#pragma unroll
                for (int qa = 0; qa < 2; ++qa) {
                    sc0[qa] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[0][c], qop[qa][c], sc0[qa], 0, 0, 0);
                    sc1[qa] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[1][c], qop[qa][c], sc1[qa], 0, 0, 0);
                }
            // The V rows are requested as soon as the first product has been issued (the K operand registers are
            // free from here on) and arrive while the soft-max arithmetic runs.
            __builtin_amdgcn_sched_barrier(0);
            u32x4 vcur[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if constexpr (DPL == 8) {
                    vcur[e] = *reinterpret_cast<const u32x4 *>(lv + vrow_rel[e] * LROW + li * 16);
                } else {
                    const u32x2 tt = *reinterpret_cast<const u32x2 *>(lv + vrow_rel[e] * LROW + li * 8);
                    vcur[e] = u32x4{tt[0], tt[1], 0u, 0u};
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int qa = 0; qa < 2; ++qa) {
                const f32x4 s0 = sc0[qa], s1 = sc1[qa];
                // raw scores; the (positive) scale is applied inside the exponent's multiply-add, the running
                // max lives in the scaled domain
                float x[8];
                const int qp = qpos[qa];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = (e < 4) ? s0[e] : s1[e - 4];
                if (!full) {
                    // key indices and death positions of the rows this lane holds (rare path: fetched here, per
                    // query tile, rather than kept in registers across the common path)
                    const int4 d0 = *reinterpret_cast<const int4 *>(&ldeath[4 * kg]);
                    const int4 d1 = *reinterpret_cast<const int4 *>(&ldeath[16 + 4 * kg]);
                    const int4 j0 = *reinterpret_cast<const int4 *>(&lkidx[4 * kg]);
                    const int4 j1 = *reinterpret_cast<const int4 *>(&lkidx[16 + 4 * kg]);
                    const int dk[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
                    const int jk[8] = {j0.x, j0.y, j0.z, j0.w, j1.x, j1.y, j1.z, j1.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (!(jk[e] <= qp && qp < dk[e])) x[e] = -INFINITY;
                }
                // scores are finite or -inf, never NaN (finite inputs)
                float tmx = x[0];
#pragma unroll
                for (int e = 1; e < 8; ++e) tmx = max_no_nan(tmx, x[e]);
                tmx = quad_rows_max(tmx) * a.scale_log2e;
                const float m_new = max_no_nan(m_run[qa], tmx);
                if (__ballot(m_new != m_run[qa])) {
                    // m_new is finite wherever it changed; exp2(-inf - finite) = 0 on a first visible tile
                    const float alpha = (m_new == m_run[qa]) ? 1.0f : fast_exp2(m_run[qa] - m_new);
                    l_run[qa] *= alpha;
#pragma unroll
                    for (int c = 0; c < DPL; ++c) oacc[qa][c] *= alpha;
                    m_run[qa] = m_new;
                }
                float p[8], psum = 0.f;
                const float neg_m = -m_run[qa];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = fast_exp2(__builtin_fmaf(x[e], a.scale_log2e, neg_m));   // x = -inf gives 0: m_run is finite
                    psum += p[e];
                }
                l_run[qa] += psum;
                uint32_t ph[4], pl[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const uint32_t b0 = __float_as_uint(p[2 * e2]), b1 = __float_as_uint(p[2 * e2 + 1]);
                    const float r0 = p[2 * e2] - __uint_as_float(b0 & 0xFFFF0000u);
                    const float r1 = p[2 * e2 + 1] - __uint_as_float(b1 & 0xFFFF0000u);
                    ph[e2] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);                     // upper halves of b0, b1
                    pl[e2] = __builtin_amdgcn_perm(__float_as_uint(r1), __float_as_uint(r0), 0x07060302u);
                }
                p_hi[qa] = __builtin_bit_cast(bf16x8, u32x4{ph[0], ph[1], ph[2], ph[3]});
                p_lo[qa] = __builtin_bit_cast(bf16x8, u32x4{pl[0], pl[1], pl[2], pl[3]});
            }
#pragma unroll
            for (int c = 0; c < DPL; ++c) {
                uint32_t va[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const uint32_t w0 = vcur[2 * e2][c >> 1];
                    const uint32_t w1 = vcur[2 * e2 + 1][c >> 1];
                    // 2x2 transpose of 16-bit elements: one byte permute per output word
                    va[e2] = (c & 1) ? __builtin_amdgcn_perm(w1, w0, 0x07060302u) : __builtin_amdgcn_perm(w1, w0, 0x05040100u);
                }
                const bf16x8 vop = __builtin_bit_cast(bf16x8, u32x4{va[0], va[1], va[2], va[3]});
#pragma unroll
                for (int qa = 0; qa < 2; ++qa) {
                    oacc[qa][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, p_hi[qa], oacc[qa][c], 0, 0, 0);
                    oacc[qa][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, p_lo[qa], oacc[qa][c], 0, 0, 0);
                }
            }
        }
      }
    };

    // Per step: tile t is computed from LDS while the rows of tile t+1 travel through registers into
    // the other LDS buffer and the list entries of tile t+2 are fetched.  Unrolled by two so that the two
    // list-entry stages swap roles without copies; every load is unconditional so the number of loads in
    // flight is the same on every path.
    Stage st;
    IdxStage ix_a, ix_b;
    load_idx(0, ix_a);
    load_idx(1, ix_b);
    n_list = a.kcount[((size_t)b * a.Hd + hd) * nqt + qt];
    const int t_end = (n_list + RP_KT - 1) / RP_KT;
    load_rows(0, ix_a, st);
    store_tile(0, st);
    __syncthreads();
    int t = 0, buf = 0;
    while (t < t_end) {
        load_idx(t + 2, ix_a);
        load_rows(t + 1, ix_b, st);
        __builtin_amdgcn_sched_barrier(0);
        compute_tile(buf);
        __builtin_amdgcn_sched_barrier(0);
        store_tile(buf ^ 1, st);
        __syncthreads();
        buf ^= 1;
        if (++t >= t_end) break;
        load_idx(t + 2, ix_b);
        load_rows(t + 1, ix_a, st);
        __builtin_amdgcn_sched_barrier(0);
        compute_tile(buf);
        __builtin_amdgcn_sched_barrier(0);
        store_tile(buf ^ 1, st);
        __syncthreads();
        buf ^= 1;
        ++t;
    }

    // ---- normalise and write -------------------------------------------------
#pragma unroll
    for (int qa = 0; qa < 2; ++qa) {
        float l = l_run[qa];
        l = quad_rows_sum(l);
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        if (qpos[qa] < T) {
            float *orow = a.out + (((size_t)b * T + qpos[qa]) * a.Hq + head) * D;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // lane (q = li, kg), register (c, r) holds d = DPL * (4kg + r) + c
                float *dst = orow + DPL * (4 * kg + r);
#pragma unroll
                for (int c = 0; c < DPL; c += 4)
                    *reinterpret_cast<float4 *>(dst + c) =
                        make_float4(oacc[qa][c][r] * inv, oacc[qa][c + 1][r] * inv, oacc[qa][c + 2][r] * inv,
                                    oacc[qa][c + 3][r] * inv);
            }
        }
    }
}

}  // namespace ngc

using namespace ngc;

extern "C" size_t ngc_replay_workspace_bytes(int32_t B, int32_t T, int32_t Hkv)
{
    if (B <= 0 || T <= 0 || Hkv <= 0) return 0;
    const size_t nqt = (size_t)(T + RP_QT - 1) / RP_QT;
    size_t lists = (size_t)B * Hkv * nqt * T * sizeof(uint16_t);
    lists = (lists + 255) & ~(size_t)255;
    size_t counts = (size_t)B * Hkv * nqt * sizeof(int32_t);
    counts = (counts + 255) & ~(size_t)255;
    const size_t tiles_max = (size_t)(T + RP_MT - 1) / RP_MT;
    return 256 + lists + counts + (size_t)B * Hkv * nqt * tiles_max * sizeof(int32_t);
}

extern "C" int ngc_replay_attn(const void *q, const void *k, const void *v, const int32_t *death,
                               int32_t B, int32_t T, int32_t Hq, int32_t Hkv, int32_t D,
                               int32_t death_per_head, float scale, float *out,
                               void *ws, size_t ws_bytes, void *stream)
{
    if (!q || !k || !v || !death || !out || !ws) return NGC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(v) |
         reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(ws)) & 15u)
        return NGC_EINVAL;
    if (B <= 0 || T <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return NGC_EINVAL;
    if (D != 64 && D != 128) return NGC_EINVAL;
    if (!(scale > 0.f) || scale > 3.0e38f) return NGC_EINVAL;   // positive and finite: the kernel takes maxima before scaling
    if ((long long)((T + RP_QT - 1) / RP_QT) * Hq * B > 0x7FFFFFFFLL) return NGC_EUNSUPPORTED;   // one workgroup each
    if ((unsigned long long)T * Hkv * D * 2 > 0xFFFFFFFFull) return NGC_EUNSUPPORTED;   // 32-bit row offsets inside a sequence
    if (T > 65535) return NGC_EUNSUPPORTED;   // 16-bit key lists
    if (ws_bytes < ngc_replay_workspace_bytes(B, T, Hkv)) return NGC_ENOSPC;
    ReplayArgs ra;
    ra.q = reinterpret_cast<const unsigned char *>(q);
    ra.k = reinterpret_cast<const unsigned char *>(k);
    ra.v = reinterpret_cast<const unsigned char *>(v);
    ra.death = death;
    ra.out = out;
    ra.B = B; ra.T = T; ra.Hq = Hq; ra.Hkv = Hkv; ra.Hd = death_per_head ? Hkv : 1;
    ra.scale_log2e = scale * 1.4426950408889634f;
    hipStream_t st = (hipStream_t)stream;
    const int nqt = (T + RP_QT - 1) / RP_QT;
    size_t lists = (size_t)B * ra.Hd * nqt * T * sizeof(uint16_t);
    lists = (lists + 255) & ~(size_t)255;
    ra.klist = reinterpret_cast<uint16_t *>(reinterpret_cast<unsigned char *>(ws) + 256);
    ra.kcount = reinterpret_cast<int32_t *>(reinterpret_cast<unsigned char *>(ws) + 256 + lists);
    size_t counts = (size_t)B * ra.Hd * nqt * sizeof(int32_t);
    counts = (counts + 255) & ~(size_t)255;
    ra.tile_death = reinterpret_cast<int32_t *>(reinterpret_cast<unsigned char *>(ws) + 256 + lists + counts);
    hipLaunchKernelGGL(replay_lists_kernel, dim3(nqt, B * ra.Hd), dim3(RP_WAVES * 64), 0, st, ra);
    NGC_HIP_CHECK(hipGetLastError());
    if (D == 128)
        hipLaunchKernelGGL(replay_attn_kernel<128>, dim3((unsigned)(nqt * Hq * B)), dim3(RP_WAVES * 64), 0, st, ra);
    else
        hipLaunchKernelGGL(replay_attn_kernel<64>, dim3((unsigned)(nqt * Hq * B)), dim3(RP_WAVES * 64), 0, st, ra);
    NGC_HIP_CHECK(hipGetLastError());
    return NGC_OK;
}
