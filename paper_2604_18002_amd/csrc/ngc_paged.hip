// Paged cache layout on gfx950: the blocks of the eviction policy are pages, so
// an eviction round permutes page tables and returns pages to a shared pool
// instead of moving K/V rows; appends take pages from that pool.
//
// Pool operations are ordered by segment id (see ngc.h), which takes a prefix
// sum over the segments of a launch: a single workgroup scans the per-segment
// counts (a few thousand integers), the data-parallel kernels before and after
// it do the per-segment work.
//
// Includes the selection (ngc_select.h), hence compiled with -ffp-contract=off.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ngc.h"
#include "ngc_device.h"
#include "ngc_select.h"

namespace ngc {

struct PagedArgs {
    int32_t *table;
    int32_t *len;
    int32_t *free_stack;
    int32_t *free_count;
    int32_t *freed;       // workspace, int32 per segment: pages a segment gives back
    int32_t *push_base;   // workspace, int32 per segment: where they go on the stack
    int32_t *status;
    int seg0, nseg;
    int page_rows, max_pages, num_pages;
};

// ------------------------------------------------------------- evict ------
//
// One workgroup per segment: the selection over the segment's pages, then the
// table edit.  The old table is staged in LDS (in the area that held the key
// codes) because the edit is an in-place permutation.  Thread j owns kept item
// j and the run of evicted pages just below it; thread K owns the run after the
// last kept item.  An evicted page t with j kept pages below it is the
// (t - j)-th evicted page.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void paged_evict_kernel(SelectArgs a, PagedArgs pa)
{
    constexpr int NW = THREADS / NGC_WAVE;
    constexpr int HIST = (SEL_BINS > SORT_BINS * NW) ? SEL_BINS : SORT_BINS * NW;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    int *misc = reinterpret_cast<int *>(reinterpret_cast<uint32_t *>(smem_raw) + a.items_cap + HIST);
    const int seg = a.seg0 + blockIdx.x;

    select_segment<THREADS, 256>(a, seg, smem_raw);   // a.k == nullptr: the row size is not used
    if (pa.table == nullptr) return;                  // selection only
    __syncthreads();   // misc[], this workgroup's kept_out writes, and the end of all reads of the codes

    const int K = misc[MISC_KEPT];
    const int rows_new = misc[MISC_ROWS];
    int n = a.len[seg];
    n = n < 0 ? 0 : (n > a.g.cap ? a.g.cap : n);      // clamps were counted by the selection
    const int N = (n + pa.page_rows - 1) / pa.page_rows;
    int32_t *tab = pa.table + (size_t)seg * pa.max_pages;
    int32_t *old = reinterpret_cast<int32_t *>(smem_raw);
    for (int i = threadIdx.x; i < N; i += THREADS) old[i] = tab[i];
    __syncthreads();
    const int32_t *kept = a.kept_out + (size_t)seg * a.max_keep;
    for (int j = threadIdx.x; j <= K; j += THREADS) {
        const int lo = (j == 0) ? 0 : kept[j - 1] + 1;
        const int hi = (j < K) ? kept[j] : N;
        if (j < K) tab[j] = old[hi];
        for (int t = lo; t < hi; ++t) tab[K + (t - j)] = old[t];
    }
    if (threadIdx.x == 0) {
        pa.len[seg] = rows_new;
        pa.freed[seg] = N - K;
    }
}

// Exclusive prefix sum of cnt[seg0 .. seg0 + nseg) by one workgroup; `per`
// consecutive segments per thread.  Returns the sum of the thread's own
// segments' predecessors; *total = sum over the launch.
template <int THREADS>
__device__ __forceinline__ int scan_segments(const int32_t *cnt, int seg0, int nseg, int per, int *tmp, int *total)
{
    const int lo = threadIdx.x * per;
    int mine = 0;
    for (int i = lo; i < lo + per && i < nseg; ++i) mine += cnt[seg0 + i];
    return block_excl_scan_i<THREADS>(mine, tmp, total);
}

constexpr int POOL_SCAN_THREADS = 1024;

// Release, step 1: stack position of every segment's first evicted page, and the new free count.
__global__ __launch_bounds__(POOL_SCAN_THREADS) void paged_release_scan_kernel(PagedArgs pa)
{
    __shared__ int tmp[32];
    const int count = *pa.free_count;
    const int per = (pa.nseg + POOL_SCAN_THREADS - 1) / POOL_SCAN_THREADS;
    int total;
    int run = scan_segments<POOL_SCAN_THREADS>(pa.freed, pa.seg0, pa.nseg, per, tmp, &total);
    const int lo = threadIdx.x * per;
    for (int i = lo; i < lo + per && i < pa.nseg; ++i) {
        pa.push_base[pa.seg0 + i] = count + run;
        run += pa.freed[pa.seg0 + i];
    }
    if (threadIdx.x == 0) {
        int c = count + total;
        if (count < 0 || c > pa.num_pages) {
            atomicAdd(&pa.status[NGC_STATUS_POOL_BOUNDS], 1);
            c = c > pa.num_pages ? pa.num_pages : (c < 0 ? 0 : c);
        }
        *pa.free_count = c;
    }
}

// Release, step 2: one wave per segment copies its evicted table entries onto the stack.
__global__ __launch_bounds__(64) void paged_release_push_kernel(PagedArgs pa)
{
    const int seg = pa.seg0 + blockIdx.x;
    const int f = pa.freed[seg];
    if (f <= 0) return;
    int n = pa.len[seg];
    n = n < 0 ? 0 : n;
    const int K = (n + pa.page_rows - 1) / pa.page_rows;   // pages still in use
    const int base = pa.push_base[seg];
    const int32_t *tab = pa.table + (size_t)seg * pa.max_pages;
    for (int r = threadIdx.x; r < f; r += 64) {
        const int at = base + r;
        if (at >= 0 && at < pa.num_pages && K + r < pa.max_pages) pa.free_stack[at] = tab[K + r];
    }
}

// ------------------------------------------------------------- append -----
//
// Grant: the segments whose last page is full, in ascending id, take pages from
// the top of the stack downwards.  One workgroup.
__global__ __launch_bounds__(POOL_SCAN_THREADS) void paged_grant_kernel(PagedArgs pa)
{
    __shared__ int tmp[32];
    const int count_raw = *pa.free_count;
    const int count = count_raw < 0 ? 0 : (count_raw > pa.num_pages ? pa.num_pages : count_raw);
    const int per = (pa.nseg + POOL_SCAN_THREADS - 1) / POOL_SCAN_THREADS;
    const int cap = pa.page_rows * pa.max_pages;
    const int lo = threadIdx.x * per;
    auto needs = [&](int seg) {
        const int n = pa.len[seg];
        return n >= 0 && n < cap && (n & (pa.page_rows - 1)) == 0;
    };
    int mine = 0;
    for (int i = lo; i < lo + per && i < pa.nseg; ++i) mine += needs(pa.seg0 + i) ? 1 : 0;
    int total;
    int rank = block_excl_scan_i<POOL_SCAN_THREADS>(mine, tmp, &total);
    for (int i = lo; i < lo + per && i < pa.nseg; ++i) {
        const int seg = pa.seg0 + i;
        if (!needs(seg)) continue;
        const int page = (rank < count) ? pa.free_stack[count - 1 - rank] : -1;
        pa.table[(size_t)seg * pa.max_pages + pa.len[seg] / pa.page_rows] = page;
        ++rank;
    }
    __syncthreads();   // every thread has read the old count
    if (threadIdx.x == 0) {
        if (count != count_raw) atomicAdd(&pa.status[NGC_STATUS_POOL_BOUNDS], 1);
        *pa.free_count = count > total ? count - total : 0;
    }
}

struct PagedAppendArgs {
    unsigned char *k_pool;
    unsigned char *v_pool;
    int32_t *pos_pool;
    const int32_t *table;
    int32_t *len;
    const unsigned char *k_new;
    const unsigned char *v_new;
    const int32_t *new_pos;
    int32_t *status;
    int seg0, src_seg0;
    int B, Hkv, page_rows, max_pages, num_pages;
};

// One wave per segment: lanes [0, PIECES) copy the K row, the next PIECES the V row.
template <int ROW_BYTES>
__global__ __launch_bounds__(64) void paged_append_kernel(PagedAppendArgs a)
{
    constexpr int PIECES = ROW_BYTES / 16;
    const int seg = a.seg0 + blockIdx.x;
    const int lane = threadIdx.x;
    const int n = a.len[seg];
    int page = -1;
    if (n >= 0 && n < a.page_rows * a.max_pages) page = a.table[(size_t)seg * a.max_pages + n / a.page_rows];
    if (page < 0 || page >= a.num_pages) {
        if (lane == 0) {
            atomicAdd(&a.status[NGC_STATUS_APPEND_FULL], 1);
            if (page >= a.num_pages) atomicAdd(&a.status[NGC_STATUS_POOL_BOUNDS], 1);
        }
        return;
    }
    const size_t row = (size_t)page * a.page_rows + (n & (a.page_rows - 1));
    const size_t src_off = (size_t)(seg - a.src_seg0) * ROW_BYTES;
    if (lane < 2 * PIECES) {
        const bool is_v = lane >= PIECES;
        const int piece = is_v ? lane - PIECES : lane;
        const unsigned char *s = (is_v ? a.v_new : a.k_new) + src_off;
        unsigned char *d = (is_v ? a.v_pool : a.k_pool) + row * ROW_BYTES;
        *reinterpret_cast<uint4 *>(d + piece * 16) = *reinterpret_cast<const uint4 *>(s + piece * 16);
    }
    __syncthreads();
    if (lane == 0) {
        if (a.pos_pool && a.new_pos) a.pos_pool[row] = a.new_pos[(seg / a.Hkv) % a.B];
        a.len[seg] = n + 1;
    }
}

}  // namespace ngc

// ============================================================ host side ====

using namespace ngc;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
constexpr size_t STATUS_BYTES = NGC_STATUS_WORDS * sizeof(int32_t);

int check_paged(const ngc_paged_cache *pc)
{
    if (!pc || !pc->k_pool || !pc->v_pool || !pc->table || !pc->len || !pc->free_stack || !pc->free_count)
        return NGC_EINVAL;
    if (!aligned16(pc->k_pool) || !aligned16(pc->v_pool)) return NGC_EINVAL;
    if (pc->L <= 0 || pc->B <= 0 || pc->Hkv <= 0 || pc->Hq <= 0 || pc->max_pages <= 0 || pc->num_pages <= 0)
        return NGC_EINVAL;
    if (pc->D != 64 && pc->D != 128) return NGC_EINVAL;
    if (pc->Hq % pc->Hkv != 0 || pc->Hq / pc->Hkv > 16) return NGC_EINVAL;
    if (pc->L > 65535 || pc->Hkv > 65534) return NGC_EINVAL;
    if (pc->page_rows < 32 || (pc->page_rows & (pc->page_rows - 1)) != 0) return NGC_EINVAL;
    if (pc->max_pages > 16384) return NGC_EUNSUPPORTED;
    if ((long long)pc->max_pages * pc->page_rows > 0x7FFFFFFFLL / 256) return NGC_EUNSUPPORTED;
    return NGC_OK;
}

int paged_layer_range(const ngc_paged_cache *pc, int layer, int *seg0, int *nseg)
{
    if (layer < -1 || layer >= pc->L) return NGC_EINVAL;
    const int per_layer = pc->B * pc->Hkv;
    *seg0 = layer < 0 ? 0 : layer * per_layer;
    *nseg = layer < 0 ? pc->L * per_layer : per_layer;
    return NGC_OK;
}

size_t paged_select_lds_bytes(int threads, int items_cap, int keep_cap)
{
    const int nw = threads / 64;
    const int hist = (SEL_BINS > SORT_BINS * nw) ? SEL_BINS : SORT_BINS * nw;
    return (size_t)items_cap * 4 + (size_t)hist * 4 + 64 * 4 + (size_t)keep_cap * 2 * 2;
}

PagedArgs paged_args(const ngc_paged_cache *pc, void *ws, int seg0, int nseg)
{
    PagedArgs pa;
    pa.table = pc->table; pa.len = pc->len;
    pa.free_stack = pc->free_stack; pa.free_count = pc->free_count;
    int32_t *meta = reinterpret_cast<int32_t *>(reinterpret_cast<unsigned char *>(ws) + STATUS_BYTES);
    const size_t nseg_total = (size_t)pc->L * pc->B * pc->Hkv;
    pa.freed = meta;
    pa.push_base = meta + nseg_total;
    pa.status = reinterpret_cast<int32_t *>(ws);
    pa.seg0 = seg0; pa.nseg = nseg;
    pa.page_rows = pc->page_rows; pa.max_pages = pc->max_pages; pa.num_pages = pc->num_pages;
    return pa;
}

}  // namespace

extern "C" size_t ngc_paged_workspace_bytes(const ngc_paged_cache *pc)
{
    if (!pc || pc->max_pages <= 0 || pc->page_rows <= 0) return 0;
    // same layout as the contiguous cache of the same logical geometry:
    // [status][2 int32 per segment][split partials of decode attention]
    ngc_cache c{};
    c.L = pc->L; c.B = pc->B; c.Hkv = pc->Hkv; c.Hq = pc->Hq; c.D = pc->D;
    c.cap = pc->max_pages * pc->page_rows;
    return ngc_workspace_bytes(&c, 0);
}

extern "C" int ngc_paged_evict(const ngc_paged_cache *pc, int32_t layer, const float *logits,
                               int64_t logit_stride, const int32_t *keep, const ngc_evict_params *p,
                               int32_t max_keep, int32_t *kept_out, int32_t *sigma_out, float *logp_out,
                               void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_paged(pc);
    if (rc) return rc;
    if (!logits || !keep || !p || !kept_out || !ws || max_keep < 1) return NGC_EINVAL;
    if (p->block != pc->page_rows || logit_stride < pc->max_pages) return NGC_EINVAL;
    if (p->flags & ~NGC_EVICT_SELECT_ONLY) return NGC_EUNSUPPORTED;
    int seg0, nseg;
    rc = paged_layer_range(pc, layer, &seg0, &nseg);
    if (rc) return rc;
    const size_t nseg_total = (size_t)pc->L * pc->B * pc->Hkv;
    if (ws_bytes < STATUS_BYTES + nseg_total * 8) return NGC_ENOSPC;
    if (!aligned16(ws)) return NGC_EINVAL;

    const int items_cap = pc->max_pages;
    int keep_cap = max_keep < items_cap ? max_keep : items_cap;
    keep_cap = (keep_cap + 7) & ~7;
    const int items_cap_al = (items_cap + 3) & ~3;
    const int threads = items_cap > 8192 ? 1024 : (items_cap > 2048 ? 512 : 256);
    const size_t lds = paged_select_lds_bytes(threads, items_cap_al, keep_cap);
    if (lds > 160 * 1024) return NGC_EUNSUPPORTED;

    SelectArgs sa;
    sa.logits = logits; sa.len = pc->len; sa.keep = keep;
    sa.kept_out = kept_out; sa.sigma_out = sigma_out; sa.logp_out = logp_out;
    sa.status = reinterpret_cast<int32_t *>(ws);
    sa.k = nullptr; sa.v = nullptr; sa.pos = nullptr; sa.len_out = nullptr;
    sa.unordered = 0;
    sa.seg0 = seg0; sa.max_keep = max_keep; sa.items_cap = items_cap_al; sa.keep_cap = keep_cap;
    sa.pool_codes = nullptr;
    sa.logit_stride = logit_stride;
    sa.g = SegGeom{pc->B, pc->Hkv, pc->max_pages * pc->page_rows, pc->page_rows};
    sa.na = NoiseArgs{p->seed, p->round, p->noise_scale, p->share_heads, p->layer_base, p->seq_base};

    PagedArgs pa = paged_args(pc, ws, seg0, nseg);
    const bool edit = !(p->flags & NGC_EVICT_SELECT_ONLY);
    if (!edit) pa.table = nullptr;

    hipStream_t st = (hipStream_t)stream;
    const void *fn = threads == 1024 ? reinterpret_cast<const void *>(&paged_evict_kernel<1024>)
                   : threads == 512  ? reinterpret_cast<const void *>(&paged_evict_kernel<512>)
                                     : reinterpret_cast<const void *>(&paged_evict_kernel<256>);
    if (lds > 64 * 1024)
        NGC_HIP_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    void *kargs[] = {&sa, &pa};
    NGC_HIP_CHECK(hipLaunchKernel(fn, dim3(nseg), dim3(threads), kargs, lds, st));
    if (edit) {
        hipLaunchKernelGGL(paged_release_scan_kernel, dim3(1), dim3(POOL_SCAN_THREADS), 0, st, pa);
        NGC_HIP_CHECK(hipGetLastError());
        hipLaunchKernelGGL(paged_release_push_kernel, dim3(nseg), dim3(64), 0, st, pa);
        NGC_HIP_CHECK(hipGetLastError());
    }
    return NGC_OK;
}

extern "C" int ngc_paged_append(const ngc_paged_cache *pc, int32_t layer, const void *k_new,
                                const void *v_new, const int32_t *new_pos,
                                void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_paged(pc);
    if (rc) return rc;
    if (!k_new || !v_new || !ws || !aligned16(k_new) || !aligned16(v_new)) return NGC_EINVAL;
    if (ws_bytes < STATUS_BYTES) return NGC_ENOSPC;
    int seg0, nseg;
    rc = paged_layer_range(pc, layer, &seg0, &nseg);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    PagedArgs pa = paged_args(pc, ws, seg0, nseg);
    hipLaunchKernelGGL(paged_grant_kernel, dim3(1), dim3(POOL_SCAN_THREADS), 0, st, pa);
    NGC_HIP_CHECK(hipGetLastError());
    PagedAppendArgs aa;
    aa.k_pool = reinterpret_cast<unsigned char *>(pc->k_pool);
    aa.v_pool = reinterpret_cast<unsigned char *>(pc->v_pool);
    aa.pos_pool = pc->pos_pool; aa.table = pc->table; aa.len = pc->len;
    aa.k_new = reinterpret_cast<const unsigned char *>(k_new);
    aa.v_new = reinterpret_cast<const unsigned char *>(v_new);
    aa.new_pos = new_pos;
    aa.status = reinterpret_cast<int32_t *>(ws);
    aa.seg0 = seg0; aa.src_seg0 = seg0;
    aa.B = pc->B; aa.Hkv = pc->Hkv;
    aa.page_rows = pc->page_rows; aa.max_pages = pc->max_pages; aa.num_pages = pc->num_pages;
    if (pc->D == 128)
        hipLaunchKernelGGL(paged_append_kernel<256>, dim3(nseg), dim3(64), 0, st, aa);
    else
        hipLaunchKernelGGL(paged_append_kernel<128>, dim3(nseg), dim3(64), 0, st, aa);
    NGC_HIP_CHECK(hipGetLastError());
    return NGC_OK;
}
