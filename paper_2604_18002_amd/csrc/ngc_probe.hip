// Measurement probes (libngc_probe.so): what this machine's memory system
// delivers to the plainest kernels of a given shape -- streaming reads, fills,
// copies in several shapes, and the access pattern of an in-place compaction
// with no selection work around it.  The measurement harness runs them beside
// the library's kernels so that every bandwidth figure can also be read against
// a ceiling measured in the same job.  Nothing here is part of the method.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ngc_probe.h"

namespace ngc_probe {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_THREADS = 256;
constexpr int PROBE_UNROLL = 4;

template <bool NT>
__global__ __launch_bounds__(PROBE_THREADS) void probe_read_kernel(const u32x4 *__restrict__ src, u32x4 *sink, size_t n)
{
    const size_t stride = (size_t)gridDim.x * PROBE_THREADS;
    size_t i = (size_t)blockIdx.x * PROBE_THREADS + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (PROBE_UNROLL - 1) * stride < n; i += PROBE_UNROLL * stride) {
        u32x4 v[PROBE_UNROLL];
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u)
            v[u] = NT ? __builtin_nontemporal_load(src + i + u * stride) : src[i + u * stride];
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u) acc ^= v[u];
    }
    for (; i < n; i += stride) acc ^= NT ? __builtin_nontemporal_load(src + i) : src[i];
    // the loads must not be optimised away; the store itself (almost) never happens
    if (acc[0] == 0x9E3779B9u && acc[1] == 0x7F4A7C15u && acc[2] == 1u) sink[0] = acc;
}

__global__ __launch_bounds__(PROBE_THREADS) void probe_fill_kernel(u32x4 *__restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * PROBE_THREADS;
    const u32x4 v = {0x01010101u, 0x02020202u, 0x03030303u, 0x04040404u};
    for (size_t i = (size_t)blockIdx.x * PROBE_THREADS + threadIdx.x; i < n; i += stride)
        __builtin_nontemporal_store(v, dst + i);
}

// Copy: every workgroup walks contiguous chunks of THREADS * UNROLL * 16 bytes, reading a whole chunk into
// registers before writing it.  PIPE: two register buffers, the next chunk's loads are issued before the stores.
template <int THREADS, int UNROLL, bool NT, bool PIPE>
__global__ __launch_bounds__(THREADS) void probe_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n)
{
    constexpr size_t CHUNK = (size_t)THREADS * UNROLL;
    const size_t step = (size_t)gridDim.x * CHUNK;
    auto load = [&](size_t c, u32x4 (&v)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t i = c + (size_t)u * THREADS + threadIdx.x;
            v[u] = NT ? __builtin_nontemporal_load(src + i) : src[i];
        }
    };
    auto store = [&](size_t c, const u32x4 (&v)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t i = c + (size_t)u * THREADS + threadIdx.x;
            if (NT) __builtin_nontemporal_store(v[u], dst + i);
            else dst[i] = v[u];
        }
    };
    size_t c = (size_t)blockIdx.x * CHUNK;
    if constexpr (!PIPE) {
        for (; c + CHUNK <= n; c += step) {
            u32x4 v[UNROLL];
            load(c, v);
            store(c, v);
        }
    } else {
        u32x4 a[UNROLL], b[UNROLL];
        if (c + CHUNK <= n) {
            load(c, a);
            while (true) {
                const bool more_b = c + step + CHUNK <= n;
                if (more_b) load(c + step, b);
                store(c, a);
                if (!more_b) break;
                c += step;
                const bool more_a = c + step + CHUNK <= n;
                if (more_a) load(c + step, a);
                store(c, b);
                if (!more_a) break;
                c += step;
            }
        }
    }
    // the tail that fills no whole chunk: the workgroup whose turn it would be copies it element by element
    const size_t tail0 = (n / CHUNK) * CHUNK;
    if (blockIdx.x == (n / CHUNK) % gridDim.x)
        for (size_t i = tail0 + threadIdx.x; i < n; i += THREADS) dst[i] = src[i];
}

// In-place compaction pattern, the loop of the eviction kernel with nothing around it (see ngc_probe.h).
// MODE 0: in place; 1: the gather reads only; 2: the packed writes only.
template <int THREADS, int UNROLL, int MODE>
__global__ __launch_bounds__(THREADS) void probe_compact_kernel(unsigned char *k, unsigned char *v, const int32_t *kept_all,
                                                                const int32_t *keep, size_t seg_bytes, int max_keep)
{
    constexpr int ROW_BYTES = 256, PIECES = 16, ROWS_PER_STEP = THREADS / PIECES, TILE_ROWS = ROWS_PER_STEP * UNROLL;
    const int seg = blockIdx.x;
    unsigned char *kbase = k + (size_t)seg * seg_bytes, *vbase = v + (size_t)seg * seg_bytes;
    const int32_t *kept = kept_all + (size_t)seg * max_keep;
    const int rows_new = keep[seg];
    if (rows_new <= 0) return;
    const int rsub = threadIdx.x / PIECES, last = rows_new - 1;
    const uint32_t col = (uint32_t)(threadIdx.x % PIECES) * 16u;
    auto sources = [&](int tile, int (&src)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            int r = tile + u * ROWS_PER_STEP + rsub;
            r = r < last ? r : last;
            src[u] = kept[r];
        }
    };
    auto load = [&](const int (&src)[UNROLL], u32x4 (&kb)[UNROLL], u32x4 (&vb)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t off = (uint32_t)src[u] * ROW_BYTES + col;
            if (MODE == 2) {
                kb[u] = u32x4{1u, 2u, 3u, off};
                vb[u] = u32x4{4u, 5u, 6u, off};
            } else {
                kb[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kbase + off));
                vb[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vbase + off));
            }
        }
    };
    u32x4 sink = {0u, 0u, 0u, 0u};
    auto store_full = [&](int tile, const u32x4 (&kb)[UNROLL], const u32x4 (&vb)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (MODE == 1) {
                sink ^= kb[u];
                sink ^= vb[u];
            } else {
                const uint32_t off = (uint32_t)(tile + u * ROWS_PER_STEP + rsub) * ROW_BYTES + col;
                __builtin_nontemporal_store(kb[u], reinterpret_cast<u32x4 *>(kbase + off));
                __builtin_nontemporal_store(vb[u], reinterpret_cast<u32x4 *>(vbase + off));
            }
        }
    };
    auto store_tail = [&](int tile, const u32x4 (&kb)[UNROLL], const u32x4 (&vb)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int r = tile + u * ROWS_PER_STEP + rsub;
            if (MODE == 1) {
                sink ^= kb[u];
                sink ^= vb[u];
            } else if (r < rows_new) {
                const uint32_t off = (uint32_t)r * ROW_BYTES + col;
                __builtin_nontemporal_store(kb[u], reinterpret_cast<u32x4 *>(kbase + off));
                __builtin_nontemporal_store(vb[u], reinterpret_cast<u32x4 *>(vbase + off));
            }
        }
    };
    u32x4 ka[UNROLL], va[UNROLL], kb[UNROLL], vb[UNROLL];
    int src[UNROLL];
    int tile = 0;
    sources(tile, src);
    load(src, ka, va);
    sources(tile + TILE_ROWS, src);
    while (true) {
        __syncthreads();
        if (tile + TILE_ROWS > rows_new) { store_tail(tile, ka, va); break; }
        load(src, kb, vb);
        sources(tile + 2 * TILE_ROWS, src);
        store_full(tile, ka, va);
        tile += TILE_ROWS;
        __syncthreads();
        if (tile + TILE_ROWS > rows_new) { store_tail(tile, kb, vb); break; }
        load(src, ka, va);
        sources(tile + 2 * TILE_ROWS, src);
        store_full(tile, kb, vb);
        tile += TILE_ROWS;
    }
    if (MODE == 1 && sink[0] == 0x9E3779B9u && sink[1] == 0x7F4A7C15u && sink[2] == 1u)
        *reinterpret_cast<u32x4 *>(kbase) = sink;
}

}  // namespace ngc_probe

using namespace ngc_probe;

namespace {
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
int launched() { return hipGetLastError() == hipSuccess ? 0 : -3; }
}  // namespace

extern "C" int ngc_probe_stream(int32_t kind, const void *src, void *dst, size_t bytes, void *stream)
{
    if (!dst || bytes < 16 || (bytes & 15u) || !aligned16(dst)) return -1;
    if (kind < 0 || kind > NGC_PROBE_FILL_NT) return -1;
    if (kind != NGC_PROBE_FILL_NT && (!src || !aligned16(src))) return -1;
    const size_t n = bytes / 16;
    size_t want = (n + PROBE_THREADS - 1) / PROBE_THREADS;
    const int grid = (int)(want < 16384 ? want : 16384);   // 64 workgroups per CU, grid-stride beyond
    hipStream_t st = (hipStream_t)stream;
    const u32x4 *s = reinterpret_cast<const u32x4 *>(src);
    u32x4 *d = reinterpret_cast<u32x4 *>(dst);
    switch (kind) {
    case NGC_PROBE_READ: hipLaunchKernelGGL(probe_read_kernel<false>, dim3(grid), dim3(PROBE_THREADS), 0, st, s, d, n); break;
    case NGC_PROBE_READ_NT: hipLaunchKernelGGL(probe_read_kernel<true>, dim3(grid), dim3(PROBE_THREADS), 0, st, s, d, n); break;
    case NGC_PROBE_COPY:
        hipLaunchKernelGGL((probe_copy_kernel<256, 4, false, false>), dim3(grid), dim3(256), 0, st, s, d, n);
        break;
    case NGC_PROBE_COPY_NT:
        hipLaunchKernelGGL((probe_copy_kernel<256, 4, true, false>), dim3(grid), dim3(256), 0, st, s, d, n);
        break;
    default: hipLaunchKernelGGL(probe_fill_kernel, dim3(grid), dim3(PROBE_THREADS), 0, st, d, n); break;
    }
    return launched();
}

extern "C" int ngc_probe_copy_shape(const void *src, void *dst, size_t bytes, int32_t threads, int32_t unroll,
                                    int32_t grid, int32_t pipelined, void *stream)
{
    if (!src || !dst || bytes < 16 || (bytes & 15u) || !aligned16(src) || !aligned16(dst)) return -1;
    if (grid < 1 || grid > (1 << 20)) return -1;
    const size_t n = bytes / 16;
    hipStream_t st = (hipStream_t)stream;
    const u32x4 *s = reinterpret_cast<const u32x4 *>(src);
    u32x4 *d = reinterpret_cast<u32x4 *>(dst);
#define NGC_PROBE_CASE(T, U)                                                                                        \
    if (threads == T && unroll == U) {                                                                              \
        if (pipelined) hipLaunchKernelGGL((probe_copy_kernel<T, U, true, true>), dim3(grid), dim3(T), 0, st, s, d, n); \
        else hipLaunchKernelGGL((probe_copy_kernel<T, U, true, false>), dim3(grid), dim3(T), 0, st, s, d, n);       \
        return launched();                                                                                          \
    }
    NGC_PROBE_CASE(256, 4) NGC_PROBE_CASE(256, 8) NGC_PROBE_CASE(256, 16)
    NGC_PROBE_CASE(512, 4) NGC_PROBE_CASE(512, 8)
    NGC_PROBE_CASE(1024, 4) NGC_PROBE_CASE(1024, 8)
#undef NGC_PROBE_CASE
    if (threads == 1024 && unroll == 16 && !pipelined) {
        hipLaunchKernelGGL((probe_copy_kernel<1024, 16, true, false>), dim3(grid), dim3(1024), 0, st, s, d, n);
        return launched();
    }
    return -1;
}

extern "C" int ngc_probe_compact(void *k, void *v, const int32_t *kept, const int32_t *keep, int32_t nseg, int32_t cap,
                                 int32_t max_keep, int32_t threads, int32_t unroll, int32_t mode, void *stream)
{
    if (!k || !v || !kept || !keep || !aligned16(k) || !aligned16(v)) return -1;
    if (nseg < 1 || cap < 1 || max_keep < 1 || max_keep > cap || mode < 0 || mode > 2) return -1;
    if ((long long)cap * 256 > 0x7FFFFFFFLL) return -1;
    const size_t seg_bytes = (size_t)cap * 256;
    hipStream_t st = (hipStream_t)stream;
    unsigned char *kb = reinterpret_cast<unsigned char *>(k), *vb = reinterpret_cast<unsigned char *>(v);
#define NGC_PROBE_CASE(T, U)                                                                                        \
    if (threads == T && unroll == U) {                                                                              \
        if (mode == 0) hipLaunchKernelGGL((probe_compact_kernel<T, U, 0>), dim3(nseg), dim3(T), 0, st, kb, vb, kept, keep, seg_bytes, (int)max_keep); \
        else if (mode == 1) hipLaunchKernelGGL((probe_compact_kernel<T, U, 1>), dim3(nseg), dim3(T), 0, st, kb, vb, kept, keep, seg_bytes, (int)max_keep); \
        else hipLaunchKernelGGL((probe_compact_kernel<T, U, 2>), dim3(nseg), dim3(T), 0, st, kb, vb, kept, keep, seg_bytes, (int)max_keep); \
        return launched();                                                                                          \
    }
    NGC_PROBE_CASE(256, 2) NGC_PROBE_CASE(256, 4) NGC_PROBE_CASE(512, 2) NGC_PROBE_CASE(512, 4)
    NGC_PROBE_CASE(1024, 2) NGC_PROBE_CASE(1024, 4)
#undef NGC_PROBE_CASE
    return -1;
}
