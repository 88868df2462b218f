/*
 * ngc_probe.h -- C ABI of the measurement probes (libngc_probe.so).
 *
 * Not part of the method and not part of libngc.so: plain streaming kernels
 * that a harness times next to the library's own kernels, so that every
 * bandwidth figure can be read against what this machine's memory system gives
 * the plainest code of the same shape.  All pointers are DEVICE pointers,
 * 16-byte aligned; the caller owns every buffer; calls only enqueue on
 * `stream` (a hipStream_t passed as void*, NULL = default stream).  Return
 * value: 0, or -1 for a bad argument, -3 for a failed launch.
 */
#ifndef NGC_PROBE_H
#define NGC_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Stream `bytes` bytes (a multiple of 16) through 16-byte-per-lane kernels.
 *   NGC_PROBE_READ / _READ_NT   read src (plain / nontemporal loads); dst is
 *                               only a sink of >= 16 bytes that is (almost)
 *                               never written
 *   NGC_PROBE_COPY / _COPY_NT   dst[i] = src[i] (plain / nontemporal accesses),
 *                               256 threads, 16 KB per workgroup step
 *   NGC_PROBE_FILL_NT           dst[i] = constant (nontemporal stores) */
#define NGC_PROBE_READ    0
#define NGC_PROBE_COPY    1
#define NGC_PROBE_READ_NT 2
#define NGC_PROBE_COPY_NT 3
#define NGC_PROBE_FILL_NT 4
int ngc_probe_stream(int32_t kind, const void *src, void *dst, size_t bytes, void *stream);

/* A plain copy in a chosen shape: every workgroup of `threads` (256, 512 or
 * 1024) threads walks contiguous chunks of threads * unroll * 16 bytes
 * (unroll 4, 8 or 16), reading a whole chunk into registers before it writes
 * it; `grid` workgroups stride over the buffer (the tail that fills no whole
 * chunk is copied element by element).  pipelined != 0: the loads of the next
 * chunk are issued before the stores of the current one.  Nontemporal
 * accesses.  Unsupported combinations return -1. */
int ngc_probe_copy_shape(const void *src, void *dst, size_t bytes, int32_t threads, int32_t unroll,
                         int32_t grid, int32_t pipelined, void *stream);

/* The access pattern of an in-place cache compaction without any selection
 * work: segment s (one workgroup each) moves, for j < keep[s], the 256-byte
 * rows kept[s][j] of its K and V areas to row j, front to back (kept ascending,
 * kept[s][j] >= j), with the software-pipelined loop the eviction kernel uses.
 *   k, v       nseg areas of cap rows of 256 bytes each (modified in place)
 *   kept       int32 [nseg][max_keep];  keep  int32 [nseg]
 *   threads    256, 512 or 1024;  unroll 2 or 4 (rows in flight per thread)
 *   mode       0 in place; 1 gather reads only; 2 packed writes only */
int ngc_probe_compact(void *k, void *v, const int32_t *kept, const int32_t *keep, int32_t nseg, int32_t cap,
                      int32_t max_keep, int32_t threads, int32_t unroll, int32_t mode, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NGC_PROBE_H */
