"""ctypes binding of ``libngc_probe.so`` (see ``include/ngc_probe.h``) and the
copy-ceiling sweep built on it.

The probes are measurement tools, not part of the method: plain streaming
kernels whose rates say what this machine's memory system gives code of a
given shape.  ``python -m paper_2604_18002_amd.probe`` runs the sweep that
backs the copy ceiling quoted next to the eviction kernel's roofline fraction
and prints one line per shape (GB/s counts bytes read + bytes written).
"""
from __future__ import annotations

import argparse
import ctypes as C
import os
from typing import Optional

import numpy as np

from ._build import PROBE_LIB_PATH

READ, COPY, READ_NT, COPY_NT, FILL_NT = 0, 1, 2, 3, 4
EXPORTS = ("ngc_probe_stream", "ngc_probe_copy_shape", "ngc_probe_compact")

_lib = None


class ProbeError(RuntimeError):
    pass


def load_library(path: Optional[str] = None) -> C.CDLL:
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or PROBE_LIB_PATH
    try:
        import torch  # noqa: F401  (its HIP runtime has to be in the process first)
    except ImportError:
        pass
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it first (python -m paper_2604_18002_amd._build)")
    lib = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.ngc_probe_stream.argtypes = [i32, vp, vp, sz, vp]
    lib.ngc_probe_stream.restype = C.c_int
    lib.ngc_probe_copy_shape.argtypes = [vp, vp, sz, i32, i32, i32, i32, vp]
    lib.ngc_probe_copy_shape.restype = C.c_int
    lib.ngc_probe_compact.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp]
    lib.ngc_probe_compact.restype = C.c_int
    if path == PROBE_LIB_PATH:
        _lib = lib
    return lib


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise ProbeError(f"{where}: {'bad argument' if rc == -1 else 'launch failed'} ({rc})")


def ngc_probe_stream(kind: int, src, dst, nbytes: int, stream=None):
    _check(load_library().ngc_probe_stream(kind, None if src is None else src.data_ptr(), dst.data_ptr(), nbytes,
                                           _stream(stream)), "ngc_probe_stream")


def ngc_probe_copy_shape(src, dst, nbytes: int, threads: int, unroll: int, grid: int, pipelined: bool, stream=None):
    _check(load_library().ngc_probe_copy_shape(src.data_ptr(), dst.data_ptr(), nbytes, threads, unroll, grid,
                                               1 if pipelined else 0, _stream(stream)), "ngc_probe_copy_shape")


def ngc_probe_compact(k, v, kept, keep, nseg: int, cap: int, max_keep: int, threads: int, unroll: int, mode: int,
                      stream=None):
    _check(load_library().ngc_probe_compact(k.data_ptr(), v.data_ptr(), kept.data_ptr(), keep.data_ptr(), nseg, cap,
                                            max_keep, threads, unroll, mode, _stream(stream)), "ngc_probe_compact")


# ------------------------------------------------------------------ sweep ---

def _time_ms(fn, reps: int = 4) -> float:
    import torch
    fn()
    torch.cuda.synchronize()
    best = None
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None or ms < best else best
    return best


def streaming_ceilings(nbytes: int = 8 << 30) -> dict:
    """Best-of-4 rates of the plain probes over `nbytes` bytes (GB/s; copies count read + write)."""
    import torch
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    src.fill_(1)
    dst.fill_(2)
    out = {"bytes": nbytes, "what": "libngc_probe.so over %d GiB, best of 4 after a warm-up; copies count read + write"
                                    % (nbytes >> 30)}
    for name, kind, factor in (("read", READ, 1.0), ("read_nontemporal", READ_NT, 1.0), ("fill_nontemporal", FILL_NT, 1.0),
                               ("copy", COPY, 2.0), ("copy_nontemporal", COPY_NT, 2.0)):
        ms = _time_ms(lambda: ngc_probe_stream(kind, src, dst, nbytes))
        out[name + "_GBs"] = factor * nbytes / (ms * 1e-3) / 1e9
    # the best plain copy shape found on this machine: 1024 threads, 128 KB per workgroup step
    ms = _time_ms(lambda: ngc_probe_copy_shape(src, dst, nbytes, 1024, 8, 2048, False))
    out["copy_best_shape_GBs"] = 2.0 * nbytes / (ms * 1e-3) / 1e9
    out["copy_best_shape"] = "1024 threads x 8 x 16 B per workgroup step, 2048 workgroups, nontemporal"
    del src, dst
    torch.cuda.empty_cache()
    return out


def read_ceiling_at(nbytes: int, launches: int, span: int = 8 << 30, trains: int = 6) -> dict:
    """Rate of the plain nontemporal read probe when it runs the way a per-layer kernel does: trains of `launches`
    back-to-back launches of `nbytes` bytes each, every launch over the next region of a `span`-byte buffer (so no
    launch finds its bytes in a cache), HIP events around each train.  A launch of a few hundred MB does not reach
    the rate of one long stream; this is the figure a kernel of that launch size can be held against."""
    import torch
    nbytes = max(4096, int(nbytes) & ~4095)
    src = torch.empty(span, dtype=torch.uint8, device="cuda")
    sink = torch.empty(4096, dtype=torch.uint8, device="cuda")
    src.fill_(1)
    regions = max(1, span // nbytes)
    nxt = 0
    ms = []
    for t in range(trains + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(launches):
            ngc_probe_stream(READ_NT, src[nxt * nbytes:], sink, nbytes)
            nxt = (nxt + 1) % regions
        e1.record()
        torch.cuda.synchronize()
        if t:   # the first train is the warm-up
            ms.append(e0.elapsed_time(e1) / launches)
    del src, sink
    torch.cuda.empty_cache()
    mean = sum(ms) / len(ms)
    return {"bytes_per_launch": nbytes, "launches_per_train": launches, "trains": trains,
            "us_per_launch": 1e3 * mean, "GBs": nbytes / (mean * 1e-3) / 1e9,
            "what": "plain nontemporal read probe, trains of back-to-back launches of this size over successive regions "
                    "of a %d GiB buffer, events around each train" % (span >> 30)}


def compaction_case(nseg: int, cap: int, n_lo: int, n_hi: int, num: int, den: int, seed: int = 12345):
    """Synthetic kept lists of the shape of a benchmark configuration: segment lengths uniform in [n_lo, n_hi],
    ceil(n num / den) rows kept, uniformly at random, ascending.  Returns (kept int32 [nseg, max_keep],
    keep int32 [nseg], rows that change place)."""
    rng = np.random.default_rng(seed)
    n = rng.integers(n_lo, n_hi + 1, size=nseg)
    keep = ((n * num + den - 1) // den).astype(np.int32)
    max_keep = int(keep.max())
    kept = np.zeros((nseg, max_keep), np.int32)
    moved = 0
    for s in range(nseg):
        rows = np.sort(rng.choice(int(n[s]), size=int(keep[s]), replace=False)).astype(np.int32)
        kept[s, :keep[s]] = rows
        moved += int((rows != np.arange(keep[s])).sum())
    return kept, keep, moved


def sweep(nbytes: int = 8 << 30, quick: bool = False):
    """Print the copy-ceiling sweep: plain streams, copy shapes, compaction-shaped copies."""
    import torch
    load_library()
    print(f"# device: {torch.cuda.get_device_name(0)}; 8 TB/s = vendor HBM peak; GB/s = (bytes read + bytes written) / time")
    c = streaming_ceilings(nbytes)
    for k in ("read_GBs", "read_nontemporal_GBs", "fill_nontemporal_GBs", "copy_GBs", "copy_nontemporal_GBs"):
        print(f"stream {k[:-4]:<18} {c[k]:8.0f} GB/s  {c[k] / 8000:.3f} of 8 TB/s", flush=True)
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    src.fill_(1)
    dst.fill_(2)
    shapes = [(256, 4, 16384), (256, 4, 32768), (256, 8, 8192), (256, 16, 4096), (512, 4, 8192), (512, 8, 4096),
              (1024, 4, 4096), (1024, 8, 2048), (1024, 8, 512), (1024, 16, 2048), (1024, 16, 512)]
    for threads, unroll, grid in shapes:
        for pipe in (False, True):
            if pipe and (unroll == 16 or quick):
                continue
            ms = _time_ms(lambda: ngc_probe_copy_shape(src, dst, nbytes, threads, unroll, grid, pipe))
            r = 2.0 * nbytes / (ms * 1e-3) / 1e9
            print(f"copy threads={threads:4d} chunk={threads * unroll * 16 // 1024:3d} KB grid={grid:5d} "
                  f"pipelined={int(pipe)}: {ms:7.3f} ms {r:6.0f} GB/s  {r / 8000:.3f} of 8 TB/s", flush=True)
    del src, dst
    torch.cuda.empty_cache()
    for name, nseg, cap, n_lo, n_hi, num, den in (("configs[2]-shaped", 3584, 4096, 4096, 4096, 1, 3),
                                                  ("configs[3]-shaped", 14336 if not quick else 4096, 8192, 4096, 8192, 2, 5),
                                                  ("configs[4]-shaped (L=4)", 4096 if not quick else 1024, 16384, 16384, 16384, 1, 3)):
        kept_h, keep_h, moved = compaction_case(nseg, cap, n_lo, n_hi, num, den)
        k = torch.empty(nseg, cap, 256, dtype=torch.uint8, device="cuda")
        v = torch.empty_like(k)
        k.fill_(1)
        v.fill_(2)
        kept = torch.from_numpy(kept_h).cuda()
        keep = torch.from_numpy(keep_h).cuda()
        total = moved * 1024.0
        print(f"# compaction pattern, {name}: {nseg} segments of {cap} rows x 256 B (K and V), {moved} rows move, "
              f"{total / 1e9:.2f} GB read + written", flush=True)
        for threads, unroll in ((256, 4), (512, 2), (512, 4), (1024, 2), (1024, 4)):
            ms = _time_ms(lambda: ngc_probe_compact(k, v, kept, keep, nseg, cap, kept.shape[1], threads, unroll, 0), reps=3)
            r = total / (ms * 1e-3) / 1e9
            print(f"compact in place threads={threads:4d} rows in flight per thread={unroll}: {ms:7.3f} ms {r:6.0f} GB/s  "
                  f"{r / 8000:.3f} of 8 TB/s", flush=True)
        for mode, what in ((1, "gather reads only"), (2, "packed writes only")):
            ms = _time_ms(lambda: ngc_probe_compact(k, v, kept, keep, nseg, cap, kept.shape[1], 1024, 4, mode), reps=3)
            r = 0.5 * total / (ms * 1e-3) / 1e9
            print(f"compact {what:<18} threads=1024: {ms:7.3f} ms {r:6.0f} GB/s one way", flush=True)
        del k, v, kept, keep
        torch.cuda.empty_cache()


if __name__ == "__main__":
    ap = argparse.ArgumentParser(description="copy-ceiling sweep on one MI355X")
    ap.add_argument("--gib", type=int, default=8, help="bytes streamed by the plain probes, in GiB")
    ap.add_argument("--quick", action="store_true", help="fewer shapes, smaller compaction cases")
    a = ap.parse_args()
    sweep(a.gib << 30, a.quick)
