"""Thin ctypes binding of ``libngc.so`` (see ``include/ngc.h``).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch tensors are used as device memory and for the current HIP stream; no
torch operator takes part in the computation.  There is no CPU fallback: a
missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

from ._build import LIB_PATH

NGC_OK = 0
NGC_EINVAL = -1
NGC_ENOSPC = -2
NGC_EHIP = -3
NGC_EUNSUPPORTED = -4

STATUS_WORDS = 64
STATUS_KEEP_CLAMPED = 0
STATUS_LEN_CLAMPED = 1
STATUS_EMPTY_ATTN = 2
STATUS_APPEND_FULL = 3
STATUS_BAD_SIGMA = 4
STATUS_POOL_BOUNDS = 5

EVICT_SELECT_ONLY = 1
EVICT_UNORDERED = 2
EVICT_POOL_HEADS = 4
SCORE_NO_CAUSAL = 1
SCORE_POOL_HEADS = 2

EXPORTS = ("ngc_version", "ngc_strerror", "ngc_workspace_bytes", "ngc_perturbed_keys", "ngc_evict",
           "ngc_subset_logprob", "ngc_cache_append", "ngc_decode_attn", "ngc_score_keys",
           "ngc_subset_logprob_backward", "ngc_replay_attn", "ngc_replay_workspace_bytes",
           "ngc_paged_workspace_bytes", "ngc_paged_evict", "ngc_paged_append", "ngc_paged_decode_attn",
           "ngc_paged_score_keys", "ngc_lmem", "ngc_keep_counts", "ngc_decode_attn_static", "ngc_decode_step")
STATIC_SCRATCH_BYTES = 2 << 20


class NgcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class ngc_cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("len", C.c_void_p), ("pos", C.c_void_p),
                ("L", C.c_int32), ("B", C.c_int32), ("Hkv", C.c_int32), ("Hq", C.c_int32),
                ("D", C.c_int32), ("cap", C.c_int32)]


class ngc_paged_cache(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("pos_pool", C.c_void_p),
                ("table", C.c_void_p), ("len", C.c_void_p), ("free_stack", C.c_void_p),
                ("free_count", C.c_void_p),
                ("L", C.c_int32), ("B", C.c_int32), ("Hkv", C.c_int32), ("Hq", C.c_int32), ("D", C.c_int32),
                ("page_rows", C.c_int32), ("max_pages", C.c_int32), ("num_pages", C.c_int32)]


class ngc_evict_params(C.Structure):
    _fields_ = [("block", C.c_int32), ("share_heads", C.c_int32), ("noise_scale", C.c_float),
                ("round", C.c_uint32), ("seed", C.c_uint64), ("flags", C.c_uint32),
                ("layer_base", C.c_int32), ("seq_base", C.c_int32), ("reserved", C.c_int32)]


_lib = None


def load_library(path: Optional[str] = None) -> C.CDLL:
    """Load the built library.  Raises if it has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    # PyTorch ships its own copy of the HIP runtime.  It has to be in the process before this library
    # pulls in the system's, or the two runtimes would not share streams and launches on torch's streams fail.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it first (python -m paper_2604_18002_amd._build); "
                           "there is no fallback path")
    lib = C.CDLL(path)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    cp, pp = C.POINTER(ngc_cache), C.POINTER(ngc_evict_params)
    lib.ngc_version.argtypes = []
    lib.ngc_version.restype = C.c_int
    lib.ngc_strerror.argtypes = [C.c_int]
    lib.ngc_strerror.restype = C.c_char_p
    lib.ngc_workspace_bytes.argtypes = [cp, i32]
    lib.ngc_workspace_bytes.restype = sz
    lib.ngc_perturbed_keys.argtypes = [cp, i32, vp, pp, vp, vp, sz, vp]
    lib.ngc_perturbed_keys.restype = C.c_int
    lib.ngc_evict.argtypes = [cp, i32, vp, vp, pp, i32, vp, vp, vp, vp, sz, vp]
    lib.ngc_evict.restype = C.c_int
    lib.ngc_subset_logprob.argtypes = [vp, vp, vp, vp, i32, i64, i32, vp, vp, sz, vp]
    lib.ngc_subset_logprob.restype = C.c_int
    lib.ngc_cache_append.argtypes = [cp, i32, vp, vp, vp, vp, sz, vp]
    lib.ngc_cache_append.restype = C.c_int
    lib.ngc_decode_attn.argtypes = [cp, i32, vp, f32, i32, vp, vp, vp, sz, vp]
    lib.ngc_decode_attn.restype = C.c_int
    lib.ngc_decode_step.argtypes = [cp, i32, vp, vp, vp, vp, f32, i32, vp, vp, vp, sz, vp]
    lib.ngc_decode_step.restype = C.c_int
    lib.ngc_decode_attn_static.argtypes = [cp, i32, vp, f32, i32, vp, vp, vp, vp]
    lib.ngc_decode_attn_static.restype = C.c_int
    lib.ngc_subset_logprob_backward.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, vp, vp, vp, sz, vp]
    lib.ngc_subset_logprob_backward.restype = C.c_int
    lib.ngc_replay_workspace_bytes.argtypes = [i32, i32, i32]
    lib.ngc_replay_workspace_bytes.restype = sz
    lib.ngc_replay_attn.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32, vp, vp, sz, vp]
    lib.ngc_replay_attn.restype = C.c_int
    lib.ngc_score_keys.argtypes = [cp, i32, vp, vp, i32, f32, C.c_uint32, i32, vp, vp, sz, vp]
    lib.ngc_score_keys.restype = C.c_int
    gp = C.POINTER(ngc_paged_cache)
    lib.ngc_paged_workspace_bytes.argtypes = [gp]
    lib.ngc_paged_workspace_bytes.restype = sz
    lib.ngc_paged_evict.argtypes = [gp, i32, vp, i64, vp, pp, i32, vp, vp, vp, vp, sz, vp]
    lib.ngc_paged_evict.restype = C.c_int
    lib.ngc_paged_append.argtypes = [gp, i32, vp, vp, vp, vp, sz, vp]
    lib.ngc_paged_append.restype = C.c_int
    lib.ngc_paged_decode_attn.argtypes = [gp, i32, vp, f32, i32, vp, vp, vp, sz, vp]
    lib.ngc_paged_decode_attn.restype = C.c_int
    lib.ngc_paged_score_keys.argtypes = [gp, i32, vp, vp, i32, f32, C.c_uint32, i32, vp, vp, sz, vp]
    lib.ngc_paged_score_keys.restype = C.c_int
    lib.ngc_lmem.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.ngc_lmem.restype = C.c_int
    lib.ngc_keep_counts.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.ngc_keep_counts.restype = C.c_int
    if path == LIB_PATH:
        _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().ngc_strerror(code).decode()


def version() -> int:
    return load_library().ngc_version()


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != NGC_OK:
        raise NgcError(rc, where)


@dataclass
class Cache:
    """Device buffers of a KV cache (torch tensors as plain memory).

    k, v: bf16 [L, B, Hkv, cap, D]; len: int32 [L, B, Hkv]; pos: int32 [L, B, Hkv, cap] or None."""
    k: object
    v: object
    len: object
    pos: object
    Hq: int

    @property
    def shape(self):
        L, B, Hkv, cap, D = self.k.shape
        return L, B, Hkv, cap, D

    def view(self) -> ngc_cache:
        L, B, Hkv, cap, D = self.k.shape
        assert self.k.is_contiguous() and self.v.is_contiguous() and self.len.is_contiguous()
        return ngc_cache(_ptr(self.k), _ptr(self.v), _ptr(self.len), _ptr(self.pos), L, B, Hkv, self.Hq, D, cap)

    @staticmethod
    def allocate(L, B, Hkv, Hq, D, cap, device="cuda", with_pos=False) -> "Cache":
        import torch
        k = torch.zeros(L, B, Hkv, cap, D, dtype=torch.bfloat16, device=device)
        v = torch.zeros_like(k)
        ln = torch.zeros(L, B, Hkv, dtype=torch.int32, device=device)
        pos = torch.zeros(L, B, Hkv, cap, dtype=torch.int32, device=device) if with_pos else None
        return Cache(k, v, ln, pos, Hq)


def make_params(block=1, share_heads=0, noise_scale=1.0, round=0, seed=0, flags=0, layer_base=0,
                seq_base=0) -> ngc_evict_params:
    return ngc_evict_params(block, share_heads, noise_scale, round, seed, flags, layer_base, seq_base, 0)


def ngc_workspace_bytes(cache: Cache, max_keep: int) -> int:
    v = cache.view()
    return int(load_library().ngc_workspace_bytes(C.byref(v), max_keep))


def allocate_workspace(cache: Cache, max_keep: int):
    """A zeroed workspace tensor (uint8) of the size the library asks for."""
    import torch
    return torch.zeros(ngc_workspace_bytes(cache, max_keep), dtype=torch.uint8, device=cache.k.device)


def read_status(ws):
    """Status counters at the start of a workspace (copies to host, synchronises)."""
    return ws[:STATUS_WORDS * 4].view(dtype=_i32()).cpu().tolist()


def _i32():
    import torch
    return torch.int32


def ngc_perturbed_keys(cache: Cache, layer: int, logits, params: ngc_evict_params, keys_out, ws, stream=None):
    v = cache.view()
    _check(load_library().ngc_perturbed_keys(C.byref(v), layer, _ptr(logits), C.byref(params), _ptr(keys_out),
                                             _ptr(ws), ws.numel(), _stream(stream)), "ngc_perturbed_keys")


def ngc_evict(cache: Cache, layer: int, logits, keep, params: ngc_evict_params, max_keep: int,
              kept_out, sigma_out, logp_out, ws, stream=None):
    v = cache.view()
    _check(load_library().ngc_evict(C.byref(v), layer, _ptr(logits), _ptr(keep), C.byref(params), max_keep,
                                    _ptr(kept_out), _ptr(sigma_out), _ptr(logp_out), _ptr(ws), ws.numel(),
                                    _stream(stream)), "ngc_evict")


def ngc_subset_logprob(logits, n_items, sigma, keep, nseg: int, logit_stride: int, sigma_stride: int,
                       logp_out, ws, stream=None):
    _check(load_library().ngc_subset_logprob(_ptr(logits), _ptr(n_items), _ptr(sigma), _ptr(keep), nseg,
                                             logit_stride, sigma_stride, _ptr(logp_out), _ptr(ws), ws.numel(),
                                             _stream(stream)), "ngc_subset_logprob")


def ngc_cache_append(cache: Cache, layer: int, k_new, v_new, new_pos, ws, stream=None):
    v = cache.view()
    _check(load_library().ngc_cache_append(C.byref(v), layer, _ptr(k_new), _ptr(v_new), _ptr(new_pos),
                                           _ptr(ws), ws.numel(), _stream(stream)), "ngc_cache_append")


def ngc_decode_attn(cache: Cache, layer: int, q, scale: float, max_len_hint: int, out, ws, stream=None,
                    lse_out=None):
    v = cache.view()
    _check(load_library().ngc_decode_attn(C.byref(v), layer, _ptr(q), scale, max_len_hint, _ptr(out),
                                          _ptr(lse_out), _ptr(ws), ws.numel(), _stream(stream)), "ngc_decode_attn")


def ngc_decode_step(cache: Cache, layer: int, k_new, v_new, new_pos, q, scale: float, max_len_hint: int, out, ws,
                    stream=None, lse_out=None):
    v = cache.view()
    _check(load_library().ngc_decode_step(C.byref(v), layer, _ptr(k_new), _ptr(v_new), _ptr(new_pos), _ptr(q), scale,
                                          max_len_hint, _ptr(out), _ptr(lse_out), _ptr(ws), ws.numel(),
                                          _stream(stream)), "ngc_decode_step")


def ngc_decode_attn_static(cache: Cache, layer: int, q, scale: float, max_len_hint: int, out, stream=None,
                           lse_out=None, status=None):
    v = cache.view()
    _check(load_library().ngc_decode_attn_static(C.byref(v), layer, _ptr(q), scale, max_len_hint, _ptr(out),
                                                 _ptr(lse_out), _ptr(status), _stream(stream)),
           "ngc_decode_attn_static")


def ngc_score_keys(cache: Cache, layer: int, q_recent, w: int, scale: float, flags: int, block: int,
                   scores_out, ws, stream=None, lse_recent=None):
    v = cache.view()
    _check(load_library().ngc_score_keys(C.byref(v), layer, _ptr(q_recent), _ptr(lse_recent), w, scale, flags, block,
                                         _ptr(scores_out), _ptr(ws), ws.numel(), _stream(stream)),
           "ngc_score_keys")


def ngc_subset_logprob_backward(logits, n_items, sigma, keep, nseg: int, logit_stride: int, sigma_stride: int,
                                max_keep: int, gout, grad_out, ws, stream=None):
    _check(load_library().ngc_subset_logprob_backward(_ptr(logits), _ptr(n_items), _ptr(sigma), _ptr(keep), nseg,
                                                      logit_stride, sigma_stride, max_keep, _ptr(gout),
                                                      _ptr(grad_out), _ptr(ws), ws.numel(), _stream(stream)),
           "ngc_subset_logprob_backward")


def ngc_replay_workspace_bytes(B: int, T: int, Hkv: int) -> int:
    return int(load_library().ngc_replay_workspace_bytes(B, T, Hkv))


def ngc_replay_attn(q, k, v, death, B: int, T: int, Hq: int, Hkv: int, D: int, death_per_head: bool,
                    scale: float, out, ws, stream=None):
    _check(load_library().ngc_replay_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(death), B, T, Hq, Hkv, D,
                                          1 if death_per_head else 0, scale, _ptr(out), _ptr(ws), ws.numel(),
                                          _stream(stream)), "ngc_replay_attn")


# ------------------------------------------------------------- paged layout ---

@dataclass
class PagedCache:
    """Device buffers of a paged KV cache (torch tensors as plain memory).

    k_pool, v_pool: bf16 [num_pages, page_rows, D]; pos_pool: int32 [num_pages, page_rows] or None;
    table: int32 [L, B, Hkv, max_pages]; len: int32 [L, B, Hkv]; free_stack: int32 [num_pages];
    free_count: int32 [1]."""
    k_pool: object
    v_pool: object
    pos_pool: object
    table: object
    len: object
    free_stack: object
    free_count: object
    Hq: int

    @property
    def page_rows(self) -> int:
        return self.k_pool.shape[1]

    @property
    def cap(self) -> int:
        return self.table.shape[3] * self.k_pool.shape[1]

    def view(self) -> ngc_paged_cache:
        num_pages, P, D = self.k_pool.shape
        L, B, Hkv, max_pages = self.table.shape
        for t in (self.k_pool, self.v_pool, self.table, self.len, self.free_stack, self.free_count):
            assert t.is_contiguous()
        return ngc_paged_cache(_ptr(self.k_pool), _ptr(self.v_pool), _ptr(self.pos_pool), _ptr(self.table),
                               _ptr(self.len), _ptr(self.free_stack), _ptr(self.free_count),
                               L, B, Hkv, self.Hq, D, P, max_pages, num_pages)

    @staticmethod
    def allocate(L, B, Hkv, Hq, D, page_rows, max_pages, num_pages, device="cuda", with_pos=False) -> "PagedCache":
        """An empty cache: every page on the free stack (page 0 on top)."""
        import torch
        k = torch.zeros(num_pages, page_rows, D, dtype=torch.bfloat16, device=device)
        v = torch.zeros_like(k)
        pos = torch.zeros(num_pages, page_rows, dtype=torch.int32, device=device) if with_pos else None
        table = torch.full((L, B, Hkv, max_pages), -1, dtype=torch.int32, device=device)
        ln = torch.zeros(L, B, Hkv, dtype=torch.int32, device=device)
        stack = torch.arange(num_pages - 1, -1, -1, dtype=torch.int32, device=device)
        count = torch.full((1,), num_pages, dtype=torch.int32, device=device)
        return PagedCache(k, v, pos, table, ln, stack, count, Hq)


def ngc_paged_workspace_bytes(pc: PagedCache) -> int:
    v = pc.view()
    return int(load_library().ngc_paged_workspace_bytes(C.byref(v)))


def allocate_paged_workspace(pc: PagedCache):
    import torch
    return torch.zeros(ngc_paged_workspace_bytes(pc), dtype=torch.uint8, device=pc.k_pool.device)


def ngc_paged_evict(pc: PagedCache, layer: int, logits, logit_stride: int, keep, params: ngc_evict_params,
                    max_keep: int, kept_out, sigma_out, logp_out, ws, stream=None):
    v = pc.view()
    _check(load_library().ngc_paged_evict(C.byref(v), layer, _ptr(logits), logit_stride, _ptr(keep),
                                          C.byref(params), max_keep, _ptr(kept_out), _ptr(sigma_out),
                                          _ptr(logp_out), _ptr(ws), ws.numel(), _stream(stream)), "ngc_paged_evict")


def ngc_paged_append(pc: PagedCache, layer: int, k_new, v_new, new_pos, ws, stream=None):
    v = pc.view()
    _check(load_library().ngc_paged_append(C.byref(v), layer, _ptr(k_new), _ptr(v_new), _ptr(new_pos),
                                           _ptr(ws), ws.numel(), _stream(stream)), "ngc_paged_append")


def ngc_paged_decode_attn(pc: PagedCache, layer: int, q, scale: float, max_len_hint: int, out, ws, stream=None,
                          lse_out=None):
    v = pc.view()
    _check(load_library().ngc_paged_decode_attn(C.byref(v), layer, _ptr(q), scale, max_len_hint, _ptr(out),
                                                _ptr(lse_out), _ptr(ws), ws.numel(), _stream(stream)),
           "ngc_paged_decode_attn")


def ngc_paged_score_keys(pc: PagedCache, layer: int, q_recent, w: int, scale: float, flags: int, block: int,
                         scores_out, ws, stream=None, lse_recent=None):
    v = pc.view()
    _check(load_library().ngc_paged_score_keys(C.byref(v), layer, _ptr(q_recent), _ptr(lse_recent), w, scale, flags,
                                               block, _ptr(scores_out), _ptr(ws), ws.numel(), _stream(stream)),
           "ngc_paged_score_keys")


def ngc_lmem(logp, rounds, reward, R: int, L: int, B: int, Hkv: int, group: int, adv_out, loss_layer, loss,
             gout, stream=None):
    _check(load_library().ngc_lmem(_ptr(logp), _ptr(rounds), _ptr(reward), R, L, B, Hkv, group, _ptr(adv_out),
                                   _ptr(loss_layer), _ptr(loss), _ptr(gout), _stream(stream)), "ngc_lmem")


def ngc_keep_counts(len_t, seg0: int, nseg: int, cap: int, block: int, num: int, den: int, min_keep: int, keep_out,
                    stream=None):
    _check(load_library().ngc_keep_counts(_ptr(len_t), seg0, nseg, cap, block, num, den, min_keep, _ptr(keep_out),
                                          _stream(stream)), "ngc_keep_counts")
