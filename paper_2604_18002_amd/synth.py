"""Seeded synthetic inputs shaped like the paper's rollout workloads.

This module only *makes data*: shapes, value distributions and length mixes.
It holds none of the method's arithmetic (no noise, no selection, no softmax)
and is the one module that both the tests of the CPU oracle and the HIP path
read, so that the two see identical bits.

bf16 tensors are produced as uint16 bit patterns (numpy has no bf16).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

DATA_SEED_BASE = 0x4E474300     # + config index
GUMBEL_SEED_BASE = 0x5EED0000   # + config index


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration (shapes only)."""
    name: str
    index: int
    L: int                 # layers
    B: int                 # sequences (rollouts) in the batch
    Hq: int                # query heads
    Hkv: int               # KV heads
    D: int                 # head dim
    n_lo: int              # initial cache rows per sequence: uniform in [n_lo, n_hi]
    n_hi: int
    keep_num: int          # retention rate keep_num / keep_den of the initial cache
    keep_den: int
    delta: int             # eviction cadence (tokens between rounds)
    decode_steps: int
    logits_kind: str       # "normal" | "drift" | "heavy"
    with_logprob: bool
    fixed_keep: Optional[int] = None   # config 0 fixes K directly
    per_head_budget: bool = False      # config 4: the budget of a sequence is split unevenly over heads

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def cap(self) -> int:
        """Allocated rows per (layer, sequence, head): the peak cache."""
        return self.n_hi

    @property
    def data_seed(self) -> int:
        return DATA_SEED_BASE + self.index

    @property
    def gumbel_seed(self) -> int:
        return GUMBEL_SEED_BASE + self.index


WORKLOADS = (
    Workload("tiny", 0, L=1, B=1, Hq=8, Hkv=2, D=64, n_lo=512, n_hi=512, keep_num=1, keep_den=2,
             delta=1, decode_steps=1, logits_kind="normal", with_logprob=True, fixed_keep=256),
    Workload("small-rollout-batch", 1, L=1, B=16, Hq=12, Hkv=2, D=128, n_lo=1024, n_hi=2048,
             keep_num=1, keep_den=2, delta=256, decode_steps=256, logits_kind="normal",
             with_logprob=True),
    Workload("1.5B-shaped", 2, L=28, B=64, Hq=12, Hkv=2, D=128, n_lo=4096, n_hi=4096,
             keep_num=1, keep_den=3, delta=256, decode_steps=1024, logits_kind="drift",
             with_logprob=True),
    Workload("7B-shaped", 3, L=28, B=128, Hq=28, Hkv=4, D=128, n_lo=4096, n_hi=8192,
             keep_num=2, keep_den=5, delta=512, decode_steps=512, logits_kind="normal",
             with_logprob=True),
    Workload("long-reasoning-stress", 4, L=4, B=256, Hq=28, Hkv=4, D=128, n_lo=16384, n_hi=16384,
             keep_num=1, keep_den=3, delta=1024, decode_steps=1024, logits_kind="heavy",
             with_logprob=True, per_head_budget=True),
    # not one of the benchmark configurations: the shape of the paper's own training runs (1.5B model, one
    # group of 16 rollouts, rounds every 350 tokens at a retention of 1/2, so the cache swings between 350
    # and 700 rows): a small-cache case where launch latency, not bandwidth, decides
    Workload("paper-rollout-group", 5, L=28, B=16, Hq=12, Hkv=2, D=128, n_lo=700, n_hi=700,
             keep_num=1, keep_den=2, delta=350, decode_steps=350, logits_kind="normal",
             with_logprob=True),
)


def workload(index: int, **overrides) -> Workload:
    w = WORKLOADS[index]
    if overrides:
        from dataclasses import replace
        w = replace(w, **overrides)
    return w


# ------------------------------------------------------------ bit formats --

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ------------------------------------------------------------ generators ---

_STREAMS = {"len": 1, "k": 2, "v": 3, "q": 4, "logits": 5, "budget": 6, "new": 7}


def _rng(w: Workload, what: str, *ids: int) -> np.random.Generator:
    """Independent stream per (workload, kind, ids...) so that any one segment
    can be generated on its own, in any order."""
    return np.random.default_rng([w.data_seed, _STREAMS[what], *[int(i) for i in ids]])


def lengths(w: Workload) -> np.ndarray:
    """Initial cache rows per sequence, int32 [B] (every layer and head of a
    sequence starts at the same length)."""
    if w.n_lo == w.n_hi:
        return np.full(w.B, w.n_hi, np.int32)
    return _rng(w, "len").integers(w.n_lo, w.n_hi + 1, size=w.B).astype(np.int32)


def segment_kv(w: Workload, l: int, b: int, h: int, n: int) -> Tuple[np.ndarray, np.ndarray]:
    """bf16 N(0,1) K and V rows of one segment, uint16 [n, D] each."""
    k = _rng(w, "k", l, b, h).standard_normal((n, w.D), dtype=np.float32)
    v = _rng(w, "v", l, b, h).standard_normal((n, w.D), dtype=np.float32)
    return f32_to_bf16_bits(k), f32_to_bf16_bits(v)


def new_token_kv(w: Workload, l: int, step: int) -> Tuple[np.ndarray, np.ndarray]:
    """K and V of the token appended at a decode step: uint16 [B, Hkv, D] each."""
    g = _rng(w, "new", l, step)
    k = g.standard_normal((w.B, w.Hkv, w.D), dtype=np.float32)
    v = g.standard_normal((w.B, w.Hkv, w.D), dtype=np.float32)
    return f32_to_bf16_bits(k), f32_to_bf16_bits(v)


def queries(w: Workload, l: int, step: int = 0) -> np.ndarray:
    """bf16 N(0,1) decode queries of one layer: uint16 [B, Hq, D]."""
    q = _rng(w, "q", l, step).standard_normal((w.B, w.Hq, w.D), dtype=np.float32)
    return f32_to_bf16_bits(q)


def segment_logits(w: Workload, l: int, b: int, h: int, n: int, rnd: int = 0) -> np.ndarray:
    """fp32 eviction logits of one segment, [n].

    normal: N(0,1).   drift: N(0,1) + 2 t / n (newer entries score higher).
    heavy:  each entry is N(0,1) w.p. 0.95 and Laplace(0, 4) w.p. 0.05."""
    g = _rng(w, "logits", l, b, h, rnd)
    s = g.standard_normal(n, dtype=np.float32)
    if w.logits_kind == "drift":
        s = s + (np.float32(2.0) * np.arange(n, dtype=np.float32) / np.float32(max(n, 1)))
    elif w.logits_kind == "heavy":
        out = g.random(n) < 0.05
        lap = g.laplace(0.0, 4.0, size=n).astype(np.float32)
        s = np.where(out, lap, s)
    elif w.logits_kind != "normal":
        raise ValueError(w.logits_kind)
    return np.ascontiguousarray(s, dtype=np.float32)


def head_budget_weights(w: Workload, l: int, b: int) -> np.ndarray:
    """Relative shares of a sequence's retention budget over its KV heads
    (all ones unless the workload splits the budget unevenly): float64 [Hkv]."""
    if not w.per_head_budget:
        return np.ones(w.Hkv)
    return _rng(w, "budget", l, b).uniform(0.5, 1.5, size=w.Hkv)


# --------------------------------------------------- bulk fills on device --

def fill_normal_bf16_(t, seed: int, chunk_elems: int = 1 << 28) -> None:
    """Fill a (possibly huge) torch bf16 tensor on its own device with N(0,1)
    values from a seeded generator, chunk by chunk (no fp32 copy of the whole)."""
    import torch
    g = torch.Generator(device=t.device)
    g.manual_seed(int(seed))
    flat = t.view(-1)
    for s in range(0, flat.numel(), chunk_elems):
        e = min(flat.numel(), s + chunk_elems)
        flat[s:e] = torch.randn(e - s, generator=g, device=t.device, dtype=torch.float32).to(torch.bfloat16)


def fill_logits_(t, w: Workload, seed: int, chunk_rows: int = 4096) -> None:
    """Fill a torch fp32 tensor [..., cap] on its device with the workload's
    logit distribution (same recipe as segment_logits, device generator)."""
    import torch
    g = torch.Generator(device=t.device)
    g.manual_seed(int(seed))
    cap = t.shape[-1]
    rows = t.view(-1, cap)
    pos = torch.arange(cap, device=t.device, dtype=torch.float32) / float(cap)
    for s in range(0, rows.shape[0], chunk_rows):
        e = min(rows.shape[0], s + chunk_rows)
        x = torch.randn(e - s, cap, generator=g, device=t.device, dtype=torch.float32)
        if w.logits_kind == "drift":
            x += 2.0 * pos
        elif w.logits_kind == "heavy":
            u = torch.rand(e - s, cap, generator=g, device=t.device)
            v = torch.rand(e - s, cap, generator=g, device=t.device) - 0.5
            lap = -4.0 * torch.sign(v) * torch.log1p(-2.0 * v.abs().clamp(max=0.4999999))
            x = torch.where(u < 0.05, lap, x)
        rows[s:e] = x
