"""Shared plumbing of the GPU parity tests: build a cache from the seeded
generators, run the HIP library through its binding, run the oracle on the
same bits segment by segment."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np

import oracle as orc
from paper_2604_18002_amd import schedule, synth


def to_bf16_tensor(u16: np.ndarray, device):
    import torch
    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).view(torch.bfloat16).to(device)


def from_bf16_tensor(t) -> np.ndarray:
    import torch
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@dataclass
class HostCase:
    """Host copy of everything a workload holds, for the segments in `segs`."""
    w: synth.Workload
    lens: np.ndarray                                  # [B] rows per sequence
    keep: np.ndarray                                  # [L, B, Hkv] items kept per segment
    segs: List[Tuple[int, int, int]]                  # segments generated on the host
    k: Dict[Tuple[int, int, int], np.ndarray]         # uint16 [n, D]
    v: Dict[Tuple[int, int, int], np.ndarray]
    logits: Dict[Tuple[int, int, int], np.ndarray]    # fp32 [n_items]


def keep_table(w: synth.Workload, lens: np.ndarray, block: int = 1) -> np.ndarray:
    """Items kept per segment under the workload's budget rule."""
    keep = np.zeros((w.L, w.B, w.Hkv), np.int32)
    for l in range(w.L):
        for b in range(w.B):
            items = (int(lens[b]) + block - 1) // block
            if w.fixed_keep is not None:
                keep[l, b, :] = min(items, w.fixed_keep)
            elif w.per_head_budget:
                total = orc.keep_count(w.Hkv * items, w.keep_num, w.keep_den)
                keep[l, b, :] = schedule.split_budget(total, synth.head_budget_weights(w, l, b),
                                                      np.full(w.Hkv, items))
            else:
                keep[l, b, :] = orc.keep_count(items, w.keep_num, w.keep_den)
    return keep


def host_case(w: synth.Workload, segs: Optional[List[Tuple[int, int, int]]] = None, block: int = 1) -> HostCase:
    lens = synth.lengths(w)
    if segs is None:
        segs = [(l, b, h) for l in range(w.L) for b in range(w.B) for h in range(w.Hkv)]
    k, v, lg = {}, {}, {}
    for (l, b, h) in segs:
        n = int(lens[b])
        k[(l, b, h)], v[(l, b, h)] = synth.segment_kv(w, l, b, h, n)
        lg[(l, b, h)] = synth.segment_logits(w, l, b, h, (n + block - 1) // block)
    return HostCase(w, lens, keep_table(w, lens, block), segs, k, v, lg)


def upload(case: HostCase, device="cuda", with_pos=False, cap=None):
    """Device cache + logits + keep for a fully host-generated case."""
    import torch
    from paper_2604_18002_amd import binding as ngc
    w = case.w
    cap = cap or w.cap
    cache = ngc.Cache.allocate(w.L, w.B, w.Hkv, w.Hq, w.D, cap, device=device, with_pos=with_pos)
    logits = torch.zeros(w.L, w.B, w.Hkv, cap, dtype=torch.float32, device=device)
    hk = np.zeros((w.L, w.B, w.Hkv, cap, w.D), np.uint16)
    hv = np.zeros_like(hk)
    hl = np.zeros((w.L, w.B, w.Hkv, cap), np.float32)
    ln = np.zeros((w.L, w.B, w.Hkv), np.int32)
    for (l, b, h) in case.segs:
        n = case.k[(l, b, h)].shape[0]
        hk[l, b, h, :n] = case.k[(l, b, h)]
        hv[l, b, h, :n] = case.v[(l, b, h)]
        s = case.logits[(l, b, h)]
        hl[l, b, h, :s.size] = s
        ln[l, b, h] = n
    cache.k.copy_(to_bf16_tensor(hk, device))
    cache.v.copy_(to_bf16_tensor(hv, device))
    cache.len.copy_(torch.from_numpy(ln))
    logits.copy_(torch.from_numpy(hl))
    if with_pos:
        cache.pos.copy_(torch.arange(cap, dtype=torch.int32).expand(w.L, w.B, w.Hkv, cap))
    keep = torch.from_numpy(case.keep).to(device)
    return cache, logits, keep


def oracle_logprob(logits: np.ndarray, sigma: np.ndarray) -> float:
    """Eq. 2 literally where that is affordable, else the O(n + K) form (the
    oracle's own tests show the two agree to 1e-12)."""
    if logits.size * max(1, sigma.size) <= 3_000_000:
        return orc.logprob_literal(logits, sigma)
    return orc.logprob_suffix(logits, sigma)


def oracle_evict_segment(case: HostCase, seg, tau, seed, rnd, block=1, share_heads=False):
    """(kept, sigma, logp, k_after, v_after) of one segment from the oracle."""
    l, b, h = seg
    s = case.logits[seg]
    K = int(case.keep[l, b, h])
    hsel = 0xFFFF if share_heads else h
    kept, sigma = orc.evict_select(s, K, tau, seed, rnd, l, b, hsel)
    lp = oracle_logprob(s, sigma)
    k_after = orc.compact_rows(case.k[seg], kept, block)
    v_after = orc.compact_rows(case.v[seg], kept, block)
    return kept, sigma, lp, k_after, v_after
