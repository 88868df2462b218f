#!/usr/bin/env python3
"""Benchmark of the NGC hot path on one MI355X.

A *step* is one grow-then-evict period of the whole batch: `delta` decode
token-steps, each of them L launches of ngc_decode_step (one per layer, the
way a model has to call it: layer l + 1's query depends on layer l's output;
every launch appends the new K/V row of its layer and attends over the
surviving rows), followed by one eviction round (Gumbel-top-k sample +
ordered-subset log-probability + in-place compaction, all layers in one
launch) that brings every segment back to its budget.  Inputs are synthetic,
seeded, and resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is tokens/s of the whole cycle; the
attention-only rate, the round-0 eviction time at peak cache, the roofline
fractions (against the 8 TB/s vendor figure and against read / copy ceilings
measured in the same job), the same decode steps with all layers in one launch
(secondary), the decode / eviction fractions of the other two configurations
the target is quoted on, the other entry points' timings, the same cycle over
the paged layout and the CPU oracle's rate are reported beside it.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "decode-attn tokens/s + eviction-step µs over evicted cache; % HBM peak"
HBM_PEAK_GBS = 8000.0

# HBM traffic per dispatch (bytes) from rocprofv3 --pmc FETCH_SIZE and --pmc
# WRITE_SIZE runs of this command on the stock workloads, each counter scaled
# by what it reads for a plain 1 GiB copy.  These are NOT counters of the run
# that prints the line: they are copied from the committed summaries named
# below and are reported together with that source.  Keyed by (config, L, B);
# other shapes report null.  "decode" is one per-layer launch at the mean
# length of a period.
PROFILE_TRAFFIC = {
    (2, 28, 64): {"file": "profiles/config2_kernels.txt"},
    (3, 28, 128): {"file": "profiles/config3_kernels.txt"},
    (4, 4, 256): {"file": "profiles/config4_kernels.txt"},
}


def profile_traffic(key, which):
    """(bytes per dispatch, source) parsed from the committed summary, or (None, None)."""
    ent = PROFILE_TRAFFIC.get(key)
    if not ent:
        return None, None
    path = os.path.join(ROOT, ent["file"])
    tag = {"decode": "bench-line traffic decode_per_layer:", "decode_batched": "bench-line traffic decode_batched:",
           "evict": "bench-line traffic evict_round0:"}[which]
    try:
        for line in open(path):
            if line.strip().startswith(tag):
                return float(line.split(":", 1)[1].split()[0]), ent["file"]
    except OSError:
        pass
    return None, None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="index into BASELINE.json configs (default 3: 7B-shaped); 5 = the small-cache shape of the paper's "
                         "own runs (latency-bound, see --per-layer)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (0 = the workload's)")
    ap.add_argument("--batch", type=int, default=0, help="override the number of sequences (0 = the workload's)")
    ap.add_argument("--evict-reps", type=int, default=10, help="timed repetitions of the round-0 eviction")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-layer", action="store_true", default=True,
                    help="also time decode attention launched layer by layer, eagerly and from a HIP graph (default)")
    ap.add_argument("--no-per-layer", dest="per_layer", action="store_false", help="skip the layer-by-layer timing")
    ap.add_argument("--no-paged", action="store_true", help="skip the paged-layout section")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the streaming read / copy probes")
    ap.add_argument("--only-replay", action="store_true",
                    help="run only the replay-attention section (for counter runs of that kernel) and print its JSON")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short eviction / decode measurement of the other configurations among configs[2..4]")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy first (reference dispatch for the HBM byte counters)")
    return ap.parse_args()


def build_workload(args):
    from paper_2604_18002_amd import synth
    over = {}
    if args.layers:
        over["L"] = args.layers
    if args.batch:
        over["B"] = args.batch
    return synth.workload(args.config, **over)


def keep_budget(w, lens):
    """Items kept per segment: the retention budget fixed at round 0."""
    from paper_2604_18002_amd import schedule, synth
    keep = np.zeros((w.L, w.B, w.Hkv), np.int32)
    for b in range(w.B):
        n = int(lens[b])
        if w.fixed_keep is not None:
            keep[:, b, :] = min(n, w.fixed_keep)
        elif w.per_head_budget:
            total = schedule.keep_count(w.Hkv * n, w.keep_num, w.keep_den)
            for l in range(w.L):
                keep[l, b, :] = schedule.split_budget(total, synth.head_budget_weights(w, l, b), np.full(w.Hkv, n))
        else:
            keep[:, b, :] = schedule.keep_count(n, w.keep_num, w.keep_den)
    return keep


def attn_bytes(w, seg_rows_total: int, nseg: int) -> float:
    """Algorithmic bytes of one decode-attention launch: every surviving K and V
    row once (bf16), plus the queries (bf16) and outputs (fp32)."""
    return seg_rows_total * 2 * w.D * 2 + nseg * w.G * w.D * (2 + 4)


def evict_bytes(w, n_items: np.ndarray, keep: np.ndarray, moved_rows: float, with_sigma=True, with_logp=True) -> float:
    """Algorithmic bytes of one eviction round: logits read once, kept (and
    sigma) written, every row that changes place read and written once in K and
    V, one log-probability per segment."""
    b = 4.0 * n_items.sum() + 4.0 * keep.sum() * (2 if with_sigma else 1)
    b += moved_rows * (2 * w.D) * 2 * 2
    if with_logp:
        b += 4.0 * keep.size
    return b


def layer_step_calls(ngc, cache, k_new, v_new, q, scale, hint, out, ws):
    """A function that issues one ngc_decode_step per layer (append + attention), with the C arguments of every
    layer built once."""
    import ctypes as C
    import torch
    lib = ngc.load_library()
    view = cache.view()
    L = cache.k.shape[0]
    stream = torch.cuda.current_stream().cuda_stream
    fn = lib.ngc_decode_step
    vref = C.byref(view)
    calls = [(vref, l, k_new[l].data_ptr(), v_new[l].data_ptr(), None, q[l].data_ptr(), scale, hint,
              out[l].data_ptr(), None, ws.data_ptr(), ws.numel(), stream) for l in range(L)]

    def run():
        for a in calls:
            rc = fn(*a)
            if rc != 0:
                raise ngc.NgcError(rc, "ngc_decode_step")
    run.keepalive = (view, k_new, v_new, q, out, ws)
    return run


def quick_config(ngc, synth, w, dev, samples=32, evict_reps=3, with_ceiling=False):
    """Round-0 and steady-state eviction, and decode steps at `samples` lengths spread over a period (one launch
    per layer, and all layers in one launch), of one workload; a few seconds."""
    import torch
    lens = synth.lengths(w)
    keep_h = keep_budget(w, lens)
    max_keep = int(keep_h.max())
    nseg = w.L * w.B * w.Hkv
    cache = ngc.Cache.allocate(w.L, w.B, w.Hkv, w.Hq, w.D, w.cap, device=dev)
    synth.fill_normal_bf16_(cache.k, w.data_seed * 2 + 0)
    synth.fill_normal_bf16_(cache.v, w.data_seed * 2 + 1)
    logits = torch.empty(w.L, w.B, w.Hkv, w.cap, dtype=torch.float32, device=dev)
    synth.fill_logits_(logits, w, w.data_seed * 2 + 2)
    len0 = torch.from_numpy(np.broadcast_to(lens[None, :, None], (w.L, w.B, w.Hkv)).copy()).to(dev)
    keep = torch.from_numpy(keep_h).to(dev)
    ws = ngc.allocate_workspace(cache, max_keep)
    kept = torch.empty(w.L, w.B, w.Hkv, max_keep, dtype=torch.int32, device=dev)
    sigma = torch.empty_like(kept)
    logp = torch.empty(w.L, w.B, w.Hkv, dtype=torch.float32, device=dev)
    g = torch.Generator(device=dev)
    g.manual_seed(w.data_seed * 2 + 3)
    q = torch.randn(w.L, w.B, w.Hq, w.D, generator=g, device=dev).to(torch.bfloat16)
    k_new = torch.randn(w.L, w.B, w.Hkv, w.D, generator=g, device=dev).to(torch.bfloat16)
    v_new = torch.randn(w.L, w.B, w.Hkv, w.D, generator=g, device=dev).to(torch.bfloat16)
    out = torch.empty(w.L, w.B, w.Hq, w.D, dtype=torch.float32, device=dev)
    scale = 1.0 / math.sqrt(w.D)
    hint = max_keep + w.delta
    slot = torch.arange(max_keep, device=dev, dtype=torch.int32)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def evict(rnd):
        ngc.ngc_evict(cache, -1, logits, keep, ngc.make_params(noise_scale=1.0, round=rnd, seed=w.gumbel_seed),
                      max_keep, kept, sigma if w.with_logprob else None, logp if w.with_logprob else None, ws)

    def timed(fn):
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def moved_rows():
        return float(((kept != slot) & (slot < keep.unsqueeze(-1))).sum().item())

    p1 = []
    for rep in range(evict_reps + 1):
        cache.len.copy_(len0)
        ms = timed(lambda: evict(0))
        if rep:
            p1.append(ms)
    n0 = np.broadcast_to(lens[None, :, None], keep_h.shape)
    p1_bytes = evict_bytes(w, n0, keep_h, moved_rows(), w.with_logprob, w.with_logprob)
    steady = []
    for rep in range(3):
        cache.len.copy_(keep + w.delta)
        steady.append(timed(lambda: evict(1 + rep)))
    st_bytes = evict_bytes(w, keep_h + w.delta, keep_h, moved_rows(), w.with_logprob, w.with_logprob)
    # decode steps at lengths spread over a period
    step_call = layer_step_calls(ngc, cache, k_new, v_new, q, scale, hint, out, ws)
    offs = sorted(set(int(round(x)) for x in np.linspace(0, w.delta - 1, samples)))
    pl_ms = pl_b = ba_ms = ba_b = 0.0
    for warm in (True, False):
        for t in offs:
            cache.len.copy_(keep + t)
            ms = timed(step_call)
            if not warm:
                pl_ms += ms
                pl_b += attn_bytes(w, int(keep_h.sum()) + (t + 1) * nseg, nseg)
            cache.len.copy_(keep + t)
            ms = timed(lambda: ngc.ngc_decode_step(cache, -1, k_new, v_new, None, q, scale, hint, out, ws))
            if not warm:
                ba_ms += ms
                ba_b += attn_bytes(w, int(keep_h.sum()) + (t + 1) * nseg, nseg)
            if warm and t >= offs[1]:
                break
    # the per-layer token-step from a HIP graph at the mid-period length (no host work between launches)
    cache.len.copy_(keep + w.delta // 2)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for l in range(w.L):
            ngc.ngc_decode_attn(cache, l, q[l], scale, hint, out[l], ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gph):
        for l in range(w.L):
            ngc.ngc_decode_attn(cache, l, q[l], scale, hint, out[l], ws)
    gph.replay()
    g_ms = timed(lambda: [gph.replay() for _ in range(10)]) / 10
    g_bytes = attn_bytes(w, int(keep_h.sum()) + (w.delta // 2) * nseg, nseg)
    del gph
    status = ngc.read_status(ws)
    assert all(x == 0 for x in status), f"config {w.index}: device status words not clean: {status[:8]}"
    p1_ms, st_ms = float(np.mean(p1)), float(np.mean(steady[1:]))
    read_at = None
    if with_ceiling:
        from paper_2604_18002_amd import probe
        read_at = probe.read_ceiling_at(int(pl_b / len(offs) / w.L), w.L)
    return {
        "decode_per_layer_frac_of_read_probe_at_launch_size":
            (pl_b / (pl_ms * 1e-3) / 1e9 / read_at["GBs"]) if read_at else None,
        "read_probe_at_decode_launch_size": read_at,
        "workload": f"configs[{w.index}] {w.name}: L={w.L} B={w.B} Hq/Hkv={w.Hq}/{w.Hkv} D={w.D} peak cache "
                    f"{w.n_lo}..{w.n_hi}, keep {w.keep_num}/{w.keep_den}, delta={w.delta}",
        "eviction_step_us": 1e3 * p1_ms, "eviction_hbm_frac": p1_bytes / (p1_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "eviction_step_us_steady": 1e3 * st_ms, "eviction_steady_hbm_frac": st_bytes / (st_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "decode_per_layer_ms_per_token_step": pl_ms / len(offs),
        "decode_per_layer_hbm_frac": pl_b / (pl_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "decode_per_layer_tokens_per_s": w.B * len(offs) / (pl_ms * 1e-3),
        "decode_per_layer_hip_graph_ms_per_token_step": g_ms,
        "decode_per_layer_hip_graph_hbm_frac": g_bytes / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "decode_all_layers_per_launch_ms": ba_ms / len(offs),
        "decode_all_layers_per_launch_hbm_frac": ba_b / (ba_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "what": f"eviction: mean of {evict_reps} round-0 launches at peak cache and of 2 steady-state rounds; decode: "
                f"{len(offs)} token-steps at lengths spread over a period, HIP events around each token-step",
    }


def replay_case(ngc, w, g, dev, block):
    """Replay attention (training forward under the replay mask), one layer, paper-like rounds."""
    import torch
    scale = 1.0 / math.sqrt(w.D)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    Bt, T = 8, 4096
    rs = np.random.default_rng(w.data_seed + block)
    death_h = np.full((Bt, T), T, np.int32)
    for bb in range(Bt):
        alive = np.zeros(0, np.int64)
        for bnd in range(w.delta, T, w.delta):
            alive = np.concatenate([alive, np.arange(bnd - w.delta, bnd)])
            nb = (alive.size + block - 1) // block
            keep_b = rs.random(nb) < (w.keep_num / w.keep_den) ** (w.delta / max(1.0, alive.size / 2))
            keep_t = np.repeat(keep_b, block)[:alive.size]
            death_h[bb, alive[~keep_t]] = bnd
            alive = alive[keep_t]
    qT = torch.randn(Bt, T, w.Hq, w.D, generator=g, device=dev).to(torch.bfloat16)
    kT = torch.randn(Bt, T, w.Hkv, w.D, generator=g, device=dev).to(torch.bfloat16)
    vT = torch.randn(Bt, T, w.Hkv, w.D, generator=g, device=dev).to(torch.bfloat16)
    oT = torch.empty(Bt, T, w.Hq, w.D, dtype=torch.float32, device=dev)
    dT = torch.from_numpy(death_h).to(dev)
    wsT = torch.zeros(ngc.ngc_replay_workspace_bytes(Bt, T, w.Hkv), dtype=torch.uint8, device=dev)
    # a train of back-to-back calls (the training forward pass issues one per layer): the first few run while
    # the clocks are still rising, the mean is taken over the rest
    warm, timed_calls = 10, 20
    for rep in range(warm):
        ngc.ngc_replay_attn(qT, kT, vT, dT, Bt, T, w.Hq, w.Hkv, w.D, False, scale, oT, wsT)
    e0, e1 = ev(), ev()
    e0.record()
    for rep in range(timed_calls):
        ngc.ngc_replay_attn(qT, kT, vT, dT, Bt, T, w.Hq, w.Hkv, w.D, False, scale, oT, wsT)
    e1.record()
    torch.cuda.synchronize()
    t_ms = e0.elapsed_time(e1) / timed_calls
    ii = np.arange(T)
    visible = sum(int(((ii[:, None] >= ii[None, :]) & (ii[:, None] < death_h[bb][None, :])).sum()) for bb in range(Bt))
    flops = 4.0 * w.D * visible * w.Hq
    causal = 4.0 * w.D * (T * (T + 1) / 2) * w.Hq * Bt
    # what the kernel issues: per tile of 128 queries, the keys visible to any of them, rounded up to 32,
    # times 128 query rows, times 6 D flops per pair (QK, PV with P in two bf16 parts)
    issued_pairs = 0
    for bb in range(Bt):
        for i0 in range(0, T, 128):
            last = min(i0 + 127, T - 1)
            n_list = int((death_h[bb][:last + 1] > i0).sum())
            issued_pairs += ((n_list + 31) // 32) * 32 * 128
    issued = 6.0 * w.D * issued_pairs * w.Hq
    return {"block": block, "B": Bt, "T": T, "ms": t_ms, "visible_pairs_frac_of_causal": flops / causal,
            "algorithmic_tflops": flops / (t_ms * 1e-3) / 1e12,
            "mfma_frac": flops / (t_ms * 1e-3) / 1e12 / 2500.0,
            "causal_equivalent_tflops": causal / (t_ms * 1e-3) / 1e12,
            "issued_mfma_tflops": issued / (t_ms * 1e-3) / 1e12,
            "issued_mfma_frac": issued / (t_ms * 1e-3) / 1e12 / 2500.0}



def _cpu_segment_work(w, keep, n_after_mid, kbits, vbits, seg):
    """One segment's share of a period on the oracle: (seconds of eviction, seconds of one decode-attention step)."""
    import oracle as orc
    from paper_2604_18002_amd import synth
    l, b, h = seg
    K = int(keep[l, b, h])
    n = K + w.delta
    s = synth.segment_logits(w, l, b, h, n, rnd=1)
    q = synth.queries(w, l)
    t0 = time.perf_counter()
    kept, sigma = orc.evict_select(s, K, 1.0, w.gumbel_seed, 1, l, b, h)
    if w.with_logprob:
        orc.logprob_suffix(s, sigma)
    orc.compact_rows(kbits[:n], kept)
    orc.compact_rows(vbits[:n], kept)
    t_evict = time.perf_counter() - t0
    m = int(n_after_mid[l, b, h])
    t0 = time.perf_counter()
    orc.decode_attn(q[b, h * w.G:(h + 1) * w.G], kbits[:m], vbits[:m], 1.0 / math.sqrt(w.D))
    return t_evict, time.perf_counter() - t0


def cpu_baseline(w, lens, keep, n_after_mid, budget_s=8.0):
    """The oracle, as it stands, timed on segments of the workload: per segment one eviction round at the
    steady-state size (select + log-prob + compaction) and one decode-attention step at the mid-period length,
    scaled to a whole period (delta token-steps, all segments).  Two legs of about `budget_s` seconds each: one
    thread, then one thread per host core given to this job (the oracle is C behind ctypes, which releases the
    interpreter lock, so plain threads run it in parallel)."""
    from concurrent.futures import ThreadPoolExecutor
    from paper_2604_18002_amd import synth
    rng = np.random.default_rng(w.data_seed)
    kmax = int(keep.max()) + w.delta
    kbits = synth.f32_to_bf16_bits(rng.standard_normal((kmax, w.D), dtype=np.float32))
    vbits = synth.f32_to_bf16_bits(rng.standard_normal((kmax, w.D), dtype=np.float32))
    segs = [(l, b, h) for l in range(w.L) for b in range(w.B) for h in range(w.Hkv)]
    total_segs = len(segs)
    # ---- one thread
    t_evict = t_attn = 0.0
    n1 = 0
    for seg in segs:
        te, ta = _cpu_segment_work(w, keep, n_after_mid, kbits, vbits, seg)
        t_evict += te
        t_attn += ta
        n1 += 1
        if t_evict + t_attn >= budget_s:
            break
    per_seg_period = (t_evict + w.delta * t_attn) / n1       # seconds of CPU per segment and period
    one = w.B * w.delta / (per_seg_period * total_segs)
    # ---- every core of this job (the GPU machines give a one-GPU job 16 cores, whatever os.cpu_count() shows)
    cores_total = os.cpu_count() or 1
    try:
        cores_total = min(cores_total, len(os.sched_getaffinity(0)))
    except (AttributeError, OSError):
        pass
    workers = max(1, min(cores_total, 16))
    per_seg_s = (t_evict + t_attn) / n1
    nn = max(workers, min(total_segs - n1, int(budget_s * workers / max(per_seg_s, 1e-6))))
    batch = segs[n1:n1 + nn] if n1 + nn <= total_segs else segs[:nn]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=workers) as ex:
        res = list(ex.map(lambda sg: _cpu_segment_work(w, keep, n_after_mid, kbits, vbits, sg), batch))
    wall = time.perf_counter() - t0
    te_all, ta_all = sum(r[0] for r in res), sum(r[1] for r in res)
    # wall time per segment with all workers busy, split between the two phases in proportion to their CPU time
    wall_per_seg = wall / len(batch)
    share_attn = ta_all / (te_all + ta_all)
    period_all = (wall_per_seg * (1 - share_attn) + w.delta * wall_per_seg * share_attn) * total_segs
    return {
        "value": one, "unit": "tokens/s", "cores": 1, "kind": "oracle",
        "sample": f"{n1} of {total_segs} (layer, sequence, head) segments: per segment one eviction round "
                  f"(select + log-prob + compaction, budget + delta -> budget) and one decode-attention step at "
                  f"mid-period length; scaled to all segments and {w.delta} token-steps per period; "
                  f"fp64 single-threaded oracle",
        "eviction_step_us": 1e6 * t_evict / n1 * total_segs,
        "decode_attn_tokens_per_s": w.B / (t_attn / n1 * total_segs),
        "cpu_seconds": t_evict + t_attn,
        "cores_total": cores_total,
        "all_cores": {
            "value": w.B * w.delta / period_all, "unit": "tokens/s", "cores": workers, "kind": "oracle",
            "sample": f"{len(batch)} further segments, same work per segment, {workers} threads (one per host core of "
                      f"this job; {cores_total} visible), wall {wall:.1f} s",
            "eviction_step_us": 1e6 * wall_per_seg * (1 - share_attn) * total_segs,
            "decode_attn_tokens_per_s": w.B / (wall_per_seg * share_attn * total_segs),
        },
    }


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; every rollout is independent, so more GPUs would only "
              "replicate this run on disjoint sequences. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_18002_amd import binding as ngc
    from paper_2604_18002_amd import synth

    ngc.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda"
    torch.cuda.set_device(0)
    w = build_workload(args)
    if args.only_replay:
        g = torch.Generator(device=dev)
        g.manual_seed(w.data_seed * 2 + 3)
        print(json.dumps({"replay_attn": {"per_token_eviction": replay_case(ngc, w, g, dev, 1),
                                          "block32_eviction": replay_case(ngc, w, g, dev, 32)}}), flush=True)
        return
    t_setup = time.time()

    if args.copy_calibration:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        a.fill_(1)
        b.copy_(a)          # the plain copy of known size: 1 GiB read, 1 GiB written
        torch.cuda.synchronize()
        del a, b

    # ------------------------------------------- streaming ceilings, same job
    # (libngc_probe.so: what this machine gives the plainest read, fill and copy kernels over 8 GiB)
    ceilings = None
    if not args.no_ceilings:
        from paper_2604_18002_amd import probe
        ceilings = probe.streaming_ceilings(8 << 30)

    # ---------------------------------------------------------------- inputs
    lens = synth.lengths(w)                                   # [B] peak rows per sequence
    keep_h = keep_budget(w, lens)                             # [L,B,Hkv]
    max_keep = int(keep_h.max())
    cap = w.cap
    cache = ngc.Cache.allocate(w.L, w.B, w.Hkv, w.Hq, w.D, cap, device=dev)
    synth.fill_normal_bf16_(cache.k, w.data_seed * 2 + 0)
    synth.fill_normal_bf16_(cache.v, w.data_seed * 2 + 1)
    logits = torch.empty(w.L, w.B, w.Hkv, cap, dtype=torch.float32, device=dev)
    synth.fill_logits_(logits, w, w.data_seed * 2 + 2)
    len0 = torch.from_numpy(np.broadcast_to(lens[None, :, None], (w.L, w.B, w.Hkv)).copy()).to(dev)
    keep = torch.from_numpy(keep_h).to(dev)
    ws = ngc.allocate_workspace(cache, max_keep)
    nseg = w.L * w.B * w.Hkv
    kept = torch.empty(w.L, w.B, w.Hkv, max_keep, dtype=torch.int32, device=dev)
    sigma = torch.empty_like(kept)
    logp = torch.empty(w.L, w.B, w.Hkv, dtype=torch.float32, device=dev)
    g = torch.Generator(device=dev)
    g.manual_seed(w.data_seed * 2 + 3)
    q = torch.randn(w.L, w.B, w.Hq, w.D, generator=g, device=dev).to(torch.bfloat16)
    k_new = torch.randn(w.L, w.B, w.Hkv, w.D, generator=g, device=dev).to(torch.bfloat16)
    v_new = torch.randn(w.L, w.B, w.Hkv, w.D, generator=g, device=dev).to(torch.bfloat16)
    out = torch.empty(w.L, w.B, w.Hq, w.D, dtype=torch.float32, device=dev)
    scale = 1.0 / math.sqrt(w.D)
    hint = max_keep + w.delta
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def evict(rnd, flags=0):
        ngc.ngc_evict(cache, -1, logits, keep,
                      ngc.make_params(noise_scale=1.0, round=rnd, seed=w.gumbel_seed, flags=flags),
                      max_keep, kept, sigma if w.with_logprob else None, logp if w.with_logprob else None, ws)

    # ------------------------------------- P1: round-0 eviction at peak cache
    # (the rows' values do not matter for timing, so only `len` is restored)
    p1_ms = []
    for rep in range(args.evict_reps + 1):
        cache.len.copy_(len0)
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        evict(0)
        e1.record()
        torch.cuda.synchronize()
        if rep > 0:
            p1_ms.append(e0.elapsed_time(e1))
    slot = torch.arange(max_keep, device=dev, dtype=torch.int32)

    def moved_rows():
        """Rows of the last round that changed place (kept index != slot)."""
        valid = slot < keep.unsqueeze(-1)
        return float(((kept != slot) & valid).sum().item())

    moved0 = moved_rows()
    n_items0 = np.broadcast_to(lens[None, :, None], keep_h.shape)
    p1_bytes = evict_bytes(w, n_items0, keep_h, moved0, w.with_logprob, w.with_logprob)
    p1_us = 1e3 * float(np.mean(p1_ms))

    # ------------------------------------------- steady-state periods (steps)
    # One launch per layer and token-step.  The launches go through the library's C entry point directly with
    # their arguments marshalled once (what the binding would build on every call), so that the host never is
    # what the GPU waits for.
    rows_after = int(keep_h.sum())             # rows in use right after a round
    step_call = layer_step_calls(ngc, cache, k_new, v_new, q, scale, hint, out, ws)
    attn_events = []

    def period(rnd, record):
        for t in range(w.delta):
            if record:
                e0, e1 = ev(), ev()
                e0.record()
            step_call()
            if record:
                e1.record()
                attn_events.append((e0, e1, rows_after + (t + 1) * nseg))
        if record:
            e0, e1 = ev(), ev()
            e0.record()
        evict(rnd)
        if record:
            e1.record()
            evict_events.append((e0, e1))

    evict_events = []
    rnd = 1
    for _ in range(args.warmup):
        period(rnd, False)
        rnd += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        period(rnd, True)
        rnd += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    attn_ms = sum(a.elapsed_time(b) for a, b, _ in attn_events)             # per token-step: L launches
    attn_b = sum(attn_bytes(w, rows, nseg) for _, _, rows in attn_events)
    n_attn = len(attn_events)
    steady_evict_ms = [a.elapsed_time(b) for a, b in evict_events]
    n_mid = keep_h + w.delta // 2
    steady_bytes = evict_bytes(w, keep_h + w.delta, keep_h, moved_rows(), w.with_logprob, w.with_logprob)
    steady_us = 1e3 * float(np.mean(steady_evict_ms))

    tokens = w.B * w.delta * args.steps
    value = tokens / elapsed
    attn_gbs = attn_b / (attn_ms * 1e-3) / 1e9
    # what the plainest read kernel reaches when it is launched the same way: one launch of a layer's bytes after
    # the other, every launch over memory no earlier launch has touched
    read_at = probe.read_ceiling_at(int(attn_b / n_attn / w.L), w.L) if ceilings is not None else None
    p1_gbs = p1_bytes / (p1_us * 1e-6) / 1e9

    # ---- secondary: the same decode steps with all layers in ONE launch (what the kernel does when the launch is
    # large; a model cannot issue it), over one period
    batched_events = []
    for t in range(w.delta):
        e0, e1 = ev(), ev()
        e0.record()
        ngc.ngc_decode_step(cache, -1, k_new, v_new, None, q, scale, hint, out, ws)
        e1.record()
        batched_events.append((e0, e1, rows_after + (t + 1) * nseg))
    evict(rnd)
    rnd += 1
    torch.cuda.synchronize()
    bat_ms = sum(a.elapsed_time(b) for a, b, _ in batched_events)
    bat_b = sum(attn_bytes(w, rows, nseg) for _, _, rows in batched_events)
    bat_gbs = bat_b / (bat_ms * 1e-3) / 1e9

    # ---- the per-layer token-step from a HIP graph (L launches captured once at the mid-period length)
    graph_info = None
    if args.per_layer:
        cache.len.copy_(keep + w.delta // 2)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for l in range(w.L):
                ngc.ngc_decode_attn(cache, l, q[l], scale, hint, out[l], ws)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        eager = out.clone()
        gph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gph):
            for l in range(w.L):
                ngc.ngc_decode_attn(cache, l, q[l], scale, hint, out[l], ws)
        out.zero_()
        gph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "graph replay differs from the eager launches"
        reps = 20
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(reps):
            gph.replay()
        e1.record()
        torch.cuda.synchronize()
        gms = e0.elapsed_time(e1) / reps
        mid_bytes = attn_bytes(w, rows_after + (w.delta // 2) * nseg, nseg)
        graph_info = {"what": "L per-layer ngc_decode_attn launches at the mid-period length, captured once and replayed",
                      "ms_per_token_step": gms, "hbm_frac": mid_bytes / (gms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del gph
        cache.len.copy_(keep)

    status = ngc.read_status(ws)
    assert all(x == 0 for x in status), f"device status words not clean: {status[:8]}"
    # sanity: lengths are back at the budget after the last round
    assert torch.equal(cache.len.cpu(), torch.from_numpy(keep_h)), "lengths drifted from the schedule"

    # ---- the same rounds with the unordered (hole filling) arrangement: same sample, fewer rows moved
    def timed_evict(rnd, flags):
        e0, e1 = ev(), ev()
        e0.record()
        evict(rnd, flags)
        e1.record()
        torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1)

    def unordered_moved():
        valid = slot < keep.unsqueeze(-1)
        return float(((kept >= keep.unsqueeze(-1)) & valid).sum().item())

    un_p1, un_steady = [], []
    for rep in range(3):
        cache.len.copy_(len0)
        torch.cuda.synchronize()
        un_p1.append(timed_evict(0, ngc.EVICT_UNORDERED))
    un_p1_moved = unordered_moved()
    for rep in range(3):
        for t in range(w.delta):
            ngc.ngc_cache_append(cache, -1, k_new, v_new, None, ws)
        torch.cuda.synchronize()
        un_steady.append(timed_evict(rnd + rep, ngc.EVICT_UNORDERED))
    un_steady_moved = unordered_moved()
    un_p1_us, un_steady_us = float(np.mean(un_p1[1:])), float(np.mean(un_steady[1:]))
    un_p1_bytes = evict_bytes(w, n_items0, keep_h, un_p1_moved, w.with_logprob, w.with_logprob)
    un_steady_bytes = evict_bytes(w, keep_h + w.delta, keep_h, un_steady_moved, w.with_logprob, w.with_logprob)
    unordered = {
        "what": "same rounds with NGC_EVICT_UNORDERED (kept rows beyond slot K fill the freed slots below K)",
        "eviction_step_us": un_p1_us, "moved_rows": un_p1_moved, "bytes_per_round": un_p1_bytes,
        "hbm_frac": un_p1_bytes / (un_p1_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
        "eviction_step_us_steady": un_steady_us, "moved_rows_steady": un_steady_moved,
        "hbm_frac_steady": un_steady_bytes / (un_steady_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
    }

    # ---- the paper's granularity on the contiguous layout: items are blocks of 32 rows and the KV heads of a
    # (layer, sequence) share one noise draw (Sec. 4.2); whole blocks (8 KB of K, 8 KB of V) move
    BLK = 32
    items_b = (lens + BLK - 1) // BLK
    keep_b_h = np.zeros((w.L, w.B, w.Hkv), np.int32)
    for b in range(w.B):
        keep_b_h[:, b, :] = (int(items_b[b]) * w.keep_num + w.keep_den - 1) // w.keep_den
    keep_b = torch.from_numpy(keep_b_h).to(dev)
    max_keep_b = int(keep_b_h.max())
    kept_b = torch.empty(w.L, w.B, w.Hkv, max_keep_b, dtype=torch.int32, device=dev)
    sigma_b = torch.empty_like(kept_b)
    b32_us = []
    for rep in range(3):
        cache.len.copy_(len0)
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        ngc.ngc_evict(cache, -1, logits, keep_b,
                      ngc.make_params(block=BLK, share_heads=1, noise_scale=1.0, round=0, seed=w.gumbel_seed),
                      max_keep_b, kept_b, sigma_b, logp, ws)
        e1.record()
        torch.cuda.synchronize()
        b32_us.append(1e3 * e0.elapsed_time(e1))
    slot_b = torch.arange(max_keep_b, device=dev, dtype=torch.int32)
    moved_blocks = ((kept_b != slot_b) & (slot_b < keep_b.unsqueeze(-1)))
    # rows of a moved block: BLK, except a segment's short last block
    n0_t = torch.from_numpy(np.broadcast_to(lens[None, :, None], keep_b_h.shape).copy()).to(dev).unsqueeze(-1)
    rows_in = torch.clamp(n0_t - kept_b * BLK, max=BLK)
    moved_b_rows = float((rows_in * moved_blocks).sum().item())
    b32_us_m = float(np.mean(b32_us[1:]))
    b32_bytes = evict_bytes(w, np.broadcast_to(items_b[None, :, None], keep_b_h.shape), keep_b_h, moved_b_rows,
                            True, True)
    block32 = {
        "what": "round 0 with blocks of 32 rows and one noise draw per (layer, sequence): whole blocks move",
        "eviction_step_us": b32_us_m, "moved_rows": moved_b_rows, "bytes_per_round": b32_bytes,
        "hbm_frac": b32_bytes / (b32_us_m * 1e-6) / 1e9 / HBM_PEAK_GBS,
    }
    del kept_b, sigma_b
    # back to the per-row schedule's state: one per-row round from the peak
    cache.len.copy_(len0)
    evict(rnd + 20)
    for t in range(w.delta):
        ngc.ngc_cache_append(cache, -1, k_new, v_new, None, ws)
    evict(rnd + 21)

    # ---- key scoring (the step before the eviction round): w = 5 recent queries, steady-state size.  The w
    # decode steps before the round hand their log-sum-exp (lse_out) and queries to two small rings; scoring then
    # reads K once.  Without the ring it has to find the normalisers itself and reads K twice (reported beside).
    w_recent = 5
    q_recent = torch.empty(w.L, w.B, w_recent, w.Hq, w.D, dtype=torch.bfloat16, device=dev)
    lse_ring = torch.empty(w.L, w.B, w_recent, w.Hq, dtype=torch.float32, device=dev)
    lse_j = torch.empty(w.L, w.B, w.Hq, dtype=torch.float32, device=dev)
    scores = torch.empty(w.L, w.B, w.Hkv, cap, dtype=torch.float32, device=dev)
    cache.len.copy_(keep + (w.delta - w_recent))
    for j in range(w_recent):
        q_j = torch.randn(w.L, w.B, w.Hq, w.D, generator=g, device=dev).to(torch.bfloat16)
        ngc.ngc_decode_step(cache, -1, k_new, v_new, None, q_j, scale, hint, out, ws, lse_out=lse_j)
        q_recent[:, :, j].copy_(q_j)
        lse_ring[:, :, j].copy_(lse_j)
    sc1_ms, sc_ms = [], []
    for rep in range(4):
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        ngc.ngc_score_keys(cache, -1, q_recent, w_recent, scale, 0, 1, scores, ws, lse_recent=lse_ring)
        e1.record()
        torch.cuda.synchronize()
        sc1_ms.append(e0.elapsed_time(e1))
    ring_scores = scores.clone()
    for rep in range(4):
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        ngc.ngc_score_keys(cache, -1, q_recent, w_recent, scale, 0, 1, scores, ws)
        e1.record()
        torch.cuda.synchronize()
        sc_ms.append(e0.elapsed_time(e1))
    # both routes give the same scores (the ring holds what the second route recomputes)
    valid = torch.arange(cap, device=dev) < cache.len.unsqueeze(-1)
    sc_diff = float(((ring_scores - scores).abs() * valid).max().item())
    assert sc_diff <= 1e-5, f"scores from decode's log-sum-exp differ from the two-pass scores by {sc_diff}"
    del ring_scores
    sc1_us, sc_us = 1e3 * float(np.mean(sc1_ms[1:])), 1e3 * float(np.mean(sc_ms[1:]))
    rows_scored = float((keep_h + w.delta).sum())
    sc_bytes = rows_scored * (2 * w.D + 4) + nseg * w_recent * w.G * w.D * 2     # K once, one score per key, queries
    scoring = {
        "what": f"ngc_score_keys, w={w_recent}, every segment at budget + delta rows, all layers in one launch; the "
                "normalisers come from the last w decode steps (lse_out ring): one pass over K",
        "us": sc1_us, "bytes": sc_bytes, "hbm_frac": sc_bytes / (sc1_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
        "two_pass_us": sc_us, "two_pass_hbm_frac": sc_bytes / (sc_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
        "two_pass_note": "without the ring (lse_recent = NULL) the kernel first finds each query's normaliser: K is "
                         "read twice, HBM traffic ~2x these bytes",
        "max_abs_difference_between_routes": sc_diff,
    }
    evict(rnd + 10)      # back to the budget

    # ---- gradient of the log-prob for the round just sampled (what Eq. 4 back-propagates)
    bwd = None
    if w.with_logprob:
        n_items_d = (keep + w.delta).reshape(-1).contiguous()
        grad = torch.empty_like(logits)
        gout = torch.randn(nseg, generator=g, device=dev)
        bw_ms = []
        for rep in range(4):
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            ngc.ngc_subset_logprob_backward(logits, n_items_d, sigma, keep.reshape(-1), nseg, cap, max_keep, max_keep,
                                            gout, grad, ws)
            e1.record()
            torch.cuda.synchronize()
            bw_ms.append(e0.elapsed_time(e1))
        bw_us = 1e3 * float(np.mean(bw_ms[1:]))
        bw_bytes = 8.0 * float((keep_h + w.delta).sum()) + 4.0 * float(keep_h.sum()) + 4.0 * nseg
        bwd = {"what": "ngc_subset_logprob_backward for every segment of the round (n = budget + delta)",
               "us": bw_us, "bytes": bw_bytes, "hbm_frac": bw_bytes / (bw_us * 1e-6) / 1e9 / HBM_PEAK_GBS}
        del grad
        # Eq. 4 itself: loss, advantages and the weights of 8 rounds' log-probabilities (latency bound: tiny)
        R_l, G_l = 8, min(16, w.B)
        lp_all = -1000.0 * torch.rand(R_l, w.L, w.B, w.Hkv, generator=g, device=dev)
        rounds_l = torch.randint(1, R_l + 1, (w.B,), generator=g, device=dev, dtype=torch.int32)
        reward_l = torch.randint(0, 2, (w.B,), generator=g, device=dev).to(torch.float32)
        loss_layer = torch.empty(w.L, dtype=torch.float32, device=dev)
        loss_l = torch.empty(1, dtype=torch.float32, device=dev)
        gout_l = torch.empty_like(lp_all)
        lm_ms = []
        for rep in range(4):
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            ngc.ngc_lmem(lp_all, rounds_l, reward_l, R_l, w.L, w.B, w.Hkv, G_l, None, loss_layer, loss_l, gout_l)
            e1.record()
            torch.cuda.synchronize()
            lm_ms.append(e0.elapsed_time(e1))
        bwd["lmem_us"] = 1e3 * float(np.mean(lm_ms[1:]))
        bwd["lmem_what"] = f"ngc_lmem: Eq. 4 over {R_l} rounds x {w.L} layers x {w.B} rollouts x {w.Hkv} heads, groups of {G_l}"

    # ---- config 4, other reading: one budget per sequence pooled over its KV heads
    pooled = None
    if w.per_head_budget and w.Hkv * cap <= 65536:
        ws_p = torch.zeros(ngc.ngc_workspace_bytes(cache, cap) + 16 * nseg * cap, dtype=torch.uint8, device=dev)
        kept_p = torch.empty(w.L, w.B, w.Hkv, cap, dtype=torch.int32, device=dev)   # a head may keep more than its even share
        sigma_p = torch.empty_like(kept_p)
        pl_ms = []
        for rep in range(3):
            cache.len.copy_(len0)
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            ngc.ngc_evict(cache, -1, logits, keep,
                          ngc.make_params(noise_scale=1.0, round=0, seed=w.gumbel_seed, flags=ngc.EVICT_POOL_HEADS),
                          cap, kept_p, sigma_p, logp, ws_p)
            e1.record()
            torch.cuda.synchronize()
            pl_ms.append(e0.elapsed_time(e1))
        lens_p = cache.len.cpu().numpy()
        slot_p = torch.arange(cap, device=dev, dtype=torch.int32)
        moved_p = float(((kept_p != slot_p) & (slot_p < cache.len.unsqueeze(-1))).sum().item())
        pl_us = 1e3 * float(np.mean(pl_ms[1:]))
        pl_bytes = evict_bytes(w, n_items0, lens_p, moved_p, True, True)
        pooled = {"what": "round 0 with NGC_EVICT_POOL_HEADS: one top-K per (layer, sequence) over all heads' rows",
                  "eviction_step_us": pl_us, "bytes_per_round": pl_bytes,
                  "hbm_frac": pl_bytes / (pl_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                  "rows_kept_per_head_min_max": [int(lens_p.min()), int(lens_p.max())]}
        assert all(x == 0 for x in ngc.read_status(ws_p)), "pooled run: status words not clean"
        del ws_p, kept_p, sigma_p
        cache.len.copy_(keep)       # back to the schedule's state

    replay = {"what": "ngc_replay_attn, one layer, rounds every delta tokens, random survivors; ms = mean of 20 back-to-back calls "
                      "after 10 untimed ones (list kernel included); bound: bf16 MFMA 2.5 PFLOP/s",
              "per_token_eviction": replay_case(ngc, w, g, dev, 1), "block32_eviction": replay_case(ngc, w, g, dev, 32)}

    # ---- the same cycle over the paged layout (pages of 32 rows = the paper's blocks): eviction edits page
    # tables, nothing moves; decode attention and append go through the table.  Runs last: the contiguous
    # cache is released first.
    paged = None
    if not args.no_paged:
        del cache, logits, kept, sigma, scores
        torch.cuda.empty_cache()
        P = 32
        max_pages = (cap + P - 1) // P + 1
        pages_b = (lens + P - 1) // P                                        # [B] pages per segment at the peak
        n_pg = np.broadcast_to(pages_b[None, :, None], (w.L, w.B, w.Hkv)).reshape(-1).astype(np.int64)
        keep_pg = np.array([(int(n) * w.keep_num + w.keep_den - 1) // w.keep_den for n in n_pg], np.int32)
        grow_pg = (w.delta + P - 1) // P + 1
        num_pages = int(n_pg.sum() + nseg * grow_pg)
        pc = ngc.PagedCache.allocate(w.L, w.B, w.Hkv, w.Hq, w.D, P, max_pages, num_pages, device=dev)
        synth.fill_normal_bf16_(pc.k_pool, w.data_seed * 2 + 10)
        synth.fill_normal_bf16_(pc.v_pool, w.data_seed * 2 + 11)
        first = np.concatenate([[0], np.cumsum(n_pg)[:-1]])
        table_h = np.full((nseg, max_pages), -1, np.int32)
        for sg in range(nseg):
            table_h[sg, :n_pg[sg]] = np.arange(first[sg], first[sg] + n_pg[sg])
        table0 = torch.from_numpy(table_h.reshape(w.L, w.B, w.Hkv, max_pages)).to(dev)
        stack0 = torch.from_numpy(np.arange(num_pages - 1, int(n_pg.sum()) - 1, -1, dtype=np.int32)).to(dev)
        n_free0 = int(stack0.numel())
        keep_p = torch.from_numpy(keep_pg.reshape(w.L, w.B, w.Hkv)).to(dev)
        max_keep_p = int(keep_pg.max())
        plog = torch.randn(w.L, w.B, w.Hkv, max_pages, generator=g, device=dev)
        kept_p = torch.empty(w.L, w.B, w.Hkv, max_keep_p, dtype=torch.int32, device=dev)
        sigma_p = torch.empty_like(kept_p)
        ws_p = ngc.allocate_paged_workspace(pc)

        def reset_paged():
            pc.table.copy_(table0)
            pc.len.copy_(len0)
            pc.free_stack[:n_free0].copy_(stack0)
            pc.free_count.fill_(n_free0)

        def paged_evict(r):
            ngc.ngc_paged_evict(pc, -1, plog, max_pages, keep_p,
                                ngc.make_params(block=P, noise_scale=1.0, round=r, seed=w.gumbel_seed),
                                max_keep_p, kept_p, sigma_p if w.with_logprob else None,
                                logp if w.with_logprob else None, ws_p)

        pg_p1 = []
        for rep in range(4):
            reset_paged()
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            paged_evict(0)
            e1.record()
            torch.cuda.synchronize()
            pg_p1.append(1e3 * e0.elapsed_time(e1))
        rows_after_p = float(pc.len.sum().item())
        hint_p = int(pc.len.max().item()) + w.delta
        pg_events, pg_evict_us = [], []
        periods = 1 + min(args.steps, 3)
        t_start = None
        for per in range(periods):
            if per == 1:
                torch.cuda.synchronize()
                t_start = time.perf_counter()
            for t in range(w.delta):
                ngc.ngc_paged_append(pc, -1, k_new, v_new, None, ws_p)
                e0, e1 = ev(), ev()
                e0.record()
                ngc.ngc_paged_decode_attn(pc, -1, q, scale, hint_p, out, ws_p)
                e1.record()
                if per > 0:
                    pg_events.append((e0, e1, rows_after_p + (t + 1) * nseg))
            e0, e1 = ev(), ev()
            e0.record()
            paged_evict(per + 1)
            e1.record()
            if per > 0:
                pg_evict_us.append((e0, e1))
            rows_after_p = float(pc.len.sum().item())     # (synchronises once per period)
        torch.cuda.synchronize()
        pg_elapsed = time.perf_counter() - t_start
        pg_attn_ms = sum(a.elapsed_time(b) for a, b, _ in pg_events)
        pg_attn_b = sum(attn_bytes(w, rows, nseg) for _, _, rows in pg_events)
        assert all(x == 0 for x in ngc.read_status(ws_p)), "paged run: status words not clean"
        used = int(((pc.len + (P - 1)) // P).sum().item())
        assert used + int(pc.free_count.item()) == num_pages, "paged run: pages lost"
        paged = {
            "what": f"same cycle over the paged layout, pages of {P} rows, keep {w.keep_num}/{w.keep_den} of the pages "
                    "per round; eviction = sampling + log-prob + page-table edit + ordered release, no K/V bytes moved",
            "pool_pages": num_pages, "pool_GB": 2.0 * num_pages * P * w.D * 2 / 1e9,
            "eviction_step_us": float(np.mean(pg_p1[1:])),
            "eviction_step_us_steady": 1e3 * float(np.mean([a.elapsed_time(b) for a, b in pg_evict_us])),
            "tokens_per_s": w.B * w.delta * (periods - 1) / pg_elapsed,
            "decode_attn_ms_per_token_step": pg_attn_ms / len(pg_events),
            "decode_attn_hbm_frac": pg_attn_b / (pg_attn_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "rows_per_segment_after_round": rows_after_p / nseg,
        }

    # ---- the other two configurations the target is quoted on: round-0 / steady-state eviction and a sampled
    # period of per-layer and all-layer decode steps (the big buffers of the main workload are released first)
    other = None
    if not args.no_other_configs:
        # (a `del` of a name the paged section already deleted raises; every name gets its own try)
        try: del cache
        except NameError: pass
        try: del logits
        except NameError: pass
        try: del kept, sigma
        except NameError: pass
        try: del scores
        except NameError: pass
        try: del ws, step_call
        except NameError: pass
        try: del pc, plog, kept_p, sigma_p, ws_p, table0, stack0
        except NameError: pass
        try: del eager
        except NameError: pass
        torch.cuda.empty_cache()
        other = {}
        for idx in (2, 3, 4):
            if idx == w.index:
                continue
            other[str(idx)] = quick_config(ngc, synth, synth.workload(idx), dev, with_ceiling=ceilings is not None)
            torch.cuda.empty_cache()

    line = {
        "metric": METRIC,
        "value": value,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{'configs[%d]' % w.index if w.index < 5 else 'extra (paper-shaped, not a BASELINE config)'} {w.name}: L={w.L} B={w.B} Hq/Hkv={w.Hq}/{w.Hkv} D={w.D} "
                        f"peak cache {w.n_lo}..{w.n_hi} rows, keep {w.keep_num}/{w.keep_den} (budget rule), "
                        f"delta={w.delta}, logits {w.logits_kind}, log-prob {'on' if w.with_logprob else 'off'}",
            "step": f"{w.delta} token-steps x {w.L} launches of ngc_decode_step (one per layer: append + decode "
                    "attention) + 1 eviction round (all layers in one launch); all layers per decode launch is "
                    "timed separately: roofline_decode_all_layers_per_launch",
            "tokens_per_step": w.B * w.delta,
        },
        "decode_attn_tokens_per_s": w.B * n_attn / (attn_ms * 1e-3),
        "decode_attn_ms_per_token_step": attn_ms / n_attn,
        "eviction_step_us": p1_us,
        "eviction_step_us_steady": steady_us,
        "eviction_steady_hbm_frac": steady_bytes / (steady_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
        "roofline": {
            "kernel": "decode_kernel<%d, false, true>, one launch per layer (append fused)" % w.D,
            "bound": "hbm", "achieved": attn_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": attn_gbs / HBM_PEAK_GBS,
            "traffic": profile_traffic((w.index, w.L, w.B), "decode")[0],
            "traffic_source": profile_traffic((w.index, w.L, w.B), "decode")[1],
            "bytes_per_launch": attn_b / n_attn / w.L, "launch_ms": attn_ms / n_attn / w.L, "launches": n_attn * w.L,
            "launch_ms_note": "HIP events around every token-step of the timed region (L back-to-back launches on the "
                              "stream) divided by L: includes the gaps between launches",
            "frac_of_measured_read_ceiling": (attn_gbs / max(ceilings["read_GBs"], ceilings["read_nontemporal_GBs"])
                                              if ceilings else None),
            "frac_of_read_probe_at_launch_size": (attn_gbs / read_at["GBs"]) if read_at else None,
            "read_probe_at_launch_size": read_at,
        },
        "roofline_decode_all_layers_per_launch": {
            "what": "the same decode steps with all layers in one launch (a model cannot issue this; it shows the kernel "
                    "when a launch is large), one period",
            "kernel": "decode_kernel<%d, false, true>" % w.D,
            "bound": "hbm", "achieved": bat_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bat_gbs / HBM_PEAK_GBS,
            "traffic": profile_traffic((w.index, w.L, w.B), "decode_batched")[0],
            "traffic_source": profile_traffic((w.index, w.L, w.B), "decode_batched")[1],
            "bytes_per_launch": bat_b / len(batched_events), "launch_ms": bat_ms / len(batched_events),
            "tokens_per_s": w.B * len(batched_events) / (bat_ms * 1e-3),
        },
        "decode_attn_per_layer_hip_graph": graph_info,
        "roofline_evict": {
            "kernels": "evict_kernel (selection + log-prob + in-place compaction fused; round 0 at peak cache)",
            "bound": "hbm", "achieved": p1_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": p1_gbs / HBM_PEAK_GBS,
            "traffic": profile_traffic((w.index, w.L, w.B), "evict")[0],
            "traffic_source": profile_traffic((w.index, w.L, w.B), "evict")[1],
            "bytes_per_round": p1_bytes, "round_ms": p1_us / 1e3, "moved_rows": moved0,
            "frac_of_measured_copy_ceiling": (p1_gbs / max(ceilings["copy_GBs"], ceilings["copy_nontemporal_GBs"],
                                                           ceilings["copy_best_shape_GBs"]) if ceilings else None),
        },
        "other_configs": other,
        "eviction_unordered": unordered,
        "eviction_block32_shared_heads": block32,
        "scoring": scoring,
        "logprob_backward": bwd,
        "eviction_pooled_heads": pooled,
        "replay_attn": replay,
        "paged_layout": paged,
        "cache_schedule": {
            "what": "rows cached per (layer, head), mean over sequences, after the workload's decode_steps tokens: "
                    "without eviction, and the peak with it (budget rule); the paper's peak-KV-reduction figure "
                    "(Sec. 5.1) for this synthetic schedule, context only",
            "rows_without_eviction": float(np.mean(lens + w.decode_steps)),
            "peak_rows_with_eviction": float(np.mean(np.maximum(lens, keep_h.mean(axis=(0, 2)) + w.delta))),
            "peak_reduction": float(np.mean((lens + w.decode_steps) /
                                            np.maximum(lens, keep_h.mean(axis=(0, 2)) + w.delta))),
        },
        "measured_ceilings": ceilings,
        "paper_context": {
            "what": "figures the paper reports, context only (no throughput, latency or bandwidth is published for "
                    "this path; the paper names neither its hardware nor its precision)",
            "peak_kv_cache_reduction": {"countdown_50pct_eviction_per_round": 2.4, "aime2025_50pct_eviction_per_round": 4.6,
                                        "math_benchmarks_range": [3, 5]},
            "countdown_accuracy_pct": {"ngc": 49.6, "best_heuristic_eviction_baseline": 21.2},
            "method_constants": {"block": 32, "recent_queries_w": 5, "cadence_delta": [256, 350]},
            "hardware": "not stated",
        },
        "setup_s": t_setup,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, lens, keep_h, n_mid)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
