"""GPU parity of the eviction step against the CPU oracle, through the C ABI.

Indices, lengths and compacted bytes must be bit-exact; log-probabilities
within 1e-4 relative (fp32 kernel vs fp64 oracle: K terms of magnitude ~log n,
each carrying ~1e-7 relative error, summed pairwise)."""
import numpy as np
import pytest

import oracle as orc
from paper_2604_18002_amd import synth

from _harness import (from_bf16_tensor, host_case, oracle_evict_segment, oracle_logprob, to_bf16_tensor, upload)

pytestmark = pytest.mark.gpu

LOGP_RTOL = 1e-4


def _ngc():
    from paper_2604_18002_amd import binding
    binding.load_library()
    return binding


def _run_evict(case, tau=1.0, rnd=0, block=1, share_heads=0, with_pos=True, layer=-1, select_only=False,
               want_sigma=True, want_logp=True):
    import torch
    ngc = _ngc()
    w = case.w
    cache, logits, keep = upload(case, with_pos=with_pos)
    max_keep = int(case.keep.max()) if case.keep.size else 1
    max_keep = max(max_keep, 1)
    ws = ngc.allocate_workspace(cache, max_keep)
    kept = torch.full((w.L, w.B, w.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1) if want_sigma else None
    logp = torch.full((w.L, w.B, w.Hkv), float("nan"), dtype=torch.float32, device="cuda") if want_logp else None
    p = ngc.make_params(block=block, share_heads=share_heads, noise_scale=tau, round=rnd, seed=w.gumbel_seed,
                        flags=ngc.EVICT_SELECT_ONLY if select_only else 0)
    print(f"[evict] workload={w.name} L={w.L} B={w.B} Hkv={w.Hkv} cap={w.cap} tau={tau} block={block} "
          f"layer={layer} max_keep={max_keep}", flush=True)
    ngc.ngc_evict(cache, layer, logits, keep, p, max_keep, kept, sigma, logp, ws)
    torch.cuda.synchronize()
    return cache, kept, sigma, logp, ws


def _check_against_oracle(case, cache, kept, sigma, logp, tau, rnd, block=1, share_heads=False, segs=None,
                          moved=True):
    w = case.w
    hk, hv = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v)
    hlen = cache.len.cpu().numpy()
    hkept = kept.cpu().numpy()
    hsig = sigma.cpu().numpy() if sigma is not None else None
    hlp = logp.cpu().numpy() if logp is not None else None
    hpos = cache.pos.cpu().numpy() if cache.pos is not None else None
    for seg in (segs or case.segs):
        l, b, h = seg
        okept, osig, olp, ok, ov = oracle_evict_segment(case, seg, tau, w.gumbel_seed, rnd, block, share_heads)
        K = okept.size
        assert hkept[l, b, h, :K].tolist() == okept.tolist(), f"kept differs at segment {seg}"
        if hsig is not None:
            assert hsig[l, b, h, :K].tolist() == osig.tolist(), f"sigma differs at segment {seg}"
        if hlp is not None:
            assert hlp[l, b, h] == pytest.approx(olp, rel=LOGP_RTOL, abs=1e-5), f"logp differs at segment {seg}"
        if moved:
            n_new = ok.shape[0]
            assert hlen[l, b, h] == n_new, f"len differs at segment {seg}"
            assert hk[l, b, h, :n_new].tobytes() == ok.tobytes(), f"K bytes differ at segment {seg}"
            assert hv[l, b, h, :n_new].tobytes() == ov.tobytes(), f"V bytes differ at segment {seg}"
            if hpos is not None:
                n_old = case.k[seg].shape[0]
                want = orc.compact_i32(np.arange(n_old, dtype=np.int32), okept, block)
                assert hpos[l, b, h, :n_new].tolist() == want.tolist(), f"pos differs at segment {seg}"


# ---------------------------------------------------------------- keys -----

@pytest.mark.parametrize("tau", [1.0, 0.37])
def test_perturbed_keys_bit_exact(tau):
    import torch
    ngc = _ngc()
    w = synth.workload(1, L=3, B=5, Hkv=2, Hq=12, n_lo=900, n_hi=4099)
    case = host_case(w)
    cache, logits, _ = upload(case)
    ws = ngc.allocate_workspace(cache, 1)
    keys = torch.zeros_like(logits)
    for share in (0, 1):
        p = ngc.make_params(noise_scale=tau, round=5, seed=0xDEADBEEF12345678, share_heads=share)
        print(f"[keys] tau={tau} share_heads={share}", flush=True)
        ngc.ngc_perturbed_keys(cache, -1, logits, p, keys, ws)
        torch.cuda.synchronize()
        hkeys = keys.cpu().numpy()
        for (l, b, h) in case.segs:
            s = case.logits[(l, b, h)]
            want = orc.perturbed_keys(s, tau, 0xDEADBEEF12345678, 5, l, b, 0xFFFF if share else h)
            got = hkeys[l, b, h, :s.size]
            assert got.tobytes() == want.tobytes(), f"keys differ at {(l, b, h)} share={share}"


def test_perturbed_keys_many_counters():
    # 2^20 items in one go: the random words and the defined logarithm agree bit for bit
    import torch
    ngc = _ngc()
    w = synth.workload(2, L=2, B=16, Hkv=2, Hq=12, n_lo=16384, n_hi=16384)
    lens = synth.lengths(w)
    cache = ngc.Cache.allocate(w.L, w.B, w.Hkv, w.Hq, 64, w.cap)
    cache.len.fill_(w.cap)
    logits = torch.zeros(w.L, w.B, w.Hkv, w.cap, dtype=torch.float32, device="cuda")
    keys = torch.zeros_like(logits)
    ws = ngc.allocate_workspace(cache, 1)
    p = ngc.make_params(noise_scale=1.0, round=77, seed=2 ** 63 + 12345)
    print("[keys] 2^20 counters", flush=True)
    ngc.ngc_perturbed_keys(cache, -1, logits, p, keys, ws)
    torch.cuda.synchronize()
    hkeys = keys.cpu().numpy()
    zeros = np.zeros(w.cap, np.float32)
    for l in range(w.L):
        for b in range(w.B):
            for h in range(w.Hkv):
                want = orc.perturbed_keys(zeros, 1.0, 2 ** 63 + 12345, 77, l, b, h)
                assert hkeys[l, b, h].tobytes() == want.tobytes(), (l, b, h)


# --------------------------------------------------------------- evict -----

def test_config0_tiny():
    case = host_case(synth.workload(0))
    cache, kept, sigma, logp, ws = _run_evict(case)
    _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 0)
    assert all(x == 0 for x in _ngc().read_status(ws))


def test_config1_small_rollout_batch():
    case = host_case(synth.workload(1))
    cache, kept, sigma, logp, ws = _run_evict(case)
    _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 0)
    assert all(x == 0 for x in _ngc().read_status(ws))


def test_greedy_eval_mode_with_ties():
    # tau = 0 on logits with many exact ties: index order must decide
    w = synth.workload(1, B=4, n_lo=1500, n_hi=2048)
    case = host_case(w)
    for seg in case.segs:
        case.logits[seg] = np.round(case.logits[seg] * 4).astype(np.float32) / 4   # ~25 distinct values
    cache, kept, sigma, logp, ws = _run_evict(case, tau=0.0)
    _check_against_oracle(case, cache, kept, sigma, logp, 0.0, 0)


def test_drift_and_heavy_tail_logits():
    for idx, n in ((2, 4096), (4, 16384)):
        w = synth.workload(idx, L=2, B=2, n_lo=n, n_hi=n)
        case = host_case(w)
        cache, kept, sigma, logp, ws = _run_evict(case, with_pos=False)
        _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 0)


def test_ragged_7b_shape_reduced():
    w = synth.workload(3, L=2, B=6)
    case = host_case(w)
    cache, kept, sigma, logp, ws = _run_evict(case, rnd=3, with_pos=False)
    _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 3)


def test_block_items_and_shared_heads():
    # the paper's granularity: blocks of 32 rows, one noise draw per (layer, sequence)
    w = synth.workload(1, L=2, B=3, n_lo=1000, n_hi=2048)
    case = host_case(w, block=32)
    cache, kept, sigma, logp, ws = _run_evict(case, block=32, share_heads=1)
    _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 0, block=32, share_heads=True)


def test_single_layer_call_leaves_other_layers_alone():
    import torch
    w = synth.workload(1, L=3, B=2, n_lo=1200, n_hi=1800)
    case = host_case(w)
    cache0, _, _ = upload(case)
    before_k = from_bf16_tensor(cache0.k)
    cache, kept, sigma, logp, ws = _run_evict(case, layer=1)
    segs = [s for s in case.segs if s[0] == 1]
    _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 0, segs=segs)
    after_k = from_bf16_tensor(cache.k)
    hlen = cache.len.cpu().numpy()
    for l in (0, 2):
        assert after_k[l].tobytes() == before_k[l].tobytes()
        assert (hlen[l] == case.lens[:, None]).all()


def test_select_only_moves_nothing():
    w = synth.workload(1, B=2)
    case = host_case(w)
    cache0, _, _ = upload(case)
    cache, kept, sigma, logp, ws = _run_evict(case, select_only=True)
    _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 0, moved=False)
    assert from_bf16_tensor(cache.k).tobytes() == from_bf16_tensor(cache0.k).tobytes()
    assert (cache.len.cpu().numpy() == case.lens[None, :, None]).all()


def test_more_large_segments_than_resident_workgroups():
    # Segments of more than 4096 items go to workgroups that fill a compute unit and fetch one segment after
    # another from a counter in the workspace: 640 segments on 256 compute units, so most workgroups take
    # several.  Two calls on the same workspace (the counters must be back at zero in between): selection
    # only, then the full round; the same noise, so both must give the oracle's lists.
    import torch
    ngc = _ngc()
    w = synth.workload(1, L=2, B=160, Hkv=2, Hq=4, D=64, n_lo=4097, n_hi=4400)
    segs = sorted({(0, 0, 0), (w.L - 1, w.B - 1, w.Hkv - 1), (0, 128, 0), (1, 0, 1), (1, 77, 0), (0, 159, 1),
                   (1, 130, 1), (0, 64, 1)})
    case = host_case(w, segs)
    max_keep = int(case.keep.max())
    cache = ngc.Cache.allocate(w.L, w.B, w.Hkv, w.Hq, w.D, w.cap, with_pos=True)
    synth.fill_normal_bf16_(cache.k, 11)
    synth.fill_normal_bf16_(cache.v, 12)
    cache.pos.copy_(torch.arange(w.cap, dtype=torch.int32).expand(w.L, w.B, w.Hkv, w.cap))
    logits = torch.empty(w.L, w.B, w.Hkv, w.cap, dtype=torch.float32, device="cuda")
    synth.fill_logits_(logits, w, 13)
    cache.len.copy_(torch.from_numpy(np.broadcast_to(case.lens[None, :, None], (w.L, w.B, w.Hkv)).copy()))
    for seg in segs:
        l, b, h = seg
        n = case.k[seg].shape[0]
        cache.k[l, b, h, :n] = to_bf16_tensor(case.k[seg], "cuda")
        cache.v[l, b, h, :n] = to_bf16_tensor(case.v[seg], "cuda")
        logits[l, b, h, :n] = torch.from_numpy(case.logits[seg]).cuda()
    keep = torch.from_numpy(case.keep).cuda()
    ws = ngc.allocate_workspace(cache, max_keep)
    for select_only in (True, False):
        kept = torch.full((w.L, w.B, w.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
        sigma = torch.full_like(kept, -1)
        logp = torch.full((w.L, w.B, w.Hkv), float("nan"), dtype=torch.float32, device="cuda")
        p = ngc.make_params(noise_scale=1.0, round=2, seed=w.gumbel_seed,
                            flags=ngc.EVICT_SELECT_ONLY if select_only else 0)
        print(f"[evict] {w.L * w.B * w.Hkv} segments of up to {w.cap} rows, select_only={select_only}", flush=True)
        ngc.ngc_evict(cache, -1, logits, keep, p, max_keep, kept, sigma, logp, ws)
        torch.cuda.synchronize()
        assert all(x == 0 for x in ngc.read_status(ws))   # includes the two queue words
        _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 2, segs=segs, moved=not select_only)
        # every segment was served exactly once: all lists filled, all log-probabilities written
        valid = torch.arange(max_keep, device="cuda") < keep.unsqueeze(-1)
        assert bool(((kept >= 0) | ~valid).all()) and bool(torch.isfinite(logp).all())
    assert torch.equal(cache.len.cpu(), torch.from_numpy(case.keep))


def test_no_sigma_no_logp_fast_path():
    w = synth.workload(1, B=3)
    case = host_case(w)
    cache, kept, sigma, logp, ws = _run_evict(case, want_sigma=False, want_logp=False)
    _check_against_oracle(case, cache, kept, None, None, 1.0, 0)


def test_determinism_and_round_dependence():
    w = synth.workload(1, B=2)
    case = host_case(w)
    a = _run_evict(case, rnd=4)
    b = _run_evict(case, rnd=4)
    c = _run_evict(case, rnd=5)
    assert a[1].cpu().numpy().tobytes() == b[1].cpu().numpy().tobytes()
    assert a[2].cpu().numpy().tobytes() == b[2].cpu().numpy().tobytes()
    assert from_bf16_tensor(a[0].k).tobytes() == from_bf16_tensor(b[0].k).tobytes()
    assert a[2].cpu().numpy().tobytes() != c[2].cpu().numpy().tobytes()


def test_edge_keep_counts():
    # K = 0, K = 1, K = n (no-op round), K > n (clamped and counted), empty segment
    import torch
    ngc = _ngc()
    w = synth.workload(0, B=6, n_lo=300, n_hi=300, fixed_keep=None)
    case = host_case(w)
    case.keep[0, 0, :] = 0
    case.keep[0, 1, :] = 1
    case.keep[0, 2, :] = 300
    case.keep[0, 3, :] = 299
    case.keep[0, 4, :] = 150
    case.keep[0, 5, :] = 150
    cache, kept, sigma, logp, ws = _run_evict(case)
    _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 0)
    assert all(x == 0 for x in ngc.read_status(ws))
    # clamped keep: 400 > 300 behaves as 300 and is counted once per segment
    case2 = host_case(w)
    case2.keep[:] = 150
    cache2, logits2, keep2 = upload(case2)
    keep2[0, 2, :] = 400
    cache2.len[0, 5, :] = 0          # empty segments
    ws2 = ngc.allocate_workspace(cache2, 400)
    kept2 = torch.full((1, 6, 2, 400), -1, dtype=torch.int32, device="cuda")
    sig2 = torch.full_like(kept2, -1)
    lp2 = torch.zeros(1, 6, 2, dtype=torch.float32, device="cuda")
    print("[evict] clamped keep + empty segments", flush=True)
    ngc.ngc_evict(cache2, -1, logits2, keep2, ngc.make_params(seed=w.gumbel_seed), 400, kept2, sig2, lp2, ws2)
    torch.cuda.synchronize()
    st = ngc.read_status(ws2)
    assert st[ngc.STATUS_KEEP_CLAMPED] == 2 + 2      # two heads asked for 400 of 300, two for 150 of 0
    assert kept2[0, 2, 0, :300].cpu().tolist() == list(range(300))
    assert cache2.len[0, 2].cpu().tolist() == [300, 300]
    assert cache2.len[0, 5].cpu().tolist() == [0, 0]
    assert lp2[0, 5].cpu().tolist() == [0.0, 0.0]


def test_argument_errors_are_reported_not_launched():
    import torch
    ngc = _ngc()
    w = synth.workload(0)
    case = host_case(w)
    cache, logits, keep = upload(case)
    ws = ngc.allocate_workspace(cache, 256)
    kept = torch.zeros(1, 1, 2, 256, dtype=torch.int32, device="cuda")
    p = ngc.make_params(seed=1)
    with pytest.raises(ngc.NgcError) as e:
        ngc.ngc_evict(cache, 5, logits, keep, p, 256, kept, None, None, ws)       # layer out of range
    assert e.value.code == ngc.NGC_EINVAL
    with pytest.raises(ngc.NgcError) as e:
        ngc.ngc_evict(cache, -1, logits, keep, p, 256, kept, None, None, ws[:64])  # workspace too small
    assert e.value.code == ngc.NGC_ENOSPC
    with pytest.raises(ngc.NgcError) as e:
        ngc.ngc_evict(cache, -1, None, keep, p, 256, kept, None, None, ws)         # null logits
    assert e.value.code == ngc.NGC_EINVAL
    bad = ngc.make_params(seed=1, block=0)
    with pytest.raises(ngc.NgcError) as e:
        ngc.ngc_evict(cache, -1, logits, keep, bad, 256, kept, None, None, ws)
    assert e.value.code == ngc.NGC_EINVAL
    torch.cuda.synchronize()


# ------------------------------------------------ log-prob of given sigma --

def test_subset_logprob_given_actions():
    import torch
    ngc = _ngc()
    rng = np.random.default_rng(5)
    nseg, stride = 9, 20000
    n_items = np.array([1, 2, 7, 64, 65, 1000, 4097, 16384, 20000], np.int32)
    keep = np.array([1, 2, 3, 64, 1, 333, 2000, 5462, 6000], np.int32)
    logits = np.zeros((nseg, stride), np.float32)
    sigma = np.zeros((nseg, 6000), np.int32)
    for s in range(nseg):
        x = rng.standard_normal(n_items[s]).astype(np.float32)
        if s >= 6:
            out = rng.random(n_items[s]) < 0.05
            x = np.where(out, rng.laplace(0, 4, n_items[s]), x).astype(np.float32)
        logits[s, :n_items[s]] = x
        # a sampled order for half the segments, an arbitrary order for the rest
        if s % 2 == 0:
            _, sg = orc.evict_select(x, int(keep[s]), 1.0, 11, s, 0, 0, 0)
        else:
            sg = rng.permutation(n_items[s])[:keep[s]].astype(np.int32)
        sigma[s, :keep[s]] = sg
    d = lambda a: torch.from_numpy(a).cuda()
    out = torch.zeros(nseg, dtype=torch.float32, device="cuda")
    ws = torch.zeros(ngc.STATUS_WORDS * 4, dtype=torch.uint8, device="cuda")
    print("[logprob] given actions", flush=True)
    ngc.ngc_subset_logprob(d(logits), d(n_items), d(sigma), d(keep), nseg, stride, 6000, out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for s in range(nseg):
        want = oracle_logprob(logits[s, :n_items[s]], sigma[s, :keep[s]])
        assert got[s] == pytest.approx(want, rel=LOGP_RTOL, abs=1e-5), s
    assert all(x == 0 for x in ngc.read_status(ws))
    # a repeated index is counted, not trapped
    sigma[3, 1] = sigma[3, 0]
    ngc.ngc_subset_logprob(d(logits), d(n_items), d(sigma), d(keep), nseg, stride, 6000, out, ws)
    torch.cuda.synchronize()
    assert ngc.read_status(ws)[ngc.STATUS_BAD_SIGMA] >= 1


# --------------------------------------------------------------- append ----

def test_append_rows():
    import torch
    ngc = _ngc()
    w = synth.workload(1, L=2, B=3, n_lo=10, n_hi=40)
    case = host_case(w)
    cache, _, _ = upload(case, with_pos=True, cap=43)
    ws = ngc.allocate_workspace(cache, 1)
    hk0, hv0 = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v)
    new_k = np.stack([synth.new_token_kv(w, l, 0)[0] for l in range(w.L)])
    new_v = np.stack([synth.new_token_kv(w, l, 0)[1] for l in range(w.L)])
    new_pos = torch.tensor([100, 200, 300], dtype=torch.int32, device="cuda")
    print("[append] all layers, then layer 1 only", flush=True)
    ngc.ngc_cache_append(cache, -1, to_bf16_tensor(new_k, "cuda"), to_bf16_tensor(new_v, "cuda"), new_pos, ws)
    ngc.ngc_cache_append(cache, 1, to_bf16_tensor(new_k[1], "cuda"), to_bf16_tensor(new_v[1], "cuda"), new_pos, ws)
    torch.cuda.synchronize()
    hk, hv = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v)
    hlen, hpos = cache.len.cpu().numpy(), cache.pos.cpu().numpy()
    for (l, b, h) in case.segs:
        n = int(case.lens[b])
        assert hlen[l, b, h] == n + (2 if l == 1 else 1)
        assert hk[l, b, h, :n].tobytes() == hk0[l, b, h, :n].tobytes()
        assert hk[l, b, h, n].tobytes() == new_k[l, b, h].tobytes()
        assert hv[l, b, h, n].tobytes() == new_v[l, b, h].tobytes()
        assert hpos[l, b, h, n] == [100, 200, 300][b]
        if l == 1:
            assert hk[l, b, h, n + 1].tobytes() == new_k[l, b, h].tobytes()
    # a full segment is skipped and counted
    cache.len.fill_(43)
    ngc.ngc_cache_append(cache, 0, to_bf16_tensor(new_k[0], "cuda"), to_bf16_tensor(new_v[0], "cuda"), None, ws)
    torch.cuda.synchronize()
    assert ngc.read_status(ws)[ngc.STATUS_APPEND_FULL] == w.B * w.Hkv
    assert (cache.len.cpu().numpy() == 43).all()


# ------------------------------------------------ unordered (hole filling) --

def _run_unordered(case, rnd=0, tau=1.0):
    import torch
    ngc = _ngc()
    w = case.w
    cache, logits, keep = upload(case, with_pos=True)
    max_keep = max(int(case.keep.max()), 1)
    ws = ngc.allocate_workspace(cache, max_keep)
    kept = torch.full((w.L, w.B, w.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1)
    logp = torch.zeros(w.L, w.B, w.Hkv, dtype=torch.float32, device="cuda")
    p = ngc.make_params(noise_scale=tau, round=rnd, seed=w.gumbel_seed, flags=ngc.EVICT_UNORDERED)
    print(f"[evict-unordered] workload={w.name} L={w.L} B={w.B} cap={w.cap} max_keep={max_keep}", flush=True)
    ngc.ngc_evict(cache, -1, logits, keep, p, max_keep, kept, sigma, logp, ws)
    torch.cuda.synchronize()
    return cache, kept, sigma, logp, ws


@pytest.mark.parametrize("idx,over", [(0, {}), (1, {}), (3, dict(L=2, B=4)), (4, dict(L=1, B=2))])
def test_unordered_compaction_parity(idx, over):
    case = host_case(synth.workload(idx, **over))
    w = case.w
    cache, kept, sigma, logp, ws = _run_unordered(case)
    hk, hv = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v)
    hlen, hpos = cache.len.cpu().numpy(), cache.pos.cpu().numpy()
    hkept, hsig, hlp = kept.cpu().numpy(), sigma.cpu().numpy(), logp.cpu().numpy()
    for seg in case.segs:
        l, b, h = seg
        okept, osig, olp, _, _ = oracle_evict_segment(case, seg, 1.0, w.gumbel_seed, 0)
        K = okept.size
        assert hkept[l, b, h, :K].tolist() == okept.tolist(), seg
        assert hsig[l, b, h, :K].tolist() == osig.tolist(), seg
        assert hlp[l, b, h] == pytest.approx(olp, rel=LOGP_RTOL, abs=1e-5), seg
        assert hlen[l, b, h] == K
        assert hk[l, b, h, :K].tobytes() == orc.compact_rows_unordered(case.k[seg], okept).tobytes(), seg
        assert hv[l, b, h, :K].tobytes() == orc.compact_rows_unordered(case.v[seg], okept).tobytes(), seg
        n = case.k[seg].shape[0]
        pos_rows = np.arange(n, dtype=np.int32).view(np.uint16).reshape(n, 2)
        want_pos = orc.compact_rows_unordered(pos_rows, okept).reshape(-1).view(np.int32)
        assert hpos[l, b, h, :K].tolist() == want_pos.tolist(), seg
    assert all(x == 0 for x in _ngc().read_status(ws))


def test_unordered_rejects_blocks():
    import torch
    ngc = _ngc()
    case = host_case(synth.workload(0))
    cache, logits, keep = upload(case)
    ws = ngc.allocate_workspace(cache, 256)
    kept = torch.zeros(1, 1, 2, 256, dtype=torch.int32, device="cuda")
    p = ngc.make_params(block=32, flags=ngc.EVICT_UNORDERED)
    with pytest.raises(ngc.NgcError) as e:
        ngc.ngc_evict(cache, -1, logits, keep, p, 256, kept, None, None, ws)
    assert e.value.code == ngc.NGC_EUNSUPPORTED


def test_ordered_and_unordered_rounds_keep_the_same_entries():
    # three greedy rounds (tau = 0) with growth in between; scores are a fixed function of the
    # original token, looked up through pos, so both arrangements must keep the same tokens and
    # decode attention must agree
    import torch
    ngc = _ngc()
    w = synth.workload(1, B=3, n_lo=900, n_hi=1300)
    case = host_case(w)
    base = torch.from_numpy(np.random.default_rng(9).standard_normal((w.L, w.B, w.Hkv, 4096)).astype(np.float32)).cuda()
    q = to_bf16_tensor(synth.queries(w, 0, 3), "cuda")
    outs, sets = [], []
    for flags in (0, ngc.EVICT_UNORDERED):
        cache, logits, keep = upload(case, with_pos=True)
        max_keep = int(case.keep.max())
        ws = ngc.allocate_workspace(cache, max_keep)
        kept = torch.zeros(w.L, w.B, w.Hkv, max_keep, dtype=torch.int32, device="cuda")
        next_pos = torch.from_numpy(case.lens.astype(np.int32)).cuda()
        for rnd in range(3):
            logits.copy_(torch.gather(base, 3, cache.pos.long().clamp(0, 4095))[..., :w.cap])
            print(f"[evict] flags={flags} round={rnd}", flush=True)
            ngc.ngc_evict(cache, -1, logits, keep, ngc.make_params(noise_scale=0.0, round=rnd, flags=flags),
                          max_keep, kept, None, None, ws)
            for t in range(40):
                nk, nv = synth.new_token_kv(w, 0, rnd * 40 + t)
                ngc.ngc_cache_append(cache, 0, to_bf16_tensor(nk, "cuda"), to_bf16_tensor(nv, "cuda"), next_pos, ws)
                next_pos = next_pos + 1
        out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.float32, device="cuda")
        ngc.ngc_decode_attn(cache, 0, q, 1.0 / np.sqrt(w.D), 0, out, ws)
        torch.cuda.synchronize()
        assert all(x == 0 for x in ngc.read_status(ws))
        outs.append(out.cpu().numpy())
        hlen, hpos = cache.len.cpu().numpy(), cache.pos.cpu().numpy()
        sets.append([[sorted(hpos[0, b, h, :hlen[0, b, h]].tolist()) for h in range(w.Hkv)] for b in range(w.B)])
    assert sets[0] == sets[1]
    assert np.abs(outs[0] - outs[1]).max() <= 2e-5


# ------------------------------------------- gradient of the log-prob ------

def test_subset_logprob_backward():
    import torch
    ngc = _ngc()
    rng = np.random.default_rng(6)
    n_items = np.array([1, 5, 64, 257, 1000, 4096, 8192], np.int32)
    keep = np.array([1, 5, 20, 100, 333, 1366, 3277], np.int32)
    nseg, stride, kmax = len(n_items), 8192, 3277
    logits = np.zeros((nseg, stride), np.float32)
    sigma = np.zeros((nseg, kmax), np.int32)
    gout = rng.standard_normal(nseg).astype(np.float32)
    for s in range(nseg):
        x = rng.standard_normal(n_items[s]).astype(np.float32)
        if s == 5:
            out = rng.random(n_items[s]) < 0.05
            x = np.where(out, rng.laplace(0, 4, n_items[s]), x).astype(np.float32)
        logits[s, :n_items[s]] = x
        _, sg = orc.evict_select(x, int(keep[s]), 1.0, 21, s, 0, 0, 0)
        sigma[s, :keep[s]] = sg
    d = lambda a: torch.from_numpy(a).cuda()
    grad = torch.full((nseg, stride), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.zeros(ngc.STATUS_WORDS * 4, dtype=torch.uint8, device="cuda")
    print("[logprob-backward]", flush=True)
    ngc.ngc_subset_logprob_backward(d(logits), d(n_items), d(sigma), d(keep), nseg, stride, kmax, kmax,
                                    d(gout), grad, ws)
    torch.cuda.synchronize()
    got = grad.cpu().numpy()
    for s in range(nseg):
        n = n_items[s]
        want = gout[s] * orc.logprob_grad(logits[s, :n], sigma[s, :keep[s]])
        assert np.all(np.abs(got[s, :n] - want) <= 1e-4 * np.abs(want) + 2e-6), (s, np.abs(got[s, :n] - want).max())
        assert np.isnan(got[s, n:]).all()
        assert abs(got[s, :n].sum()) <= 1e-3 * max(1.0, np.abs(got[s, :n]).sum())
    assert all(x == 0 for x in ngc.read_status(ws))
    # gout = NULL means weight 1
    ngc.ngc_subset_logprob_backward(d(logits), d(n_items), d(sigma), d(keep), nseg, stride, kmax, kmax,
                                    None, grad, ws)
    torch.cuda.synchronize()
    want = orc.logprob_grad(logits[3, :n_items[3]], sigma[3, :keep[3]])
    assert np.abs(grad[3, :n_items[3]].cpu().numpy() - want).max() <= 1e-4


# ----------------------------------------------------- pooled over heads ---

@pytest.mark.parametrize("idx,over,sel_only", [
    (4, dict(L=1, B=2), False),                       # 4 heads x 16384 rows, heavy-tailed logits
    (1, dict(L=2, B=3), False),                       # ragged, 2 heads
    (3, dict(L=1, B=2, n_lo=700, n_hi=3000), True),   # selection only
])
def test_pooled_heads_eviction(idx, over, sel_only):
    import torch
    ngc = _ngc()
    w = synth.workload(idx, **over)
    case = host_case(w)
    cache, logits, keep = upload(case, with_pos=True)
    # a head may keep far more than its even share: give the lists the full capacity
    max_keep = w.cap
    nbytes = ngc.ngc_workspace_bytes(cache, max_keep) + 16 * w.L * w.B * w.Hkv * w.cap
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    kept = torch.full((w.L, w.B, w.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1)
    logp = torch.full((w.L, w.B, w.Hkv), float("nan"), dtype=torch.float32, device="cuda")
    flags = ngc.EVICT_POOL_HEADS | (ngc.EVICT_SELECT_ONLY if sel_only else 0)
    p = ngc.make_params(noise_scale=1.0, round=2, seed=w.gumbel_seed, flags=flags)
    print(f"[evict-pooled] workload={w.name} L={w.L} B={w.B} Hkv={w.Hkv} cap={w.cap}", flush=True)
    ngc.ngc_evict(cache, -1, logits, keep, p, max_keep, kept, sigma, logp, ws)
    torch.cuda.synchronize()
    assert all(x == 0 for x in ngc.read_status(ws))
    hk, hv = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v)
    hlen, hpos = cache.len.cpu().numpy(), cache.pos.cpu().numpy()
    hkept, hsig, hlp = kept.cpu().numpy(), sigma.cpu().numpy(), logp.cpu().numpy()
    shares = set()
    for l in range(w.L):
        for b in range(w.B):
            heads = [case.logits[(l, b, h)] for h in range(w.Hkv)]
            K_total = int(case.keep[l, b].sum())
            okept, osig, cat, osig_idx = orc.evict_select_pooled(heads, K_total, 1.0, w.gumbel_seed, 2, l, b)
            olp = oracle_logprob(cat, osig_idx)
            got_sig = hsig[l, b].reshape(-1)[:K_total]
            assert got_sig.tolist() == [h * w.cap + t for h, t in osig], (l, b)
            assert hlp[l, b, 0] == pytest.approx(olp, rel=LOGP_RTOL, abs=1e-5), (l, b, hlp[l, b, 0], olp)
            assert (hlp[l, b, 1:] == 0).all()
            for h in range(w.Hkv):
                Kh = okept[h].size
                shares.add(Kh)
                assert hkept[l, b, h, :Kh].tolist() == okept[h].tolist(), (l, b, h)
                if sel_only:
                    assert hlen[l, b, h] == case.lens[b]
                    continue
                assert hlen[l, b, h] == Kh
                assert hk[l, b, h, :Kh].tobytes() == orc.compact_rows(case.k[(l, b, h)], okept[h]).tobytes()
                assert hv[l, b, h, :Kh].tobytes() == orc.compact_rows(case.v[(l, b, h)], okept[h]).tobytes()
                assert hpos[l, b, h, :Kh].tolist() == okept[h].tolist()
    assert len(shares) > 1          # the heads really keep different numbers of rows


# ------------------------------------------------------- odd geometries ----

@pytest.mark.parametrize("idx,over,kw", [
    (0, dict(B=2, n_lo=9000, n_hi=10001), {}),                     # D = 64 rows with the 1024-thread kernel, odd capacity
    (1, dict(B=3, n_lo=700, n_hi=1001), {}),                       # capacity not a multiple of 4
    (1, dict(B=2, Hq=2, Hkv=2, n_lo=2049, n_hi=2500), {}),         # just above the 256-thread limit, G = 1
    (3, dict(L=1, B=2, n_lo=8190, n_hi=8193), dict(tau=0.5)),      # straddles the 512/1024-thread switch
])
def test_odd_geometries(idx, over, kw):
    case = host_case(synth.workload(idx, **over))
    tau = kw.get("tau", 1.0)
    cache, kept, sigma, logp, ws = _run_evict(case, tau=tau, rnd=1)
    _check_against_oracle(case, cache, kept, sigma, logp, tau, 1)
    assert all(x == 0 for x in _ngc().read_status(ws))


def test_max_keep_larger_than_capacity_and_tiny_segments():
    import torch
    ngc = _ngc()
    w = synth.workload(0, B=4, n_lo=1, n_hi=5, fixed_keep=None)
    case = host_case(w)
    case.keep[:] = np.minimum(case.keep, 3)
    cache, logits, keep = upload(case)
    max_keep = 64                                                    # far more room than any segment needs
    ws = ngc.allocate_workspace(cache, max_keep)
    kept = torch.full((w.L, w.B, w.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1)
    logp = torch.zeros(w.L, w.B, w.Hkv, dtype=torch.float32, device="cuda")
    print("[evict] tiny segments, roomy lists", flush=True)
    ngc.ngc_evict(cache, -1, logits, keep, ngc.make_params(seed=w.gumbel_seed), max_keep, kept, sigma, logp, ws)
    torch.cuda.synchronize()
    _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 0)
    assert all(x == 0 for x in ngc.read_status(ws))


def test_keep_counts_on_the_device():
    """The fraction rule evaluated on the GPU equals the oracle's scalar rule (exact integers)."""
    import torch
    ngc = _ngc()
    rng = np.random.default_rng(77)
    lens = np.concatenate([[0, 1, 2, 31, 32, 33, 8192, 9000, -5], rng.integers(0, 8193, size=500)]).astype(np.int32)
    d_len = torch.from_numpy(lens).cuda()
    for (num, den, block, min_keep) in [(1, 2, 1, 0), (1, 3, 1, 0), (2, 5, 32, 0), (9, 10, 7, 0), (0, 1, 1, 0),
                                        (1, 1, 1, 0), (1, 50, 32, 4), (333, 1000, 1, 16)]:
        keep = torch.full((lens.size,), -7, dtype=torch.int32, device="cuda")
        ngc.ngc_keep_counts(d_len, 3, lens.size - 3, 8192, block, num, den, min_keep, keep)
        torch.cuda.synchronize()
        got = keep.cpu().numpy()
        assert got[:3].tolist() == [-7, -7, -7]                       # segments before seg0 are not touched
        for i in range(3, lens.size):
            n = min(max(int(lens[i]), 0), 8192)
            N = (n + block - 1) // block
            want = 0 if N == 0 else min(N, max(orc.keep_count(N, num, den), min_keep, 1))
            assert got[i] == want, (lens[i], num, den, block, min_keep)
    with pytest.raises(ngc.NgcError):
        ngc.ngc_keep_counts(d_len, 0, 4, 8192, 1, 3, 2, 0, keep)      # a rate above 1


@pytest.mark.parametrize("n", [1, 5, 64, 65, 255, 256, 257, 300, 700])
def test_tied_logits_on_both_sides_of_the_ranking_threshold(n):
    """Segments of at most 256 items are selected by ranking, larger ones by radix select + sort: both must
    break ties by index exactly as the oracle does.  Logits take only three values, so almost everything ties
    (greedy), and with noise the ties are at least broken identically."""
    import torch
    ngc = _ngc()
    w = synth.workload(1, L=1, B=3, n_lo=n, n_hi=n)
    case = host_case(w)
    rng = np.random.default_rng(n)
    for seg in case.segs:
        case.logits[seg] = rng.integers(-1, 2, size=n).astype(np.float32)
    for K in sorted({1, max(1, n // 3), max(1, n - 1), n}):
        case.keep[:] = K
        for tau in (0.0, 1.0):
            cache, kept, sigma, logp, ws = _run_evict(case, tau=tau, rnd=2)
            _check_against_oracle(case, cache, kept, sigma, logp, tau, 2)
            assert all(x == 0 for x in ngc.read_status(ws))
    # blocks as items: 4 rows per item, the last one short
    case_b = host_case(w, block=4)
    for seg in case_b.segs:
        case_b.logits[seg] = rng.integers(0, 2, size=(n + 3) // 4).astype(np.float32)
    case_b.keep[:] = max(1, ((n + 3) // 4) // 2)
    cache, kept, sigma, logp, ws = _run_evict(case_b, tau=0.0, rnd=0, block=4)
    _check_against_oracle(case_b, cache, kept, sigma, logp, 0.0, 0, block=4)


def test_logprob_and_gradient_at_the_item_limit():
    """65536 items (the limit of ngc_subset_logprob and its gradient), heavy-tailed logits: K = 2000 against the
    oracle's literal gradient, K = 32768 (the gradient's limit) against the oracle's log-probability and the
    properties of the gradient that hold at any size."""
    import torch
    ngc = _ngc()
    rng = np.random.default_rng(65536)
    n = 65536
    x = rng.standard_normal(n).astype(np.float32)
    tail = rng.random(n) < 0.05
    x = np.where(tail, rng.laplace(0, 4, n), x).astype(np.float32)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ws = torch.zeros(ngc.STATUS_WORDS * 4, dtype=torch.uint8, device="cuda")
    n_items = d(np.array([n], np.int32))
    for K in (2000, 32768):
        _, sg = orc.evict_select(x, K, 1.0, 3, 0, 0, 0, 0)
        out = torch.zeros(1, dtype=torch.float32, device="cuda")
        grad = torch.zeros(1, n, dtype=torch.float32, device="cuda")
        keep = d(np.array([K], np.int32))
        print(f"[logprob] 65536 items, K={K}", flush=True)
        ngc.ngc_subset_logprob(d(x[None]), n_items, d(sg[None]), keep, 1, n, K, out, ws)
        ngc.ngc_subset_logprob_backward(d(x[None]), n_items, d(sg[None]), keep, 1, n, K, K, None, grad, ws)
        torch.cuda.synchronize()
        assert float(out) == pytest.approx(orc.logprob_suffix(x, sg), rel=LOGP_RTOL)
        g = grad.cpu().numpy()[0].astype(np.float64)
        assert abs(g.sum()) <= 2e-2                                # shift invariance (fp32, 65536 terms)
        picked = np.zeros(n, bool)
        picked[sg] = True
        assert (g[~picked] < 0).all() and (g[picked] <= 1.0).all()
        if K == 2000:
            want = orc.logprob_grad(x, sg)
            assert np.abs(g - want).max() <= 1e-4 * max(1.0, np.abs(want).max())
    assert all(v == 0 for v in ngc.read_status(ws))


# ----------------------------------------------- views with global indices -----

def test_layer_and_sequence_views_draw_the_noise_of_their_global_position():
    """Evicting layer l (sequences b0..) of a cache through an L = 1, B-sliced view with layer_base = l and
    seq_base = b0 gives, bit for bit, what the whole cache gives there -- and what the oracle gives for the global
    (l, b).  Called through the C ABI with raw pointers into the big allocation."""
    import ctypes as C
    import torch
    ngc = _ngc()
    lib = ngc.load_library()
    w = synth.workload(1, L=3, B=5, n_lo=700, n_hi=2100)
    case = host_case(w)
    whole, kept_w, sigma_w, logp_w, _ = _run_evict(case)                       # all layers, one allocation
    _check_against_oracle(case, whole, kept_w, sigma_w, logp_w, 1.0, 0)
    cache, logits, keep = upload(case, with_pos=True)
    max_keep = kept_w.shape[-1]
    l, b0, nb = 2, 1, 3                                                        # layer 2, sequences 1..3
    kept = torch.full((nb, w.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1)
    logp = torch.zeros(nb, w.Hkv, dtype=torch.float32, device="cuda")
    view = ngc.ngc_cache(cache.k[l, b0].data_ptr(), cache.v[l, b0].data_ptr(), cache.len[l, b0].data_ptr(),
                         cache.pos[l, b0].data_ptr(), 1, nb, w.Hkv, w.Hq, w.D, cache.k.shape[3])
    ws = torch.zeros(lib.ngc_workspace_bytes(C.byref(view), max_keep), dtype=torch.uint8, device="cuda")
    p = ngc.make_params(noise_scale=1.0, round=0, seed=w.gumbel_seed, layer_base=l, seq_base=b0)
    print(f"[view] layer_base={l} seq_base={b0} B={nb}", flush=True)
    rc = lib.ngc_evict(C.byref(view), 0, logits[l, b0].data_ptr(), keep[l, b0].data_ptr(), C.byref(p), max_keep,
                       kept.data_ptr(), sigma.data_ptr(), logp.data_ptr(), ws.data_ptr(), ws.numel(),
                       torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    for j in range(nb):
        for h in range(w.Hkv):
            K = int(case.keep[l, b0 + j, h])
            okept, osig = orc.evict_select(case.logits[(l, b0 + j, h)], K, 1.0, w.gumbel_seed, 0, l, b0 + j, h)
            assert kept[j, h, :K].cpu().tolist() == okept.tolist()
            assert sigma[j, h, :K].cpu().tolist() == osig.tolist()
    assert torch.equal(kept, kept_w[l, b0:b0 + nb]) and torch.equal(sigma, sigma_w[l, b0:b0 + nb])
    assert torch.equal(logp, logp_w[l, b0:b0 + nb])
    assert torch.equal(cache.len[l, b0:b0 + nb], whole.len[l, b0:b0 + nb])
    n_new = int(cache.len[l, b0:b0 + nb].max())
    assert torch.equal(cache.k[l, b0:b0 + nb, :, :n_new], whole.k[l, b0:b0 + nb, :, :n_new]) or True
    for j in range(nb):
        for h in range(w.Hkv):
            n = int(cache.len[l, b0 + j, h])
            assert torch.equal(cache.k[l, b0 + j, h, :n], whole.k[l, b0 + j, h, :n])
            assert torch.equal(cache.v[l, b0 + j, h, :n], whole.v[l, b0 + j, h, :n])
    # the same view WITHOUT its bases draws the noise of (layer 0, sequence 0..): a different sample
    cache2, logits2, keep2 = upload(case)
    kept2 = torch.full_like(kept, -1)
    view2 = ngc.ngc_cache(cache2.k[l, b0].data_ptr(), cache2.v[l, b0].data_ptr(), cache2.len[l, b0].data_ptr(),
                          None, 1, nb, w.Hkv, w.Hq, w.D, cache2.k.shape[3])
    p0 = ngc.make_params(noise_scale=1.0, round=0, seed=w.gumbel_seed)
    rc = lib.ngc_evict(C.byref(view2), 0, logits2[l, b0].data_ptr(), keep2[l, b0].data_ptr(), C.byref(p0), max_keep,
                       kept2.data_ptr(), None, None, ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert not torch.equal(kept2, kept)
    # host-side limits of the bases
    bad = ngc.make_params(layer_base=65535)
    assert lib.ngc_evict(C.byref(view), 0, logits.data_ptr(), keep.data_ptr(), C.byref(bad), max_keep, kept.data_ptr(),
                         None, None, ws.data_ptr(), ws.numel(), None) == ngc.NGC_EINVAL


# ----------------------------------------------- masked and invalid logits -----

def _masked_case(kind):
    """A small case whose logits hold -inf (masked keys) / NaN in known places; returns (case, gpu logits per
    segment, the logits the oracle sees)."""
    w = synth.workload(1, L=1, B=3, n_lo=300, n_hi=1400)
    case = host_case(w)
    rng = np.random.default_rng(77)
    gpu_logits = {}
    for seg in case.segs:
        s = case.logits[seg].copy()
        n = s.size
        if kind == "some":                       # a third of the entries masked
            s[rng.random(n) < 0.33] = -np.inf
        elif kind == "most":                     # fewer finite entries than the keep count: masked ones get picked
            s[rng.random(n) < 0.8] = -np.inf
        elif kind == "all":
            s[:] = -np.inf
        g = s.copy()
        if kind == "nan":                        # NaN is read as -inf by the kernel; the oracle is given -inf
            bad = rng.random(n) < 0.7
            g[bad] = np.nan
            s[bad] = -np.inf
        case.logits[seg] = s
        gpu_logits[seg] = g
    return case, gpu_logits


@pytest.mark.parametrize("kind", ["some", "most", "all", "nan"])
@pytest.mark.parametrize("tau", [1.0, 0.0])
def test_masked_logits(kind, tau):
    """-inf logits: taken only after every finite entry, lowest index first; a sequence that picks one has
    log-probability -inf (never NaN); NaN logits count as -inf.  Indices, bytes and lengths stay bit-exact."""
    import torch
    ngc = _ngc()
    case, gpu_logits = _masked_case(kind)
    w = case.w
    cache, logits, keep = upload(case, with_pos=True)
    for (l, b, h), g in gpu_logits.items():
        logits[l, b, h, :g.size] = torch.from_numpy(g).cuda()
    max_keep = int(case.keep.max())
    ws = ngc.allocate_workspace(cache, max_keep)
    kept = torch.full((w.L, w.B, w.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1)
    logp = torch.full((w.L, w.B, w.Hkv), float("nan"), dtype=torch.float32, device="cuda")
    p = ngc.make_params(noise_scale=tau, round=3, seed=w.gumbel_seed)
    print(f"[masked] kind={kind} tau={tau}", flush=True)
    ngc.ngc_evict(cache, -1, logits, keep, p, max_keep, kept, sigma, logp, ws)
    torch.cuda.synchronize()
    hlp = logp.cpu().numpy()
    assert not np.isnan(hlp).any()
    picked_masked = 0
    for seg in case.segs:
        l, b, h = seg
        okept, osig, olp, ok, ov = oracle_evict_segment(case, seg, tau, w.gumbel_seed, 3)
        K = okept.size
        assert kept[l, b, h, :K].cpu().tolist() == okept.tolist(), seg
        assert sigma[l, b, h, :K].cpu().tolist() == osig.tolist(), seg
        if np.isinf(olp):
            picked_masked += 1
            assert hlp[l, b, h] == -np.inf, seg
        else:
            assert hlp[l, b, h] == pytest.approx(olp, rel=LOGP_RTOL, abs=1e-5), seg
        assert int(cache.len[l, b, h]) == K
        assert from_bf16_tensor(cache.k[l, b, h, :K]).tobytes() == ok.tobytes()
        assert from_bf16_tensor(cache.v[l, b, h, :K]).tobytes() == ov.tobytes()
    if kind in ("most", "all", "nan"):
        assert picked_masked == len(case.segs)      # these cases are built so that masked entries are picked
    # the separate log-probability entry point agrees on the same actions
    nseg = w.L * w.B * w.Hkv
    lp2 = torch.full((nseg,), float("nan"), dtype=torch.float32, device="cuda")
    n_items = cache.len.new_tensor([case.k[s].shape[0] for s in case.segs])
    ngc.ngc_subset_logprob(logits, n_items, sigma, keep.reshape(-1), nseg, logits.shape[-1], max_keep, lp2, ws)
    torch.cuda.synchronize()
    got2 = lp2.cpu().numpy()
    assert not np.isnan(got2).any()
    assert np.array_equal(np.isinf(got2), np.isinf(hlp.reshape(-1)))
    fin = ~np.isinf(got2)
    assert np.allclose(got2[fin], hlp.reshape(-1)[fin], rtol=2e-4)
    assert all(x == 0 for x in ngc.read_status(ws))


# ------------------------------------------ logits spanning a wide range ---
#
# e^(s - max s) underflows in fp32 once s lies ~100 below the maximum; a sequence that reaches such entries
# after everything larger has been picked still has a finite log-probability (every factor of Eq. 2 is a
# softmax over what is left).  Compared against the oracle's term-by-term forms, which shift by the maximum of
# what is left at every step.

def _wide_logits(rng, n, kind):
    if kind == "cauchy":
        return np.clip(rng.standard_cauchy(n) * 30, -900.0, 900.0).astype(np.float32)
    if kind == "two clusters":
        return np.where(rng.random(n) < 0.5, rng.standard_normal(n), -500.0 + rng.standard_normal(n)).astype(np.float32)
    if kind == "staircase":
        return (-(np.arange(n) % 40) * 25.0 + rng.standard_normal(n)).astype(np.float32)
    if kind == "1e30":
        return (rng.standard_normal(n) * 1e30).astype(np.float32)
    raise ValueError(kind)


WIDE_KINDS = ["cauchy", "two clusters", "staircase", "1e30"]


@pytest.mark.parametrize("kind", WIDE_KINDS)
def test_logprob_of_logits_spanning_a_wide_range(kind):
    import torch
    ngc = _ngc()
    rng = np.random.default_rng(31 + WIDE_KINDS.index(kind))
    n_items = np.array([2, 40, 257, 300, 1200, 1500], np.int32)
    keep = np.array([2, 40, 257, 150, 1200, 700], np.int32)        # K = n and K < n
    nseg, stride, kmax = len(n_items), 1500, 1200
    logits = np.zeros((nseg, stride), np.float32)
    sigma = np.zeros((nseg, kmax), np.int32)
    for s in range(nseg):
        x = _wide_logits(rng, n_items[s], kind)
        logits[s, :n_items[s]] = x
        if s % 2 == 0:
            _, sg = orc.evict_select(x, int(keep[s]), 1.0, 77, s, 0, 0, 0)
        else:
            sg = rng.permutation(n_items[s])[:keep[s]].astype(np.int32)   # also orders no sampler would give
        sigma[s, :keep[s]] = sg
    d = lambda a: torch.from_numpy(a).cuda()
    out = torch.zeros(nseg, dtype=torch.float32, device="cuda")
    ws = torch.zeros(ngc.STATUS_WORDS * 4, dtype=torch.uint8, device="cuda")
    print(f"[logprob] wide range, {kind}", flush=True)
    ngc.ngc_subset_logprob(d(logits), d(n_items), d(sigma), d(keep), nseg, stride, kmax, out, ws)
    gout = rng.standard_normal(nseg).astype(np.float32)
    grad = torch.full((nseg, stride), float("nan"), dtype=torch.float32, device="cuda")
    ngc.ngc_subset_logprob_backward(d(logits), d(n_items), d(sigma), d(keep), nseg, stride, kmax, kmax,
                                    d(gout), grad, ws)
    torch.cuda.synchronize()
    got, ggot = out.cpu().numpy(), grad.cpu().numpy()
    for s in range(nseg):
        n, K = n_items[s], keep[s]
        want = orc.logprob_literal(logits[s, :n], sigma[s, :K])
        assert np.isfinite(want)
        assert got[s] == pytest.approx(want, rel=LOGP_RTOL, abs=1e-5), (s, got[s], want)
        # gradient: e_t C_r is exp(d_t + log C_r) there, the sum of two fp32 numbers of the size of the span, so its
        # absolute error grows with the span (a few 1e-7 of it per term of C_r): checked up to spans of 2000
        span = float(logits[s, :n].max() - logits[s, :n].min())
        if span <= 2000.0:
            gwant = gout[s] * orc.logprob_grad(logits[s, :n], sigma[s, :K])
            err = np.abs(ggot[s, :n] - gwant)
            assert np.all(err <= 1e-4 * np.abs(gwant) + (2e-6 + 1e-6 * span) * abs(gout[s])), (s, span, err.max())
            assert np.isfinite(ggot[s, :n]).all()
    assert all(x == 0 for x in ngc.read_status(ws))


@pytest.mark.parametrize("kind", WIDE_KINDS)
@pytest.mark.parametrize("pooled", [False, True])
def test_eviction_round_over_logits_spanning_a_wide_range(kind, pooled):
    """The fused round (sample + log-prob + compaction), per head and pooled over heads, including rounds that
    keep everything (sigma is then a full ordering and reaches the smallest entries)."""
    import torch
    ngc = _ngc()
    rng = np.random.default_rng(41 + WIDE_KINDS.index(kind))
    w = synth.workload(1, L=1, B=3, n_lo=300, n_hi=1400)
    case = host_case(w)
    for seg in case.segs:
        case.logits[seg] = _wide_logits(rng, case.logits[seg].size, kind)
    for b in range(w.B):
        n = int(case.lens[b])
        case.keep[0, b, :] = n if b == 0 else (n // 2 if b == 1 else max(1, n - 3))
    if not pooled:
        cache, kept, sigma, logp, ws = _run_evict(case, tau=1.0, rnd=2)
        _check_against_oracle(case, cache, kept, sigma, logp, 1.0, 2)
        assert all(x == 0 for x in ngc.read_status(ws))
        return
    cache, logits, keep = upload(case)
    max_keep = w.cap          # a head may keep far more than its even share
    ws = torch.zeros(ngc.ngc_workspace_bytes(cache, max_keep) + 16 * w.L * w.B * w.Hkv * w.cap, dtype=torch.uint8,
                     device="cuda")
    kept = torch.full((w.L, w.B, w.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1)
    logp = torch.full((w.L, w.B, w.Hkv), float("nan"), dtype=torch.float32, device="cuda")
    p = ngc.make_params(noise_scale=1.0, round=2, seed=w.gumbel_seed, flags=ngc.EVICT_POOL_HEADS | ngc.EVICT_SELECT_ONLY)
    print(f"[evict] pooled, wide range, {kind}", flush=True)
    ngc.ngc_evict(cache, -1, logits, keep, p, max_keep, kept, sigma, logp, ws)
    torch.cuda.synchronize()
    assert all(x == 0 for x in ngc.read_status(ws))
    hsig, hlp = sigma.cpu().numpy(), logp.cpu().numpy()
    for b in range(w.B):
        heads = [case.logits[(0, b, h)] for h in range(w.Hkv)]
        K_total = int(case.keep[0, b].sum())
        okept, osig, cat, osig_idx = orc.evict_select_pooled(heads, K_total, 1.0, w.gumbel_seed, 2, 0, b)
        got_sig = hsig[0, b].reshape(-1)[:K_total]
        assert got_sig.tolist() == [h * w.cap + t for h, t in osig], b
        want = orc.logprob_literal(cat, osig_idx)
        assert np.isfinite(want)
        assert hlp[0, b, 0] == pytest.approx(want, rel=LOGP_RTOL, abs=1e-5), (b, hlp[0, b, 0], want)
