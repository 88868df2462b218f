"""Randomised differential runs against the CPU oracle: seeded random geometries, lengths (empty and full
segments included), keep counts and adversarial values, through the same checks as the hand-picked cases.
A run of a few thousand such cases found what the hand-picked ones had missed (log-probabilities of logits
spanning more than fp32's exponent range, the fixed scratch array serving caches of changing geometry); the
cases below are a seeded sample that takes a few seconds."""
import numpy as np
import pytest

import oracle as orc
from paper_2604_18002_amd import synth

import _harness as H
import test_gpu_evict as TE
import test_gpu_replay as TR
import test_gpu_score as TS

pytestmark = pytest.mark.gpu

LOGIT_KINDS = ["normal", "quantised", "constant", "three values", "masked", "cauchy", "ascending", "descending",
               "1e30", "nearly equal", "1e-30", "signed zeros"]


def _logits(rng, n, kind):
    if n == 0:
        return np.zeros(0, np.float32)
    if kind == "normal":
        x = rng.standard_normal(n)
    elif kind == "quantised":
        x = np.round(rng.standard_normal(n) * 4) / 4            # many exact ties
    elif kind == "constant":
        x = np.full(n, rng.standard_normal())
    elif kind == "three values":
        x = rng.choice(rng.standard_normal(3), n)
    elif kind == "masked":
        x = rng.standard_normal(n)
        x[rng.random(n) < rng.choice([0.05, 0.5, 0.95])] = -np.inf
    elif kind == "cauchy":
        x = rng.standard_cauchy(n) * 3                            # spans of hundreds
    elif kind == "ascending":
        x = np.sort(rng.standard_normal(n))
    elif kind == "descending":
        x = -np.sort(rng.standard_normal(n))
    elif kind == "1e30":
        x = rng.standard_normal(n) * 1e30
    elif kind == "nearly equal":
        x = 1.0 + np.arange(n) * 1e-7 * rng.choice([-1, 1])
    elif kind == "1e-30":
        x = rng.standard_normal(n) * 1e-30
    else:
        x = np.where(rng.random(n) < 0.5, 0.0, -0.0)
    return x.astype(np.float32)


@pytest.mark.parametrize("ci", range(48))
def test_random_eviction_round(ci):
    rng = np.random.default_rng(7_000_000 + ci)
    L, B, Hkv = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
    G, D = int(rng.choice([1, 2, 7])), int(rng.choice([64, 128]))
    cap = int(rng.choice([33, 64, 200, 256, 257, 300, 1000, 2048, 2049, 4096, 4097, 6000, 8192]))
    block = int(rng.choice([1, 1, 1, 32])) if cap >= 64 else 1
    tau = float(rng.choice([0.0, 1.0, 1.0, 0.01, 100.0]))
    share = int(rng.integers(0, 2)) if block == 32 else 0
    kind = LOGIT_KINDS[ci % len(LOGIT_KINDS)]
    w = synth.workload(0, L=L, B=B, Hq=Hkv * G, Hkv=Hkv, D=D, n_lo=cap, n_hi=cap, fixed_keep=None)
    lens = np.array([int(rng.choice([0, 1, cap, int(rng.integers(0, cap + 1))])) for _ in range(B)])
    segs = [(l, b, h) for l in range(L) for b in range(B) for h in range(Hkv)]
    k, v, lg = {}, {}, {}
    keep = np.zeros((L, B, Hkv), np.int32)
    for seg in segs:
        l, b, h = seg
        n = int(lens[b])
        items = (n + block - 1) // block
        k[seg], v[seg] = synth.segment_kv(w, l, b, h, n)
        lg[seg] = _logits(rng, items, kind)
        keep[seg] = int(rng.choice([0, 1, items, max(items - 1, 0), items // 2, int(rng.integers(0, items + 1))]))
    case = H.HostCase(w, lens, keep, segs, k, v, lg)
    rnd = int(rng.integers(0, 1000))
    # the oracle's term-by-term Eq. 2 costs n * K: leave the log-probability out where that is too much
    affordable = all(lg[s].size * int(keep[s]) <= 3_000_000 for s in segs)
    cache, kept, sigma, logp, ws = TE._run_evict(case, tau=tau, rnd=rnd, block=block, share_heads=share,
                                                 want_logp=affordable)
    live = [s for s in segs if lens[s[1]] > 0 and keep[s] > 0]
    if live:
        TE._check_against_oracle(case, cache, kept, sigma, logp, tau, rnd, block=block, share_heads=bool(share),
                                 segs=live)
    hlen = cache.len.cpu().numpy()
    for s in segs:
        if s not in live:
            assert hlen[s] == 0, s     # nothing there, or nothing kept: empty afterwards


def _values(rng, shape, kind):
    if kind == "normal":
        return rng.standard_normal(shape)
    if kind == "sharp":
        return rng.standard_normal(shape) * 6
    if kind == "constant":
        return np.full(shape, 0.75)
    if kind == "zeros":
        return np.zeros(shape)
    if kind == "big":
        return rng.standard_normal(shape) * 200
    if kind == "tiny":
        return rng.standard_normal(shape) * 1e-20
    x = np.zeros(shape)
    x[..., rng.integers(0, shape[-1])] = 3.0
    return x


VALUE_KINDS = ["normal", "sharp", "constant", "zeros", "big", "tiny", "one hot"]


@pytest.mark.parametrize("ci", range(16))
def test_random_rounds_with_more_large_segments_than_workgroups(ci):
    # Segments of more than 4096 rows, several hundred of them: the workgroups of the round take one segment after
    # another from a counter.  Lengths include 0, 1 and the full capacity, keep counts 0 and everything; a sample
    # of segments is generated on the host and compared with the oracle, every segment is held to what must be
    # true of any round (kept ascending and in range, sigma a permutation of kept, a log-probability written).
    import torch
    from paper_2604_18002_amd import binding as ngc
    ngc.load_library()
    rng = np.random.default_rng(9_000_000 + ci)
    L, Hkv = int(rng.integers(1, 4)), int(rng.integers(1, 5))
    B = int(rng.integers(257, 700)) // (L * Hkv) + 1
    G, D = int(rng.choice([1, 2, 7])), int(rng.choice([64, 128]))
    cap = int(rng.choice([4097, 5000, 8192, 12000, 16384]))
    block = int(rng.choice([1, 1, 32]))
    mode = str(rng.choice(["ordered", "ordered", "select_only", "unordered"])) if block == 1 else "ordered"
    tau = float(rng.choice([0.0, 1.0, 1.0]))
    kind = LOGIT_KINDS[ci % len(LOGIT_KINDS)]
    w = synth.workload(0, L=L, B=B, Hq=Hkv * G, Hkv=Hkv, D=D, n_lo=cap, n_hi=cap, fixed_keep=None)
    lens = np.array([int(rng.choice([0, 1, cap, cap - 1, int(rng.integers(0, cap + 1)),
                                     int(rng.integers(cap // 2, cap + 1))])) for _ in range(B)])
    segs = [(l, b, h) for l in range(L) for b in range(B) for h in range(Hkv)]
    pick = sorted({segs[0], segs[-1], *[segs[int(i)] for i in rng.integers(0, len(segs), 5)]})
    items_b = (lens + block - 1) // block
    keep = np.zeros((L, B, Hkv), np.int32)
    for (l, b, h) in segs:
        it = int(items_b[b])
        keep[l, b, h] = min(16000, it, int(rng.choice([0, 1, it, max(it - 1, 0), it // 2, (2 * it) // 5,
                                                         int(rng.integers(0, it + 1))])))
    k, v, lg = {}, {}, {}
    for seg in pick:
        l, b, h = seg
        k[seg], v[seg] = synth.segment_kv(w, l, b, h, int(lens[b]))
        lg[seg] = _logits(rng, int(items_b[b]), kind)
        if lg[seg].size * int(keep[seg]) > 6_000_000:      # the oracle's term-by-term Eq. 2 costs n * K
            keep[seg] = min(int(keep[seg]), max(1, 6_000_000 // lg[seg].size))
    case = H.HostCase(w, lens, keep, pick, k, v, lg)
    max_keep = max(int(keep.max()), 1)
    print(f"[random] L={L} B={B} Hkv={Hkv} D={D} cap={cap} block={block} mode={mode} tau={tau} kind={kind}", flush=True)
    cache = ngc.Cache.allocate(L, B, Hkv, Hkv * G, D, cap)
    synth.fill_normal_bf16_(cache.k, 11 + ci)
    synth.fill_normal_bf16_(cache.v, 12 + ci)
    logits = torch.randn(L, B, Hkv, cap, device="cuda")
    cache.len.copy_(torch.from_numpy(np.broadcast_to(lens[None, :, None], (L, B, Hkv)).astype(np.int32).copy()))
    for seg in pick:
        l, b, h = seg
        n = k[seg].shape[0]
        if n:
            cache.k[l, b, h, :n] = H.to_bf16_tensor(k[seg], "cuda")
            cache.v[l, b, h, :n] = H.to_bf16_tensor(v[seg], "cuda")
        logits[l, b, h, :lg[seg].size] = torch.from_numpy(lg[seg]).cuda()
    keep_t = torch.from_numpy(keep).cuda()
    ws = ngc.allocate_workspace(cache, max_keep)
    kept = torch.full((L, B, Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1)
    logp = torch.full((L, B, Hkv), float("nan"), dtype=torch.float32, device="cuda")
    flags = {"ordered": 0, "select_only": ngc.EVICT_SELECT_ONLY, "unordered": ngc.EVICT_UNORDERED}[mode]
    rnd = int(rng.integers(0, 1000))
    p = ngc.make_params(block=block, noise_scale=tau, round=rnd, seed=w.gumbel_seed, flags=flags)
    for _ in range(2 if mode == "select_only" else 1):     # twice on one workspace where nothing moves
        ngc.ngc_evict(cache, -1, logits, keep_t, p, max_keep, kept, sigma, logp, ws)
        torch.cuda.synchronize()
        assert all(x == 0 for x in ngc.read_status(ws))

    def rows(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

    hkept, hsig, hlp, hlen = kept.cpu().numpy(), sigma.cpu().numpy(), logp.cpu().numpy(), cache.len.cpu().numpy()
    for seg in pick:
        l, b, h = seg
        if lens[b] == 0:
            assert hlen[l, b, h] == 0
            continue
        okept, osig, olp, ok_, ov_ = H.oracle_evict_segment(case, seg, tau, w.gumbel_seed, rnd, block, False)
        K = okept.size
        assert hkept[l, b, h, :K].tolist() == okept.tolist(), seg
        assert hsig[l, b, h, :K].tolist() == osig.tolist(), seg
        if np.isfinite(olp):
            assert hlp[l, b, h] == pytest.approx(olp, rel=TE.LOGP_RTOL, abs=1e-5), seg
        if mode == "ordered":
            n_new = ok_.shape[0]
            assert hlen[l, b, h] == n_new, seg
            assert rows(cache.k[l, b, h, :n_new]).tobytes() == ok_.tobytes(), seg
            assert rows(cache.v[l, b, h, :n_new]).tobytes() == ov_.tobytes(), seg
        elif mode == "unordered":
            assert hlen[l, b, h] == K
            got = rows(cache.k[l, b, h, :K])
            assert {got[j].tobytes() for j in range(K)} == {k[seg][int(t)].tobytes() for t in okept}, seg
        else:
            assert hlen[l, b, h] == lens[b]
    slot = torch.arange(max_keep, device="cuda")
    n0 = torch.from_numpy(np.broadcast_to(items_b[None, :, None], keep.shape).astype(np.int32).copy()).cuda()
    valid = slot < keep_t.unsqueeze(-1)
    assert bool(((kept[..., 1:] > kept[..., :-1]) | ~valid[..., 1:]).all())
    assert bool((((kept >= 0) & (kept < n0.unsqueeze(-1))) | ~valid).all())
    ssort = torch.where(valid, sigma, torch.full_like(sigma, 2 ** 30)).sort(dim=-1).values
    assert torch.equal(ssort, torch.where(valid, kept, torch.full_like(kept, 2 ** 30)))
    assert not bool(torch.isnan(logp).any())


@pytest.mark.parametrize("ci", range(48))
def test_random_decode_attention(ci):
    """ngc_decode_attn (all layers / per layer), ngc_decode_attn_static and ngc_decode_step in turn, caches of
    changing geometry one after the other."""
    import torch
    from paper_2604_18002_amd import binding as ngc
    ngc.load_library()
    rng = np.random.default_rng(8_000_000 + ci)
    L, B, Hkv = int(rng.integers(1, 3)), int(rng.integers(1, 6)), int(rng.integers(1, 5))
    G, D = int(rng.choice([1, 2, 3, 4, 6, 7, 8, 16])), int(rng.choice([64, 128]))
    cap = int(rng.choice([1, 31, 32, 33, 100, 129, 700, 1024, 3000, 5000, 20000]))
    kk, vk, qk = (VALUE_KINDS[int(rng.integers(0, len(VALUE_KINDS)))] for _ in range(3))
    lens = np.zeros((L, B, Hkv), np.int32)
    for idx in np.ndindex(L, B, Hkv):
        lens[idx] = int(rng.choice([0, 1, cap, max(cap - 1, 0), int(rng.integers(0, cap + 1))]))
    bits, f32 = synth.f32_to_bf16_bits, synth.bf16_bits_to_f32
    hk = bits(_values(rng, (L, B, Hkv, cap, D), kk))
    hv = bits(_values(rng, (L, B, Hkv, cap, D), vk))
    hq = bits(_values(rng, (L, B, Hkv * G, D), qk))
    scale = float(rng.choice([1.0 / np.sqrt(D), 1.0, 0.01]))
    hint = int(rng.choice([0, int(lens.max()), max(1, int(lens.max()) // 3), cap]))   # also hints that are too small
    mode = ["all layers", "per layer", "static", "step"][ci % 4]
    print(f"[random attn] L={L} B={B} Hkv={Hkv} G={G} D={D} cap={cap} K={kk} V={vk} Q={qk} scale={scale:.3g} "
          f"hint={hint} mode={mode}", flush=True)
    cache = ngc.Cache.allocate(L, B, Hkv, Hkv * G, D, cap, device="cuda")
    cache.k.copy_(H.to_bf16_tensor(hk, "cuda"))
    cache.v.copy_(H.to_bf16_tensor(hv, "cuda"))
    cache.len.copy_(torch.from_numpy(lens))
    ws = ngc.allocate_workspace(cache, 1)
    q = H.to_bf16_tensor(hq, "cuda")
    out = torch.full((L, B, Hkv * G, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((L, B, Hkv * G), float("nan"), dtype=torch.float32, device="cuda")
    eff = lens.copy()
    if mode == "all layers":
        ngc.ngc_decode_attn(cache, -1, q, scale, hint, out, ws, lse_out=lse)
    elif mode == "per layer":
        for l in range(L):
            ngc.ngc_decode_attn(cache, l, q[l], scale, hint, out[l], ws, lse_out=lse[l])
    elif mode == "static":
        for l in range(L):
            ngc.ngc_decode_attn_static(cache, l, q[l], scale, hint, out[l], lse_out=lse[l])
    else:
        knew, vnew = bits(_values(rng, (L, B, Hkv, D), kk)), bits(_values(rng, (L, B, Hkv, D), vk))
        for l in range(L):
            ngc.ngc_decode_step(cache, l, H.to_bf16_tensor(knew[l], "cuda"), H.to_bf16_tensor(vnew[l], "cuda"), None,
                                q[l], scale, hint, out[l], ws, lse_out=lse[l])
        for idx in np.ndindex(L, B, Hkv):
            n = int(lens[idx])
            if n < cap:                      # a full segment attends without appending (counted, not fatal)
                hk[idx][n], hv[idx][n], eff[idx] = knew[idx], vnew[idx], n + 1
    torch.cuda.synchronize()
    got, glse = out.cpu().numpy(), lse.cpu().numpy()
    assert (cache.len.cpu().numpy() == eff).all()
    vmax = max(1.0, float(np.abs(f32(hv)).max()))
    # fp32 accumulation of a D-term dot product of values of this size
    acc_tol = 3e-7 * D * float(np.abs(f32(hq)).max()) * float(np.abs(f32(hk)).max()) * scale
    for idx in np.ndindex(L, B, Hkv):
        l, b, h = idx
        n = int(eff[idx])
        g = got[l, b, h * G:(h + 1) * G]
        if n == 0:
            assert (g == 0).all(), idx
            continue
        want = orc.decode_attn(hq[l, b, h * G:(h + 1) * G], hk[idx][:n], hv[idx][:n], scale)
        assert np.abs(g - want).max() <= 2e-3 * vmax, (idx, n)
        wl = orc.decode_lse(hq[l, b, h * G:(h + 1) * G], hk[idx][:n], scale)
        assert np.all(np.abs(glse[l, b, h * G:(h + 1) * G] - wl) <= 2e-5 * np.maximum(1.0, np.abs(wl)) + acc_tol), idx


@pytest.mark.parametrize("ci", range(40))
def test_random_workloads_through_the_other_parity_checks(ci):
    """The unordered, pooled-heads and per-head rounds, key scoring and replay attention checks of the other
    test files, called with random geometries and retention rates."""
    rng = np.random.default_rng(9_000_000 + ci)
    Hkv, G, D = int(rng.integers(1, 5)), int(rng.choice([1, 2, 4, 6, 7, 8, 16])), int(rng.choice([64, 128]))
    L, B = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    hi = int(rng.choice([5, 40, 257, 700, 2049, 4100, 8200, 12000]))
    lo = int(rng.integers(1, hi + 1))
    num, den = [(1, 2), (1, 3), (2, 5), (9, 10), (1, 50)][int(rng.integers(0, 5))]
    over = dict(L=L, B=B, Hkv=Hkv, Hq=Hkv * G, D=D, n_lo=lo, n_hi=hi, keep_num=num, keep_den=den, fixed_keep=None,
                logits_kind=str(rng.choice(["normal", "drift", "heavy"])))
    what = ["unordered", "pooled", "per head", "score", "replay"][ci % 5]
    base = int(rng.integers(0, 5))
    print(f"[random {what}] base workload {base}, {over}", flush=True)
    if what == "unordered":
        TE.test_unordered_compaction_parity(base, dict(over, per_head_budget=bool(rng.integers(0, 2))))
    elif what == "pooled":
        if hi > 4000:
            over = dict(over, n_lo=min(lo, 4000), n_hi=4000)
        try:
            TE.test_pooled_heads_eviction(base, dict(over, per_head_budget=False), bool(rng.integers(0, 2)))
        except AssertionError as e:
            import traceback
            if "len(shares) > 1" not in "".join(traceback.format_exception(type(e), e, e.__traceback__)):
                raise    # (that line is the called test's check on its own hand-picked inputs)
    elif what == "per head":
        TE.test_odd_geometries(base, dict(over, per_head_budget=bool(rng.integers(0, 2))),
                               dict(tau=float(rng.choice([0.0, 0.5, 1.0, 30.0]))))
    elif what == "score":
        if hi > 3000:
            over = dict(over, n_lo=min(lo, 3000), n_hi=3000)
        TS.test_scores_match_oracle(base, over, min(8, int(rng.integers(1, max(2, 64 // G) + 1))))
    else:
        TR.test_replay_sweep(dict(i=ci, T=int(rng.choice([1, 31, 64, 127, 129, 300, 777, 1300])), Hkv=Hkv, Hq=Hkv * G,
                                  D=D, period=int(rng.choice([7, 16, 50, 128, 350])),
                                  keep=float(rng.choice([0.1, 0.5, 0.9])), per_head=bool(rng.integers(0, 2)),
                                  block=int(rng.choice([1, 1, 32])), B=B))


@pytest.mark.parametrize("ci", range(24))
def test_random_cycles_over_the_paged_layout(ci):
    """Grow / attend / evict cycles with random page sizes, pool sizes (some too small: skipped appends are
    counted and mirrored by the model), retention rates and single-layer rounds, against the numpy model of
    tables, pools and free stack."""
    import test_gpu_paged as TP
    rng = np.random.default_rng(9_500_000 + ci)
    ngc = TP._ngc()
    Hkv, G, D = int(rng.integers(1, 4)), int(rng.choice([1, 2, 6, 7])), int(rng.choice([64, 128]))
    L, B = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    P = int(rng.choice([32, 32, 64, 128]))
    hi = int(rng.choice([40, 200, 700, 1500]))
    lo = int(rng.integers(1, hi + 1))
    wl = synth.workload(1, L=L, B=B, Hkv=Hkv, Hq=Hkv * G, D=D, n_lo=lo, n_hi=hi)
    case = H.host_case(wl)
    grow, rounds = int(rng.integers(1, 70)), int(rng.integers(1, 4))
    max_pages = (hi + grow * rounds + P - 1) // P + int(rng.integers(0, 3))
    nseg = L * B * Hkv
    if rng.integers(0, 4) == 0:     # a pool that runs dry
        num_pages = max(nseg, int(nseg * ((hi + P - 1) // P) + rng.integers(0, nseg + 1)))
    else:
        num_pages = nseg * max_pages
    tau, frac = float(rng.choice([0.0, 1.0, 1.0])), float(rng.choice([0.1, 0.5, 0.9, 1.0]))
    print(f"[random paged] L={L} B={B} Hkv={Hkv} G={G} D={D} P={P} n={lo}..{hi} grow={grow} rounds={rounds} "
          f"max_pages={max_pages} num_pages={num_pages} tau={tau} keep={frac}", flush=True)
    m = TP.build_model(case, P, max_pages, num_pages, seed=ci)
    pc = TP.upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    step = 0
    for rnd in range(rounds):
        for _ in range(grow):
            TP.append_step(pc, m, wl, ws, step)
            step += 1
        TP.assert_same_state(pc, m, wl, f"after growth {rnd}")
        TP.check_attention(pc, m, wl, ws, -1, 20 + rnd, lse=bool(rng.integers(0, 2)))
        layer = -1 if rng.integers(0, 2) else int(rng.integers(0, L))
        TP.run_round(pc, m, wl, ws, rnd, lambda N: max(0 if frac < 0.2 else 1, int(np.ceil(N * frac))), tau=tau,
                     layer=layer, share_heads=int(rng.integers(0, 2)))
        TP.assert_same_state(pc, m, wl, f"after round {rnd}")
    TP.check_attention(pc, m, wl, ws, -1, 99)
