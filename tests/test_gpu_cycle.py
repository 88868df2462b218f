"""The whole cycle over several rounds, contiguous layout: grow (append + decode attention, keeping each
step's log-sum-exp), score the keys with the last w queries (one pass over K, normalisers from decode),
evict at the paper's granularity (blocks, scores pooled over heads, one noise draw per layer), repeat.
The oracle tracks its own copy of the cache; every decode output, every score vector, every sampled action
and the cache contents after every round are compared.  The eviction takes the ORACLE's scores (rounded to
fp32) as logits, so both sides select on identical numbers and the comparison stays bit-exact over rounds;
the kernel's own scores are checked against them within tolerance."""
import numpy as np
import pytest

import oracle as orc
from paper_2604_18002_amd import synth

from _harness import from_bf16_tensor, host_case, to_bf16_tensor, upload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block,D", [(8, 64), (32, 128)])
def test_three_rounds_of_score_evict_grow(block, D):
    import torch
    from paper_2604_18002_amd import binding as ngc
    delta, w_, rounds = 44, 5, 3
    wl = synth.workload(1, L=2, B=2, Hkv=2, Hq=6, D=D, n_lo=150, n_hi=330)
    case = host_case(wl)
    cap = wl.cap + delta + 8
    cache, _, _ = upload(case, with_pos=True, cap=cap)
    ws = ngc.allocate_workspace(cache, cap)
    scale = 1.0 / np.sqrt(D)
    G = wl.G
    # the oracle's copy of the cache: rows and original positions per segment
    ok = {s: case.k[s].copy() for s in case.segs}
    ov = {s: case.v[s].copy() for s in case.segs}
    opos = {s: np.arange(case.k[s].shape[0], dtype=np.int32) for s in case.segs}
    step = 0
    for rnd in range(rounds):
        recent_q, recent_lse = [], []
        for t in range(delta):
            nk = np.stack([synth.new_token_kv(wl, l, step)[0] for l in range(wl.L)])
            nv = np.stack([synth.new_token_kv(wl, l, step)[1] for l in range(wl.L)])
            q = np.stack([synth.queries(wl, l, 500 + step) for l in range(wl.L)])
            new_pos = torch.tensor([int(case.lens[b]) + step for b in range(wl.B)], dtype=torch.int32, device="cuda")
            ngc.ngc_cache_append(cache, -1, to_bf16_tensor(nk, "cuda"), to_bf16_tensor(nv, "cuda"), new_pos, ws)
            out = torch.zeros(wl.L, wl.B, wl.Hq, D, dtype=torch.float32, device="cuda")
            lse = torch.zeros(wl.L, wl.B, wl.Hq, dtype=torch.float32, device="cuda")
            ngc.ngc_decode_attn(cache, -1, to_bf16_tensor(q, "cuda"), scale, 0, out, ws, lse_out=lse)
            for s in case.segs:
                l, b, h = s
                ok[s] = np.concatenate([ok[s], nk[l, b, h][None]])
                ov[s] = np.concatenate([ov[s], nv[l, b, h][None]])
                opos[s] = np.concatenate([opos[s], np.array([int(case.lens[b]) + step], np.int32)])
            if t % 11 == 0 or t >= delta - w_:
                got = out.cpu().numpy()
                for s in case.segs:
                    l, b, h = s
                    want = orc.decode_attn(q[l, b, h * G:(h + 1) * G], ok[s], ov[s], scale)
                    assert np.abs(got[l, b, h * G:(h + 1) * G] - want).max() <= 2e-3, (rnd, t, s)
            if t >= delta - w_:
                recent_q.append(q)
                recent_lse.append(lse)
            step += 1
        # ---- score with the last w queries, normalisers from decode --------------------------------------
        q_recent = np.stack(recent_q, axis=2)                                        # [L, B, w, Hq, D]
        lse_recent = torch.stack(recent_lse, dim=2).contiguous()
        scores = torch.zeros(wl.L, wl.B, wl.Hkv, cap, dtype=torch.float32, device="cuda")
        print(f"[cycle] round {rnd}: score (pooled, block {block}), evict", flush=True)
        ngc.ngc_score_keys(cache, -1, to_bf16_tensor(q_recent, "cuda"), w_, scale, ngc.SCORE_POOL_HEADS, block, scores, ws,
                           lse_recent=lse_recent)
        torch.cuda.synchronize()
        gs = scores.cpu().numpy()
        oscores = np.zeros((wl.L, wl.B, wl.Hkv, cap), np.float32)
        items, keep_h = {}, np.zeros((wl.L, wl.B, wl.Hkv), np.int32)
        for l in range(wl.L):
            for b in range(wl.B):
                per_head = [orc.block_means(orc.score_keys(q_recent[l, b, :, h * G:(h + 1) * G], ok[(l, b, h)], scale, True),
                                            block) for h in range(wl.Hkv)]
                pooled = np.mean(per_head, axis=0).astype(np.float32)
                N = pooled.size
                oscores[l, b, :, :N] = pooled
                items[(l, b)] = N
                keep_h[l, b, :] = max(1, (N + 1) // 2)
                for h in range(wl.Hkv):
                    assert np.all(np.abs(gs[l, b, h, :N] - pooled) <= 2e-4 * np.abs(pooled) + 1e-9), (rnd, l, b, h)
        # ---- evict on the oracle's scores -----------------------------------------------------------------
        max_keep = int(keep_h.max())
        kept = torch.full((wl.L, wl.B, wl.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
        sigma = torch.full_like(kept, -1)
        logp = torch.zeros(wl.L, wl.B, wl.Hkv, dtype=torch.float32, device="cuda")
        p = ngc.make_params(block=block, share_heads=1, noise_scale=1.0, round=rnd, seed=wl.gumbel_seed)
        ngc.ngc_evict(cache, -1, torch.from_numpy(oscores).cuda(), torch.from_numpy(keep_h).cuda(), p, max_keep,
                      kept, sigma, logp, ws)
        torch.cuda.synchronize()
        assert all(x == 0 for x in ngc.read_status(ws))
        hk, hv = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v)
        hkept, hsig, hlp = kept.cpu().numpy(), sigma.cpu().numpy(), logp.cpu().numpy()
        hlen, hpos = cache.len.cpu().numpy(), cache.pos.cpu().numpy()
        for s in case.segs:
            l, b, h = s
            N, K = items[(l, b)], int(keep_h[l, b, h])
            okept, osig = orc.evict_select(oscores[l, b, h, :N], K, 1.0, wl.gumbel_seed, rnd, l, b, 0xFFFF)
            assert hkept[l, b, h, :K].tolist() == okept.tolist() and hsig[l, b, h, :K].tolist() == osig.tolist(), (rnd, s)
            want_lp = orc.logprob_literal(oscores[l, b, h, :N], osig)
            assert hlp[l, b, h] == pytest.approx(want_lp, rel=1e-4, abs=1e-5), (rnd, s)
            ok[s] = orc.compact_rows(ok[s], okept, block)
            ov[s] = orc.compact_rows(ov[s], okept, block)
            opos[s] = orc.compact_i32(opos[s], okept, block)
            n = ok[s].shape[0]
            assert hlen[l, b, h] == n, (rnd, s)
            assert hk[l, b, h, :n].tobytes() == ok[s].tobytes() and hv[l, b, h, :n].tobytes() == ov[s].tobytes(), (rnd, s)
            assert hpos[l, b, h, :n].tolist() == opos[s].tolist(), (rnd, s)


def test_three_rounds_over_the_paged_layout():
    """The same cycle with pages as blocks: paged append (ordered grants), paged decode (with log-sum-exp),
    paged scoring (one score per page, pooled over heads), paged eviction (table edit + ordered release) on
    the oracle's scores; tables, stack, lengths and rows equal to the oracle's model after every round."""
    import torch
    from paper_2604_18002_amd import binding as ngc
    from test_gpu_paged import (build_model, upload_model, assert_same_state, device_rows, _segs, _sid)
    P, D, delta, w_, rounds = 32, 128, 70, 5, 3
    wl = synth.workload(1, L=2, B=2, Hkv=2, Hq=6, D=D, n_lo=200, n_hi=520)
    case = host_case(wl)
    max_pages = (wl.cap + delta) // P + 3
    cap = max_pages * P
    nseg = wl.L * wl.B * wl.Hkv
    m = build_model(case, P, max_pages, nseg * max_pages // 2 + 8, seed=77)      # a pool that needs the evicted pages back
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    scale = 1.0 / np.sqrt(D)
    G = wl.G
    step = 0
    for rnd in range(rounds):
        recent_q, recent_lse = [], []
        for t in range(delta):
            nk = np.stack([synth.new_token_kv(wl, l, step)[0] for l in range(wl.L)])
            nv = np.stack([synth.new_token_kv(wl, l, step)[1] for l in range(wl.L)])
            q = np.stack([synth.queries(wl, l, 900 + step) for l in range(wl.L)])
            ngc.ngc_paged_append(pc, -1, to_bf16_tensor(nk, "cuda"), to_bf16_tensor(nv, "cuda"), None, ws)
            skipped = m.append([_sid(wl, s) for s in _segs(wl)], [nk[s[0], s[1], s[2]] for s in _segs(wl)],
                               [nv[s[0], s[1], s[2]] for s in _segs(wl)])
            assert skipped == []
            out = torch.zeros(wl.L, wl.B, wl.Hq, D, dtype=torch.float32, device="cuda")
            lse = torch.zeros(wl.L, wl.B, wl.Hq, dtype=torch.float32, device="cuda")
            ngc.ngc_paged_decode_attn(pc, -1, to_bf16_tensor(q, "cuda"), scale, 0, out, ws, lse_out=lse)
            if t % 23 == 0 or t == delta - 1:
                got = out.cpu().numpy()
                for s in _segs(wl):
                    l, b, h = s
                    k, v = m.rows(_sid(wl, s))
                    want = orc.decode_attn(q[l, b, h * G:(h + 1) * G], k, v, scale)
                    assert np.abs(got[l, b, h * G:(h + 1) * G] - want).max() <= 2e-3, (rnd, t, s)
            if t >= delta - w_:
                recent_q.append(q)
                recent_lse.append(lse)
            step += 1
        assert_same_state(pc, m, wl, f"grown, round {rnd}")
        q_recent = np.stack(recent_q, axis=2)
        lse_recent = torch.stack(recent_lse, dim=2).contiguous()
        scores = torch.zeros(wl.L, wl.B, wl.Hkv, cap, dtype=torch.float32, device="cuda")
        print(f"[paged cycle] round {rnd}: score, evict", flush=True)
        ngc.ngc_paged_score_keys(pc, -1, to_bf16_tensor(q_recent, "cuda"), w_, scale, ngc.SCORE_POOL_HEADS, P, scores, ws,
                                 lse_recent=lse_recent)
        torch.cuda.synchronize()
        gs = scores.cpu().numpy()
        oscores = np.zeros((wl.L, wl.B, wl.Hkv, cap), np.float32)
        keep_h = np.zeros((wl.L, wl.B, wl.Hkv), np.int32)
        for l in range(wl.L):
            for b in range(wl.B):
                per_head = [orc.block_means(orc.score_keys(q_recent[l, b, :, h * G:(h + 1) * G],
                                                           m.rows(_sid(wl, (l, b, h)))[0], scale, True), P)
                            for h in range(wl.Hkv)]
                pooled = np.mean(per_head, axis=0).astype(np.float32)
                N = pooled.size
                oscores[l, b, :, :N] = pooled
                keep_h[l, b, :] = max(1, N // 2)
                for h in range(wl.Hkv):
                    assert np.all(np.abs(gs[l, b, h, :N] - pooled) <= 2e-4 * np.abs(pooled) + 1e-9), (rnd, l, b, h)
        max_keep = int(keep_h.max())
        kept = torch.full((nseg, max_keep), -1, dtype=torch.int32, device="cuda")
        sigma = torch.full_like(kept, -1)
        logp = torch.zeros(nseg, dtype=torch.float32, device="cuda")
        p = ngc.make_params(block=P, share_heads=1, noise_scale=1.0, round=rnd, seed=wl.gumbel_seed)
        ngc.ngc_paged_evict(pc, -1, torch.from_numpy(oscores).cuda(), cap, torch.from_numpy(keep_h).cuda(), p, max_keep,
                            kept, sigma, logp, ws)
        torch.cuda.synchronize()
        hkept, hsig = kept.cpu().numpy(), sigma.cpu().numpy()
        lists = []
        for s in _segs(wl):
            l, b, h = s
            sid = _sid(wl, s)
            N, K = m.pages_in_use(sid), int(keep_h[l, b, h])
            okept, osig = orc.evict_select(oscores[l, b, h, :N], K, 1.0, wl.gumbel_seed, rnd, l, b, 0xFFFF)
            assert hkept[sid, :K].tolist() == okept.tolist() and hsig[sid, :K].tolist() == osig.tolist(), (rnd, s)
            lists.append(okept.tolist())
        m.evict([_sid(wl, s) for s in _segs(wl)], lists)
        assert_same_state(pc, m, wl, f"evicted, round {rnd}")
        for sid in range(nseg):
            k, v = device_rows(pc, m, sid)
            mk, mv = m.rows(sid)
            assert k.tobytes() == mk.tobytes() and v.tobytes() == mv.tobytes(), (rnd, sid)
    assert all(x == 0 for x in ngc.read_status(ws))
