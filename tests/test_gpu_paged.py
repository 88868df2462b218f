"""GPU parity of the paged layout: page-table eviction, pool grant / release order,
append, decode attention and scoring through the page table, against the oracle's
model of the layout (tables, stack and lengths bit for bit; attention and scores
within the tolerances of the contiguous path)."""
import numpy as np
import pytest

import oracle as orc
from paper_2604_18002_amd import synth
from _harness import from_bf16_tensor, host_case, oracle_logprob, to_bf16_tensor

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3
LOGP_RTOL = 1e-4


def _ngc():
    from paper_2604_18002_amd import binding
    return binding


def _segs(wl):
    return [(l, b, h) for l in range(wl.L) for b in range(wl.B) for h in range(wl.Hkv)]


def _sid(wl, seg):
    l, b, h = seg
    return (l * wl.B + b) * wl.Hkv + h


def build_model(case, P, max_pages, num_pages, seed=0):
    """Oracle model holding the case's rows on pages drawn at random from the pool."""
    wl = case.w
    rng = np.random.default_rng(seed)
    m = orc.PagedCache(wl.L * wl.B * wl.Hkv, P, max_pages, num_pages, wl.D)
    m.free_stack[:] = rng.permutation(num_pages).astype(np.int32)
    for seg in case.segs:
        s = _sid(wl, seg)
        k, v = case.k[seg], case.v[seg]
        n = k.shape[0]
        for p in range((n + P - 1) // P):
            m.free_count -= 1
            page = int(m.free_stack[m.free_count])
            m.table[s, p] = page
            lo, hi = p * P, min((p + 1) * P, n)
            m.k_pool[page, :hi - lo] = k[lo:hi]
            m.v_pool[page, :hi - lo] = v[lo:hi]
            m.pos_pool[page, :hi - lo] = np.arange(lo, hi)
        m.len[s] = n
    return m


def upload_model(m, wl, with_pos=True):
    import torch
    ngc = _ngc()
    pc = ngc.PagedCache.allocate(wl.L, wl.B, wl.Hkv, wl.Hq, wl.D, m.P, m.max_pages, m.num_pages, with_pos=with_pos)
    pc.k_pool.copy_(to_bf16_tensor(m.k_pool, "cuda"))
    pc.v_pool.copy_(to_bf16_tensor(m.v_pool, "cuda"))
    if with_pos:
        pc.pos_pool.copy_(torch.from_numpy(m.pos_pool))
    pc.table.copy_(torch.from_numpy(m.table.reshape(wl.L, wl.B, wl.Hkv, m.max_pages)))
    pc.len.copy_(torch.from_numpy(m.len.reshape(wl.L, wl.B, wl.Hkv)))
    pc.free_stack.copy_(torch.from_numpy(m.free_stack))
    pc.free_count.fill_(int(m.free_count))
    return pc


def assert_same_state(pc, m, wl, what):
    """Tables (entries in use), lengths, free stack and count, and the pools' rows in use."""
    import torch
    torch.cuda.synchronize()
    table = pc.table.cpu().numpy().reshape(-1, m.max_pages)
    ln = pc.len.cpu().numpy().reshape(-1)
    assert ln.tolist() == m.len.tolist(), what
    count = int(pc.free_count.cpu().item())
    assert count == m.free_count, what
    assert pc.free_stack.cpu().numpy()[:count].tolist() == m.free_stack[:count].tolist(), what
    for s in range(m.nseg):
        used = m.pages_in_use(s)
        assert table[s, :used].tolist() == m.table[s, :used].tolist(), (what, s)
    # every page exactly once
    owned = [int(table[s, i]) for s in range(m.nseg) for i in range(m.pages_in_use(s))]
    assert sorted(owned + pc.free_stack.cpu().numpy()[:count].tolist()) == list(range(m.num_pages)), what


def device_rows(pc, m, s):
    """Logical rows of a segment gathered from the device pools through the device table."""
    table = pc.table.cpu().numpy().reshape(-1, m.max_pages)
    n = int(pc.len.cpu().numpy().reshape(-1)[s])
    pages = table[s, :(n + m.P - 1) // m.P]
    k = from_bf16_tensor(pc.k_pool[pages.tolist()]).reshape(-1, m.D)[:n]
    v = from_bf16_tensor(pc.v_pool[pages.tolist()]).reshape(-1, m.D)[:n]
    return k, v


def check_attention(pc, m, wl, ws, layer, salt, lse=False):
    import torch
    ngc = _ngc()
    scale = 1.0 / np.sqrt(wl.D)
    layers = range(wl.L) if layer < 0 else [layer]
    q = np.stack([synth.queries(wl, l, salt) for l in layers])                 # [nl, B, Hq, D]
    out = torch.zeros(len(layers), wl.B, wl.Hq, wl.D, dtype=torch.float32, device="cuda")
    lse_t = torch.zeros(len(layers), wl.B, wl.Hq, dtype=torch.float32, device="cuda") if lse else None
    print(f"[paged attn] layer={layer} salt={salt}", flush=True)
    ngc.ngc_paged_decode_attn(pc, layer, to_bf16_tensor(q if layer < 0 else q[0], "cuda"), scale, 0, out, ws,
                              lse_out=lse_t)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    got_lse = lse_t.cpu().numpy() if lse else None
    worst = 0.0
    for i, l in enumerate(layers):
        for b in range(wl.B):
            for h in range(wl.Hkv):
                k, v = m.rows(_sid(wl, (l, b, h)))
                if k.shape[0] == 0:
                    assert not got[i, b, h * wl.G:(h + 1) * wl.G].any()
                    continue
                want = orc.decode_attn(q[i, b, h * wl.G:(h + 1) * wl.G], k, v, scale)
                worst = max(worst, float(np.abs(got[i, b, h * wl.G:(h + 1) * wl.G] - want).max()))
                if lse:
                    want_lse = orc.decode_lse(q[i, b, h * wl.G:(h + 1) * wl.G], k, scale)
                    assert np.abs(got_lse[i, b, h * wl.G:(h + 1) * wl.G] - want_lse).max() <= 2e-5
    assert worst <= ATTN_TOL, worst


def block_logits(wl, seg, n_items):
    return synth.segment_logits(wl, seg[0], seg[1], seg[2], n_items)


def run_round(pc, m, wl, ws, rnd, keep_of, tau=1.0, layer=-1, share_heads=0, select_only=False):
    """One eviction round on device and on the model; compares the sampled actions."""
    import torch
    ngc = _ngc()
    P = m.P
    segs = [s for s in _segs(wl) if layer < 0 or s[0] == layer]
    logits = np.zeros((m.nseg, m.max_pages), np.float32)
    keep = np.zeros(m.nseg, np.int32)
    for seg in _segs(wl):
        s = _sid(wl, seg)
        N = m.pages_in_use(s)
        logits[s, :N] = block_logits(wl, (seg[0] * 7 + rnd, seg[1], seg[2]), N)
        keep[s] = keep_of(N)
    max_keep = max(1, int(keep.max()))
    kept = torch.full((m.nseg, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1)
    logp = torch.zeros(m.nseg, dtype=torch.float32, device="cuda")
    flags = ngc.EVICT_SELECT_ONLY if select_only else 0
    p = ngc.make_params(block=P, share_heads=share_heads, noise_scale=tau, round=rnd, seed=wl.gumbel_seed, flags=flags)
    print(f"[paged evict] round={rnd} layer={layer} tau={tau} select_only={select_only}", flush=True)
    ngc.ngc_paged_evict(pc, layer, torch.from_numpy(logits).cuda(), m.max_pages, torch.from_numpy(keep).cuda(), p,
                        max_keep, kept, sigma, logp, ws)
    torch.cuda.synchronize()
    hk, hs, hl = kept.cpu().numpy(), sigma.cpu().numpy(), logp.cpu().numpy()
    kept_lists = []
    for seg in segs:
        s = _sid(wl, seg)
        N, K = m.pages_in_use(s), int(min(keep[s], m.pages_in_use(s)))
        hsel = 0xFFFF if share_heads else seg[2]
        okept, osig = orc.evict_select(logits[s, :N], K, tau, wl.gumbel_seed, rnd, seg[0], seg[1], hsel)
        assert hk[s, :K].tolist() == okept.tolist(), seg
        assert hs[s, :K].tolist() == osig.tolist(), seg
        want_lp = oracle_logprob(logits[s, :N], osig)
        assert abs(hl[s] - want_lp) <= LOGP_RTOL * max(1.0, abs(want_lp)), (seg, hl[s], want_lp)
        kept_lists.append(okept.tolist())
    if not select_only:
        m.evict([_sid(wl, seg) for seg in segs], kept_lists)
    return kept_lists


def append_step(pc, m, wl, ws, step, layer=-1):
    import torch
    ngc = _ngc()
    layers = range(wl.L) if layer < 0 else [layer]
    nk = np.stack([synth.new_token_kv(wl, l, step)[0] for l in layers])        # [nl, B, Hkv, D]
    nv = np.stack([synth.new_token_kv(wl, l, step)[1] for l in layers])
    new_pos = torch.full((wl.B,), 100000 + step, dtype=torch.int32, device="cuda")
    ngc.ngc_paged_append(pc, layer, to_bf16_tensor(nk if layer < 0 else nk[0], "cuda"),
                         to_bf16_tensor(nv if layer < 0 else nv[0], "cuda"), new_pos, ws)
    segs = [s for s in _segs(wl) if layer < 0 or s[0] == layer]
    rows_k = [nk[(seg[0] if layer < 0 else 0), seg[1], seg[2]] for seg in segs]
    rows_v = [nv[(seg[0] if layer < 0 else 0), seg[1], seg[2]] for seg in segs]
    return m.append([_sid(wl, seg) for seg in segs], rows_k, rows_v, [100000 + step] * len(segs))


@pytest.mark.parametrize("D,P", [(128, 32), (64, 32), (128, 64), (64, 128)])
def test_attention_through_the_page_table(D, P):
    ngc = _ngc()
    wl = synth.workload(1, L=2, B=3, D=D, n_lo=40, n_hi=1500)
    case = host_case(wl)
    max_pages = (wl.cap + P - 1) // P + 1
    m = build_model(case, P, max_pages, wl.L * wl.B * wl.Hkv * max_pages + 5, seed=D + P)
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    check_attention(pc, m, wl, ws, -1, 1, lse=True)
    check_attention(pc, m, wl, ws, 1, 2)
    assert all(x == 0 for x in ngc.read_status(ws))


def test_long_segments_split_over_workgroups():
    # few segments, many tiles: the split path and its merge, through the table
    ngc = _ngc()
    wl = synth.workload(1, L=1, B=2, n_lo=5000, n_hi=9000)
    case = host_case(wl)
    P = 32
    max_pages = (wl.cap + P - 1) // P
    m = build_model(case, P, max_pages, wl.B * wl.Hkv * max_pages, seed=5)
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    check_attention(pc, m, wl, ws, -1, 3, lse=True)
    check_attention(pc, m, wl, ws, 0, 4)


@pytest.mark.parametrize("P,tau", [(32, 1.0), (64, 1.0), (32, 0.0)])
def test_eviction_edits_tables_and_releases_pages(P, tau):
    ngc = _ngc()
    wl = synth.workload(1, L=2, B=4, n_lo=700, n_hi=2048)
    case = host_case(wl)
    max_pages = wl.cap // P + 2
    m = build_model(case, P, max_pages, wl.L * wl.B * wl.Hkv * max_pages, seed=P)
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    before = [m.rows(s) for s in range(m.nseg)]
    kept = run_round(pc, m, wl, ws, 0, lambda N: (N + 1) // 2, tau=tau)
    assert_same_state(pc, m, wl, "after round 0")
    # nothing moved: the survivors are the same bytes, seen through the new table
    for s in range(m.nseg):
        n0 = before[s][0].shape[0]
        rows = np.concatenate([np.arange(b * P, min((b + 1) * P, n0)) for b in kept[s]])
        k, v = device_rows(pc, m, s)
        assert k.tobytes() == before[s][0][rows].tobytes() and v.tobytes() == before[s][1][rows].tobytes()
    check_attention(pc, m, wl, ws, -1, 7)
    assert all(x == 0 for x in ngc.read_status(ws))


def test_select_only_and_single_layer_rounds():
    ngc = _ngc()
    wl = synth.workload(1, L=3, B=3, n_lo=300, n_hi=900)
    case = host_case(wl)
    P = 32
    max_pages = wl.cap // P + 3
    m = build_model(case, P, max_pages, wl.L * wl.B * wl.Hkv * max_pages, seed=9)
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    run_round(pc, m, wl, ws, 0, lambda N: max(1, N // 3), select_only=True)
    assert_same_state(pc, m, wl, "select only changes nothing")
    run_round(pc, m, wl, ws, 1, lambda N: max(1, N // 3), layer=1)          # only layer 1 evicts
    assert_same_state(pc, m, wl, "layer 1 evicted")
    run_round(pc, m, wl, ws, 2, lambda N: max(1, (2 * N) // 3), share_heads=1)
    assert_same_state(pc, m, wl, "all layers, shared noise")
    check_attention(pc, m, wl, ws, -1, 11)
    assert all(x == 0 for x in ngc.read_status(ws))


def test_grow_then_evict_cycles():
    """Several rounds of (delta appends + attention, eviction): tables, stack order, pool rows,
    positions and attention stay equal to the model's."""
    import torch
    ngc = _ngc()
    wl = synth.workload(1, L=2, B=3, n_lo=100, n_hi=420)
    case = host_case(wl)
    P = 32
    max_pages = 24
    m = build_model(case, P, max_pages, 260, seed=13)
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    step = 0
    for rnd in range(3):
        for _ in range(45):
            skipped = append_step(pc, m, wl, ws, step)
            assert skipped == []
            step += 1
        assert_same_state(pc, m, wl, f"after growth {rnd}")
        check_attention(pc, m, wl, ws, -1, 20 + rnd)
        run_round(pc, m, wl, ws, rnd, lambda N: max(1, (N + 1) // 2))
        assert_same_state(pc, m, wl, f"after round {rnd}")
    # single-layer appends
    for _ in range(3):
        assert append_step(pc, m, wl, ws, step, layer=1) == []
        step += 1
    assert_same_state(pc, m, wl, "after single-layer appends")
    for s in range(m.nseg):
        k, v = device_rows(pc, m, s)
        mk, mv = m.rows(s)
        assert k.tobytes() == mk.tobytes() and v.tobytes() == mv.tobytes(), s
    table = pc.table.cpu().numpy().reshape(-1, m.max_pages)
    pos_pool = pc.pos_pool.cpu().numpy()
    for s in range(m.nseg):
        n = int(m.len[s])
        got = [int(pos_pool[table[s, r // P], r % P]) for r in range(n)]
        assert got == m.positions(s).tolist()
    check_attention(pc, m, wl, ws, -1, 30)
    assert all(x == 0 for x in ngc.read_status(ws))


def test_pool_exhaustion_and_capacity_are_counted_not_fatal():
    ngc = _ngc()
    wl = synth.workload(1, L=1, B=4, n_lo=64, n_hi=64)        # every segment: 2 full pages of 32
    case = host_case(wl)
    P, max_pages = 32, 4
    nseg = wl.B * wl.Hkv
    m = build_model(case, P, max_pages, 2 * nseg + 3, seed=17)  # 3 spare pages for 8 segments
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    skipped = append_step(pc, m, wl, ws, 0)
    assert len(skipped) == nseg - 3                            # the three lowest segments got the spare pages
    st = ngc.read_status(ws)
    assert st[ngc.STATUS_APPEND_FULL] == nseg - 3 and st[ngc.STATUS_POOL_BOUNDS] == 0
    assert_same_state(pc, m, wl, "pool exhausted")
    # free everything of the last segment, then the stalled segments can grow again (lowest first)
    keep_one = [[0]] * (nseg - 1) + [[]]
    import torch
    logits = torch.zeros(nseg, max_pages, dtype=torch.float32, device="cuda")
    logits[:, 0] = 5.0                                         # greedy: page 0 of every segment survives
    keep = torch.tensor([1] * (nseg - 1) + [0], dtype=torch.int32, device="cuda")
    kept = torch.zeros(nseg, 1, dtype=torch.int32, device="cuda")
    ngc.ngc_paged_evict(pc, -1, logits, max_pages, keep, ngc.make_params(block=P, noise_scale=0.0), 1, kept, None,
                        None, ws)
    m.evict(range(nseg), keep_one)
    assert_same_state(pc, m, wl, "after freeing")
    for step in range(1, 3 * P + 5):                           # up to capacity: 4 pages of 32 rows
        append_step(pc, m, wl, ws, step)
    assert_same_state(pc, m, wl, "after refill")
    check_attention(pc, m, wl, ws, -1, 40)


def test_scores_through_the_page_table_feed_the_round():
    import torch
    ngc = _ngc()
    wl = synth.workload(1, L=2, B=3, n_lo=500, n_hi=1300)
    case = host_case(wl)
    P, w_ = 32, 5
    max_pages = wl.cap // P + 2
    cap = max_pages * P
    m = build_model(case, P, max_pages, wl.L * wl.B * wl.Hkv * max_pages, seed=21)
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    scale = 1.0 / np.sqrt(wl.D)
    q = np.stack([np.stack([synth.queries(wl, l, 300 + j) for j in range(w_)], axis=1) for l in range(wl.L)])
    scores = torch.zeros(wl.L, wl.B, wl.Hkv, cap, dtype=torch.float32, device="cuda")
    print("[paged score] per row, then per page", flush=True)
    ngc.ngc_paged_score_keys(pc, -1, to_bf16_tensor(q, "cuda"), w_, scale, 0, 1, scores, ws)
    torch.cuda.synchronize()
    per_row = scores.cpu().numpy()
    ngc.ngc_paged_score_keys(pc, -1, to_bf16_tensor(q, "cuda"), w_, scale, 0, P, scores, ws)
    torch.cuda.synchronize()
    per_page = scores.cpu().numpy()
    for (l, b, h) in _segs(wl):
        k, _ = m.rows(_sid(wl, (l, b, h)))
        psi = orc.score_keys(q[l, b, :, h * wl.G:(h + 1) * wl.G], k, scale, True)
        assert np.all(np.abs(per_row[l, b, h, :psi.size] - psi) <= 2e-3 * np.abs(psi) + 1e-7)
        want = orc.block_means(psi, P)
        assert np.all(np.abs(per_page[l, b, h, :want.size] - want) <= 2e-3 * np.abs(want) + 1e-7)
    # the round takes the scores where the scoring kernel left them (stride = max_pages * P)
    keep = torch.from_numpy(np.array([max(1, m.pages_in_use(s) // 2) for s in range(m.nseg)], np.int32)).cuda()
    max_keep = int(keep.max().item())
    kept = torch.zeros(m.nseg, max_keep, dtype=torch.int32, device="cuda")
    ngc.ngc_paged_evict(pc, -1, scores, cap, keep, ngc.make_params(block=P, noise_scale=0.0), max_keep, kept,
                        None, None, ws)
    torch.cuda.synchronize()
    hk = kept.cpu().numpy()
    flat = per_page.reshape(m.nseg, cap)
    for s in range(m.nseg):
        N, K = m.pages_in_use(s), max(1, m.pages_in_use(s) // 2)
        # greedy top-K of the device's own scores, by a library sort (ties by index)
        order = np.argsort(-flat[s, :N].astype(np.float64), kind="stable")[:K]
        assert hk[s, :K].tolist() == sorted(order.tolist())
    assert all(x == 0 for x in ngc.read_status(ws))


def test_identity_table_gives_the_contiguous_result_bit_for_bit():
    """A contiguous cache is a paged one whose table counts 0, 1, 2, ...: both entry points must
    then return the same bits (same tiles, same order of operations)."""
    import torch
    ngc = _ngc()
    wl = synth.workload(1, L=2, B=5, n_lo=200, n_hi=2048)
    case = host_case(wl)
    from _harness import upload
    cache, _, _ = upload(case)
    P = 64
    mp = wl.cap // P
    nseg = wl.L * wl.B * wl.Hkv
    table = (torch.arange(nseg, dtype=torch.int32, device="cuda")[:, None] * mp +
             torch.arange(mp, dtype=torch.int32, device="cuda")[None]).view(wl.L, wl.B, wl.Hkv, mp).contiguous()
    pc = ngc.PagedCache(cache.k.view(nseg * mp, P, wl.D), cache.v.view(nseg * mp, P, wl.D), None, table, cache.len,
                        torch.zeros(nseg * mp, dtype=torch.int32, device="cuda"),
                        torch.zeros(1, dtype=torch.int32, device="cuda"), wl.Hq)
    ws = ngc.allocate_workspace(cache, 1)
    q = np.stack([synth.queries(wl, l, 77) for l in range(wl.L)])
    a = torch.zeros(wl.L, wl.B, wl.Hq, wl.D, dtype=torch.float32, device="cuda")
    b = torch.zeros_like(a)
    la = torch.zeros(wl.L, wl.B, wl.Hq, dtype=torch.float32, device="cuda")
    lb = torch.zeros_like(la)
    scale = 1.0 / np.sqrt(wl.D)
    for hint in (0, 300):                        # two different splits of the work
        ngc.ngc_decode_attn(cache, -1, to_bf16_tensor(q, "cuda"), scale, hint, a, ws, lse_out=la)
        ngc.ngc_paged_decode_attn(pc, -1, to_bf16_tensor(q, "cuda"), scale, hint, b, ws, lse_out=lb)
        torch.cuda.synchronize()
        assert torch.equal(a, b) and torch.equal(la, lb)


def test_full_size_paged_sampled_segments():
    """Config 2 at full size in the launch configuration bench.py times (pages of 32 rows, all layers per
    launch): pools filled on the device, a sample of segments generated on the host; round 0, one append,
    decode attention; sampled segments against the oracle, pool accounting everywhere."""
    import torch
    ngc = _ngc()
    w = synth.workload(2)
    P = 32
    rng = np.random.default_rng(202)
    segs = {(0, 0, 0), (w.L - 1, w.B - 1, w.Hkv - 1)}
    while len(segs) < 20:
        segs.add((int(rng.integers(w.L)), int(rng.integers(w.B)), int(rng.integers(w.Hkv))))
    segs = sorted(segs)
    case = host_case(w, segs)
    nseg = w.L * w.B * w.Hkv
    max_pages = w.cap // P + 1
    n_pg = np.broadcast_to(((case.lens + P - 1) // P)[None, :, None], (w.L, w.B, w.Hkv)).reshape(-1).astype(np.int64)
    keep_pg = ((n_pg + 2) // 3).astype(np.int32)
    spare = nseg * 2
    num_pages = int(n_pg.sum()) + spare
    print(f"[full paged] pool {2 * num_pages * P * w.D * 2 / 1e9:.1f} GB, {nseg} segments", flush=True)
    pc = ngc.PagedCache.allocate(w.L, w.B, w.Hkv, w.Hq, w.D, P, max_pages, num_pages)
    synth.fill_normal_bf16_(pc.k_pool, 1)
    synth.fill_normal_bf16_(pc.v_pool, 2)
    # segment s owns pages perm[first_s ...]: scattered over the pool
    perm = np.random.default_rng(7).permutation(num_pages).astype(np.int32)
    first = np.concatenate([[0], np.cumsum(n_pg)[:-1]])
    table_h = np.full((nseg, max_pages), -1, np.int32)
    for s in range(nseg):
        table_h[s, :n_pg[s]] = perm[first[s]:first[s] + n_pg[s]]
    stack_h = perm[int(n_pg.sum()):].copy()
    pc.table.copy_(torch.from_numpy(table_h.reshape(w.L, w.B, w.Hkv, max_pages)))
    pc.free_stack[:spare].copy_(torch.from_numpy(stack_h))
    pc.free_count.fill_(spare)
    pc.len.copy_(torch.from_numpy(np.broadcast_to(case.lens[None, :, None], (w.L, w.B, w.Hkv)).copy()))
    logits = torch.randn(nseg, max_pages, device="cuda")
    host_logits = {}
    for seg in segs:
        s = _sid(w, seg)
        n = case.k[seg].shape[0]
        kk = np.zeros((n_pg[s] * P, w.D), np.uint16)
        vv = np.zeros_like(kk)
        kk[:n], vv[:n] = case.k[seg], case.v[seg]
        idx = torch.from_numpy(table_h[s, :n_pg[s]].astype(np.int64)).cuda()
        pc.k_pool[idx] = to_bf16_tensor(kk.reshape(-1, P, w.D), "cuda")
        pc.v_pool[idx] = to_bf16_tensor(vv.reshape(-1, P, w.D), "cuda")
        host_logits[seg] = synth.segment_logits(w, seg[0], seg[1], seg[2], int(n_pg[s]))
        logits[s, :n_pg[s]] = torch.from_numpy(host_logits[seg]).cuda()
    keep = torch.from_numpy(keep_pg).cuda()
    max_keep = int(keep_pg.max())
    kept = torch.empty(nseg, max_keep, dtype=torch.int32, device="cuda")
    sigma = torch.empty_like(kept)
    logp = torch.empty(nseg, dtype=torch.float32, device="cuda")
    ws = ngc.allocate_paged_workspace(pc)
    print("[full paged] evict, all layers", flush=True)
    ngc.ngc_paged_evict(pc, -1, logits, max_pages, keep, ngc.make_params(block=P, noise_scale=1.0, round=0,
                                                                        seed=w.gumbel_seed),
                        max_keep, kept, sigma, logp, ws)
    torch.cuda.synchronize()
    g = torch.Generator(device="cuda")
    g.manual_seed(4)
    k_new = torch.randn(w.L, w.B, w.Hkv, w.D, generator=g, device="cuda").to(torch.bfloat16)
    v_new = torch.randn(w.L, w.B, w.Hkv, w.D, generator=g, device="cuda").to(torch.bfloat16)
    q = torch.randn(w.L, w.B, w.Hq, w.D, generator=g, device="cuda").to(torch.bfloat16)
    out = torch.empty(w.L, w.B, w.Hq, w.D, dtype=torch.float32, device="cuda")
    print("[full paged] append + decode attention, all layers", flush=True)
    ngc.ngc_paged_append(pc, -1, k_new, v_new, None, ws)
    scale = 1.0 / np.sqrt(w.D)
    ngc.ngc_paged_decode_attn(pc, -1, q, scale, int(keep_pg.max()) * P + w.delta, out, ws)
    torch.cuda.synchronize()
    assert all(x == 0 for x in ngc.read_status(ws))

    def bits(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

    # pool accounting everywhere (inputs only: page counts and keep counts)
    freed = n_pg - keep_pg
    push_at = spare + np.concatenate([[0], np.cumsum(freed)[:-1]])
    table_d = pc.table.cpu().numpy().reshape(nseg, max_pages)
    len_d = pc.len.cpu().numpy().reshape(-1)
    stack_d = pc.free_stack.cpu().numpy()
    count_d = int(pc.free_count.item())
    # after the round every segment has K full pages (4096 rows = 128 full pages, so no short page), and the
    # append that follows takes one page per segment from the top of the stack, lowest segment first
    assert len_d.tolist() == (keep_pg * P + 1).tolist()
    total_after_round = spare + int(freed.sum())
    assert count_d == total_after_round - nseg
    for seg in segs:
        s = _sid(w, seg)
        N, K = int(n_pg[s]), int(keep_pg[s])
        okept, osig = orc.evict_select(host_logits[seg], K, 1.0, w.gumbel_seed, 0, seg[0], seg[1], seg[2])
        assert kept[s, :K].cpu().numpy().tolist() == okept.tolist(), seg
        assert sigma[s, :K].cpu().numpy().tolist() == osig.tolist(), seg
        want_lp = oracle_logprob(host_logits[seg], osig)
        assert float(logp[s]) == pytest.approx(want_lp, rel=LOGP_RTOL), seg
        gone = [t for t in range(N) if t not in set(okept.tolist())]
        assert table_d[s, :K].tolist() == table_h[s, okept].tolist(), seg
        # released pages sit on the stack where the segment order puts them, unless a later grant took them
        for r, t in enumerate(gone):
            at = int(push_at[s]) + r
            if at < count_d:
                assert stack_d[at] == table_h[s, t], (seg, r)
        # the page granted for the appended row (its id depends on every segment's sample: checked to be valid
        # here, exactly in the small cases)
        page = int(table_d[s, K])
        assert 0 <= page < num_pages
        rows = np.concatenate([np.arange(b * P, (b + 1) * P) for b in okept])
        kk = np.concatenate([case.k[seg][rows], bits(k_new[seg[0], seg[1], seg[2]])[None]])
        vv = np.concatenate([case.v[seg][rows], bits(v_new[seg[0], seg[1], seg[2]])[None]])
        # the appended row really is in the granted page
        assert bits(pc.k_pool[page, 0]).tobytes() == kk[-1].tobytes()
        want = orc.decode_attn(bits(q[seg[0], seg[1], seg[2] * w.G:(seg[2] + 1) * w.G]), kk, vv, scale)
        got = out[seg[0], seg[1], seg[2] * w.G:(seg[2] + 1) * w.G].cpu().numpy()
        assert np.abs(got - want).max() <= ATTN_TOL, (seg, np.abs(got - want).max())
    # every page exactly once, at any size
    used = torch.from_numpy(np.concatenate([table_d[s, :keep_pg[s] + 1] for s in range(nseg)])).cuda()
    everything = torch.cat([used, pc.free_stack[:count_d]]).sort().values
    assert torch.equal(everything, torch.arange(num_pages, dtype=torch.int32, device="cuda"))
    assert bool(torch.isfinite(out).all())


def test_degenerate_segments_and_rounds():
    """Empty, one-row, exactly-one-page and completely full segments; rounds that keep everything, nothing, or
    ask for more than there is (clamped and counted); appends into empty and into full segments."""
    import torch
    ngc = _ngc()
    P, max_pages, D = 32, 4, 64
    wl = synth.workload(0, L=1, B=4, D=D, n_lo=1, n_hi=1)             # shapes only: Hq 8, Hkv 2
    nseg = wl.B * wl.Hkv
    lens = [0, 1, P, P * max_pages, P + 5, 0, 2 * P, 3 * P - 1]
    rng = np.random.default_rng(31)
    m = orc.PagedCache(nseg, P, max_pages, 40, D)
    m.free_stack[:] = rng.permutation(40).astype(np.int32)
    for s, n in enumerate(lens):
        for p in range((n + P - 1) // P):
            m.free_count -= 1
            m.table[s, p] = m.free_stack[m.free_count]
            rows = min(P, n - p * P)
            m.k_pool[m.table[s, p], :rows] = synth.f32_to_bf16_bits(rng.standard_normal((rows, D), dtype=np.float32))
            m.v_pool[m.table[s, p], :rows] = synth.f32_to_bf16_bits(rng.standard_normal((rows, D), dtype=np.float32))
        m.len[s] = n
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    check_attention(pc, m, wl, ws, -1, 1, lse=False)                    # two empty segments: zeros, counted
    st = ngc.read_status(ws)
    assert st[ngc.STATUS_EMPTY_ATTN] == 2

    def round_with(keep_list, rnd):
        logits = torch.from_numpy(rng.standard_normal((nseg, max_pages)).astype(np.float32)).cuda()
        keep = torch.tensor(keep_list, dtype=torch.int32, device="cuda")
        max_keep = max(1, max(keep_list))
        kept = torch.full((nseg, max_keep), -1, dtype=torch.int32, device="cuda")
        sigma = torch.full_like(kept, -1)
        logp = torch.full((nseg,), 7.0, dtype=torch.float32, device="cuda")
        ngc.ngc_paged_evict(pc, -1, logits, max_pages, keep, ngc.make_params(block=P, noise_scale=1.0, round=rnd, seed=5),
                            max_keep, kept, sigma, logp, ws)
        torch.cuda.synchronize()
        hl, hk, hs, hp = logits.cpu().numpy(), kept.cpu().numpy(), sigma.cpu().numpy(), logp.cpu().numpy()
        lists = []
        for s in range(nseg):
            N = m.pages_in_use(s)
            K = max(0, min(keep_list[s], N))
            b, h = divmod(s, wl.Hkv)
            okept, osig = orc.evict_select(hl[s, :N], K, 1.0, 5, rnd, 0, b, h)
            assert hk[s, :K].tolist() == okept.tolist() and hs[s, :K].tolist() == osig.tolist(), s
            want = oracle_logprob(hl[s, :N], osig) if K else 0.0
            assert abs(hp[s] - want) <= LOGP_RTOL * max(1.0, abs(want)), s
            lists.append(okept.tolist())
        m.evict(range(nseg), lists)
        assert_same_state(pc, m, wl, f"round {rnd}")

    before = ngc.read_status(ws)[ngc.STATUS_KEEP_CLAMPED]
    round_with([m.pages_in_use(s) for s in range(nseg)], 0)            # keep everything: nothing changes
    assert ngc.read_status(ws)[ngc.STATUS_KEEP_CLAMPED] == before
    round_with([m.pages_in_use(s) + 3 for s in range(nseg)], 1)        # more than there is: clamped, counted
    assert ngc.read_status(ws)[ngc.STATUS_KEEP_CLAMPED] == before + nseg
    assert append_step(pc, m, wl, ws, 0) == [3]                        # the full segment cannot grow
    assert_same_state(pc, m, wl, "append into empty and full segments")
    round_with([1, 0, 1, 2, 1, 1, 0, 2], 2)                            # some segments evict everything
    check_attention(pc, m, wl, ws, -1, 2)
    for step in range(1, 4):
        append_step(pc, m, wl, ws, step)
    assert_same_state(pc, m, wl, "regrowth")
    check_attention(pc, m, wl, ws, 0, 3)


def test_large_pages():
    # pages of 256 rows (8 tiles per page), D = 64
    ngc = _ngc()
    wl = synth.workload(1, L=1, B=3, D=64, n_lo=300, n_hi=2000)
    case = host_case(wl)
    P = 256
    max_pages = wl.cap // P + 2
    m = build_model(case, P, max_pages, wl.B * wl.Hkv * max_pages, seed=41)
    pc = upload_model(m, wl)
    ws = ngc.allocate_paged_workspace(pc)
    check_attention(pc, m, wl, ws, -1, 1, lse=True)
    run_round(pc, m, wl, ws, 0, lambda N: max(1, N - 2))
    assert_same_state(pc, m, wl, "large pages, round 0")
    for step in range(3):
        assert append_step(pc, m, wl, ws, step) == []
    assert_same_state(pc, m, wl, "large pages, appends")
    check_attention(pc, m, wl, ws, -1, 2)
    assert all(x == 0 for x in ngc.read_status(ws))
