"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation), so its
calls can be captured in a HIP graph.  Replays are checked against eager runs several times, with
eager work between the replays."""
import numpy as np
import pytest

from paper_2604_18002_amd import synth

from _harness import host_case, to_bf16_tensor, upload

pytestmark = pytest.mark.gpu


def test_decode_step_and_eviction_round_under_graph_capture():
    import torch
    from paper_2604_18002_amd import binding as ngc
    ngc.load_library()
    w = synth.workload(3, L=2, B=4, n_lo=5000, n_hi=8192)     # 8192-item segments: the large-LDS eviction path
    case = host_case(w)
    scale = 1.0 / np.sqrt(w.D)
    max_keep = int(case.keep.max())
    nk = to_bf16_tensor(np.stack([synth.new_token_kv(w, l, 0)[0] for l in range(w.L)]), "cuda")
    nv = to_bf16_tensor(np.stack([synth.new_token_kv(w, l, 0)[1] for l in range(w.L)]), "cuda")
    q = to_bf16_tensor(np.stack([synth.queries(w, l, 1) for l in range(w.L)]), "cuda")

    def fresh():
        cache, logits, keep = upload(case)
        ws = ngc.allocate_workspace(cache, max_keep)
        kept = torch.zeros(w.L, w.B, w.Hkv, max_keep, dtype=torch.int32, device="cuda")
        sigma = torch.zeros_like(kept)
        logp = torch.zeros(w.L, w.B, w.Hkv, dtype=torch.float32, device="cuda")
        out = torch.zeros(w.L, w.B, w.Hq, w.D, dtype=torch.float32, device="cuda")
        return cache, logits, keep, ws, kept, sigma, logp, out

    def step(st, rnd):
        cache, logits, keep, ws, kept, sigma, logp, out = st
        ngc.ngc_evict(cache, -1, logits, keep, ngc.make_params(noise_scale=1.0, round=rnd, seed=7), max_keep,
                      kept, sigma, logp, ws)
        ngc.ngc_cache_append(cache, -1, nk, nv, None, ws)
        ngc.ngc_decode_attn(cache, -1, q, scale, 0, out, ws)

    # eager reference: evict + append + attend once
    ref = fresh()
    print("[graph] eager reference", flush=True)
    step(ref, 0)
    torch.cuda.synchronize()

    st = fresh()
    lens0, k0, v0 = st[0].len.clone(), st[0].k.clone(), st[0].v.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up outside capture (first-use work of the runtime)
        step(st, 0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    print("[graph] capture", flush=True)
    with torch.cuda.graph(g):
        step(st, 0)
    for rep in range(3):
        # eager work between replays: restore the cache the captured round starts from, scribble on the outputs
        st[0].len.copy_(lens0)
        st[0].k.copy_(k0)
        st[0].v.copy_(v0)
        st[7].fill_(float("nan"))
        st[4].fill_(-1)
        torch.cuda.synchronize()
        print(f"[graph] replay {rep}", flush=True)
        g.replay()
        torch.cuda.synchronize()
        valid = torch.arange(max_keep, device="cuda") < st[2].unsqueeze(-1)      # entries past K are unspecified
        assert torch.equal(st[4][valid], ref[4][valid]), f"kept differs on replay {rep}"
        assert torch.equal(st[5][valid], ref[5][valid]), f"sigma differs on replay {rep}"
        assert torch.equal(st[6], ref[6]), f"logp differs on replay {rep}"
        assert torch.equal(st[0].len, ref[0].len)
        assert torch.equal(st[7], ref[7]), f"attention output differs on replay {rep}"
    assert all(x == 0 for x in ngc.read_status(st[3]))


def test_paged_round_and_step_under_graph_capture():
    """Paged layout: round (selection, table edit, ordered release) + append (ordered grant) + decode
    attention captured once; every replay must rebuild exactly the eager tables, stack and outputs."""
    import torch
    from paper_2604_18002_amd import binding as ngc
    from test_gpu_paged import build_model, upload_model
    ngc.load_library()
    w = synth.workload(1, L=2, B=4, n_lo=600, n_hi=1600)
    case = host_case(w)
    P = 32
    max_pages = w.cap // P + 2
    nseg = w.L * w.B * w.Hkv
    model = build_model(case, P, max_pages, nseg * max_pages, seed=3)
    scale = 1.0 / np.sqrt(w.D)
    nk = to_bf16_tensor(np.stack([synth.new_token_kv(w, l, 0)[0] for l in range(w.L)]), "cuda")
    nv = to_bf16_tensor(np.stack([synth.new_token_kv(w, l, 0)[1] for l in range(w.L)]), "cuda")
    q = to_bf16_tensor(np.stack([synth.queries(w, l, 1) for l in range(w.L)]), "cuda")
    keep_h = np.array([max(1, model.pages_in_use(s) // 2) for s in range(nseg)], np.int32)
    max_keep = int(keep_h.max())
    g0 = torch.Generator(device="cuda")
    g0.manual_seed(11)
    logits = torch.randn(nseg, max_pages, generator=g0, device="cuda")
    keep = torch.from_numpy(keep_h).cuda()

    def fresh():
        pc = upload_model(model, w, with_pos=False)
        ws = ngc.allocate_paged_workspace(pc)
        kept = torch.zeros(nseg, max_keep, dtype=torch.int32, device="cuda")
        sigma = torch.zeros_like(kept)
        logp = torch.zeros(nseg, dtype=torch.float32, device="cuda")
        out = torch.zeros(w.L, w.B, w.Hq, w.D, dtype=torch.float32, device="cuda")
        return pc, ws, kept, sigma, logp, out

    def step(st):
        pc, ws, kept, sigma, logp, out = st
        ngc.ngc_paged_evict(pc, -1, logits, max_pages, keep, ngc.make_params(block=P, noise_scale=1.0, round=0, seed=7),
                            max_keep, kept, sigma, logp, ws)
        ngc.ngc_paged_append(pc, -1, nk, nv, None, ws)
        ngc.ngc_paged_decode_attn(pc, -1, q, scale, 0, out, ws)

    ref = fresh()
    print("[paged graph] eager reference", flush=True)
    step(ref)
    torch.cuda.synchronize()

    st = fresh()
    pc = st[0]
    saved = [t.clone() for t in (pc.table, pc.len, pc.free_stack, pc.free_count, pc.k_pool, pc.v_pool)]

    def restore():
        for dst, src in zip((pc.table, pc.len, pc.free_stack, pc.free_count, pc.k_pool, pc.v_pool), saved):
            dst.copy_(src)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(st)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    restore()
    torch.cuda.synchronize()
    gph = torch.cuda.CUDAGraph()
    print("[paged graph] capture", flush=True)
    with torch.cuda.graph(gph):
        step(st)
    used = torch.from_numpy(np.array([[i <= keep_h[s] for i in range(max_pages)] for s in range(nseg)])).cuda()
    used = used.view(w.L, w.B, w.Hkv, max_pages)          # K kept pages + the page the append was granted
    for rep in range(3):
        restore()
        st[5].fill_(float("nan"))
        st[2].fill_(-1)
        torch.cuda.synchronize()
        print(f"[paged graph] replay {rep}", flush=True)
        gph.replay()
        torch.cuda.synchronize()
        valid = torch.arange(max_keep, device="cuda") < keep.unsqueeze(-1)
        assert torch.equal(st[2][valid], ref[2][valid]) and torch.equal(st[3][valid], ref[3][valid])
        assert torch.equal(st[4], ref[4])
        assert torch.equal(pc.len, ref[0].len) and torch.equal(pc.free_count, ref[0].free_count)
        n_free = int(pc.free_count.item())
        assert torch.equal(pc.free_stack[:n_free], ref[0].free_stack[:n_free])
        assert torch.equal(pc.table[used], ref[0].table[used])
        assert torch.equal(st[5], ref[5]), f"attention output differs on replay {rep}"
    assert all(x == 0 for x in ngc.read_status(st[1]))
