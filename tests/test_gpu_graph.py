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
