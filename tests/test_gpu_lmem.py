"""Eq. 4 on the GPU: the eviction loss, the advantages, and the weights the loss puts on every round's
log-probability; then the whole chain sample -> log-prob -> loss -> gradient of the logits."""
import numpy as np
import pytest

import oracle as orc

pytestmark = pytest.mark.gpu


def _ngc():
    from paper_2604_18002_amd import binding
    return binding


@pytest.mark.parametrize("R,L,B,H,G", [(1, 1, 2, 1, 2), (6, 28, 32, 2, 16), (9, 3, 48, 4, 8), (3, 2, 8192, 1, 16)])
def test_loss_advantages_and_weights(R, L, B, H, G):
    import torch
    ngc = _ngc()
    rng = np.random.default_rng(R * 1000 + B)
    logp = (-5000.0 * rng.random((R, L, B, H))).astype(np.float32)
    rounds = rng.integers(0, R + 1, size=B).astype(np.int32)
    rounds[0] = 0
    rounds[-1] = R
    reward = rng.integers(0, 2, size=B).astype(np.float32)
    d = lambda x: torch.from_numpy(x).cuda()
    adv = torch.zeros(B, dtype=torch.float32, device="cuda")
    per_layer = torch.zeros(L, dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    gout = torch.full((R, L, B, H), 7.0, dtype=torch.float32, device="cuda")
    print(f"[lmem] R={R} L={L} B={B} H={H} G={G}", flush=True)
    ngc.ngc_lmem(d(logp), d(rounds), d(reward), R, L, B, H, G, adv, per_layer, loss, gout)
    torch.cuda.synchronize()
    want_layers, want = orc.lmem(logp, rounds, reward, G)
    oadv = orc.advantages(reward, G)
    assert np.abs(adv.cpu().numpy() - oadv).max() <= 1e-7
    # fp32 inputs, fp64 accumulation: the error is the rounding of the per-rollout weight (2^-24 relative per term)
    w = np.where(np.arange(R)[:, None] < rounds[None, :], 1.0 / np.maximum(rounds, 1)[None, :], 0.0)
    scale = (np.abs(logp.astype(np.float64)) * w[:, None, :, None] * np.abs(oadv)[None, None, :, None]).sum(axis=(0, 2, 3)) / B
    assert np.all(np.abs(per_layer.cpu().numpy() - want_layers) <= 2e-7 * scale + 1e-30)
    assert abs(float(loss) - want) <= 2e-7 * scale.sum() + 1e-30
    want_g = -(w[:, None, :, None] * oadv[None, None, :, None]) / B * np.ones((R, L, B, H))
    got_g = gout.cpu().numpy()
    assert np.all(np.abs(got_g - want_g) <= 3e-7 * np.abs(want_g))
    # determinism: the same call again gives the same bits
    per_layer2 = torch.zeros_like(per_layer)
    loss2 = torch.zeros_like(loss)
    ngc.ngc_lmem(d(logp), d(rounds), d(reward), R, L, B, H, G, None, per_layer2, loss2, None)
    torch.cuda.synchronize()
    assert torch.equal(per_layer, per_layer2) and torch.equal(loss, loss2)
    with pytest.raises(ngc.NgcError):
        ngc.ngc_lmem(d(logp), d(rounds), d(reward), R, L, B, H, B + 1 if B > 2 else 3, None, per_layer2, loss2, None)


def test_chain_sample_logprob_loss_gradient():
    """Two rounds of selection (no rows moved) over fixed logits -> their log-probabilities -> Eq. 4 ->
    d loss / d logits through ngc_subset_logprob_backward, against the oracle's chain."""
    import torch
    from paper_2604_18002_amd import synth
    from _harness import host_case, upload, oracle_logprob
    ngc = _ngc()
    wl = synth.workload(1, L=2, B=4, n_lo=300, n_hi=700)
    case = host_case(wl)
    cache, logits, keep = upload(case)
    R, G = 2, 2
    nseg = wl.L * wl.B * wl.Hkv
    max_keep = int(case.keep.max())
    ws = ngc.allocate_workspace(cache, max_keep)
    logp = torch.zeros(R, wl.L, wl.B, wl.Hkv, dtype=torch.float32, device="cuda")
    sigmas = [torch.zeros(wl.L, wl.B, wl.Hkv, max_keep, dtype=torch.int32, device="cuda") for _ in range(R)]
    kept = torch.zeros(wl.L, wl.B, wl.Hkv, max_keep, dtype=torch.int32, device="cuda")
    for t in range(R):
        p = ngc.make_params(noise_scale=1.0, round=t, seed=wl.gumbel_seed, flags=ngc.EVICT_SELECT_ONLY)
        ngc.ngc_evict(cache, -1, logits, keep, p, max_keep, kept, sigmas[t], logp[t], ws)
    rounds = np.array([2, 1, 2, 0], np.int32)
    reward = np.array([1, 0, 0, 1], np.float32)
    per_layer = torch.zeros(wl.L, dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    gout = torch.zeros_like(logp)
    ngc.ngc_lmem(logp, torch.from_numpy(rounds).cuda(), torch.from_numpy(reward).cuda(), R, wl.L, wl.B, wl.Hkv, G,
                 None, per_layer, loss, gout)
    n_items = cache.len.reshape(-1).contiguous()
    grads = [torch.zeros_like(logits) for _ in range(R)]
    for t in range(R):
        ngc.ngc_subset_logprob_backward(logits, n_items, sigmas[t], keep.reshape(-1), nseg, wl.cap, max_keep, max_keep,
                                        gout[t].reshape(-1), grads[t], ws)
    torch.cuda.synchronize()
    total_grad = sum(g.cpu().numpy().astype(np.float64) for g in grads)
    # oracle chain on the same logits
    olp = np.zeros((R, wl.L, wl.B, wl.Hkv))
    osig = {}
    for t in range(R):
        for (l, b, h) in case.segs:
            s = case.logits[(l, b, h)]
            K = int(case.keep[l, b, h])
            _, sg = orc.evict_select(s, K, 1.0, wl.gumbel_seed, t, l, b, h)
            osig[(t, l, b, h)] = sg
            olp[t, l, b, h] = oracle_logprob(s, sg)
    assert np.allclose(logp.cpu().numpy(), olp, rtol=1e-4)
    _, want_loss = orc.lmem(olp, rounds, reward, G)
    assert float(loss) == pytest.approx(want_loss, rel=2e-4)
    adv = orc.advantages(reward, G)
    for (l, b, h) in case.segs:
        s = case.logits[(l, b, h)]
        want = np.zeros(s.size)
        for t in range(int(rounds[b])):
            want += (-adv[b] / (wl.B * rounds[b])) * orc.logprob_grad(s, osig[(t, l, b, h)])
        got = total_grad[l, b, h, :s.size]
        assert np.abs(got - want).max() <= 1e-4 * max(1e-3, np.abs(want).max()), (l, b, h)
