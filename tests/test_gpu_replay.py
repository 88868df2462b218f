"""GPU parity of replay attention (Sec. 4.5, Appendix A.3) against the CPU oracle.
Tolerance as for decode attention: 2e-3 max-abs (the kernel's own error is ~1e-5)."""
import numpy as np
import pytest

import oracle as orc
from paper_2604_18002_amd import synth

from _harness import to_bf16_tensor

pytestmark = pytest.mark.gpu

ATOL = 2e-3


def _ngc():
    from paper_2604_18002_amd import binding
    binding.load_library()
    return binding


def _rand_bf16(rng, shape):
    return synth.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def _random_death(rng, T, period, keep_frac, block=1):
    """Periodic rounds keeping a random fraction of the alive tokens (whole blocks if block > 1)."""
    boundaries, decisions, alive = [], [], []
    nxt = 0
    for bnd in range(period, T, period):
        alive += list(range(nxt, bnd))
        nxt = bnd
        if block == 1:
            dec = (rng.random(len(alive)) < keep_frac).astype(np.int32)
        else:
            nb = (len(alive) + block - 1) // block
            dec = np.repeat((rng.random(nb) < keep_frac).astype(np.int32), block)[:len(alive)]
        boundaries.append(bnd)
        decisions.append(dec)
        alive = [t for t, k in zip(alive, dec) if k]
    return orc.replay_death(T, boundaries, decisions)


def _run(q, k, v, death, Hq, Hkv, D, per_head, scale):
    import torch
    ngc = _ngc()
    B, T = q.shape[0], q.shape[1]
    out = torch.full((B, T, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.zeros(ngc.ngc_replay_workspace_bytes(B, T, Hkv), dtype=torch.uint8, device="cuda")
    print(f"[replay] B={B} T={T} Hq={Hq} Hkv={Hkv} D={D} per_head={per_head}", flush=True)
    ngc.ngc_replay_attn(to_bf16_tensor(q, "cuda"), to_bf16_tensor(k, "cuda"), to_bf16_tensor(v, "cuda"),
                        torch.from_numpy(death).cuda(), B, T, Hq, Hkv, D, per_head, scale, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _check(q, k, v, death, Hq, Hkv, D, per_head, scale, got):
    B, T = q.shape[0], q.shape[1]
    G = Hq // Hkv
    for b in range(B):
        for h in range(Hkv):
            d = death[b, h] if per_head else death[b]
            want = orc.replay_attn(q[b, :, h * G:(h + 1) * G], k[b, :, h], v[b, :, h], d, scale)
            diff = np.abs(got[b, :, h * G:(h + 1) * G] - want).max()
            assert diff <= ATOL, (b, h, diff)
    assert np.all(np.isfinite(got))


def test_figure_example():
    rng = np.random.default_rng(60)
    T, Hq, Hkv, D = 10, 4, 2, 64
    q, k, v = _rand_bf16(rng, (1, T, Hq, D)), _rand_bf16(rng, (1, T, Hkv, D)), _rand_bf16(rng, (1, T, Hkv, D))
    death = orc.replay_death(T, [5, 8], [[1, 0, 1, 0, 1], [1, 0, 1, 0, 1, 1]])[None]
    got = _run(q, k, v, death, Hq, Hkv, D, False, 0.125)
    _check(q, k, v, death, Hq, Hkv, D, False, 0.125, got)


@pytest.mark.parametrize("T,Hq,Hkv,D,period,per_head,block", [
    (300, 12, 2, 128, 64, True, 1),       # several query tiles, ragged tail, per-head decisions
    (1050, 12, 2, 128, 256, False, 32),   # the paper's training length, blocks of 32, one decision per layer
    (517, 8, 2, 64, 100, True, 1),        # D = 64
    (129, 7, 1, 128, 1000, False, 1),     # no round fires: plain causal attention
])
def test_replay_parity(T, Hq, Hkv, D, period, per_head, block):
    rng = np.random.default_rng(T)
    B = 2
    q, k, v = _rand_bf16(rng, (B, T, Hq, D)), _rand_bf16(rng, (B, T, Hkv, D)), _rand_bf16(rng, (B, T, Hkv, D))
    if per_head:
        death = np.stack([np.stack([_random_death(rng, T, period, 0.5, block) for _ in range(Hkv)]) for _ in range(B)])
    else:
        death = np.stack([_random_death(rng, T, period, 0.5, block) for _ in range(B)])
    scale = 1.0 / np.sqrt(D)
    got = _run(q, k, v, death.astype(np.int32), Hq, Hkv, D, per_head, scale)
    _check(q, k, v, death, Hq, Hkv, D, per_head, scale, got)


def test_replay_equals_the_rollout():
    """Generate with the library (append, decode, evict every `period` tokens, greedy scores from a fixed
    table), then replay the whole trajectory in one call: every token's output must agree."""
    import torch
    ngc = _ngc()
    rng = np.random.default_rng(61)
    B, Hq, Hkv, D, T, period = 2, 12, 2, 128, 200, 48
    G = Hq // Hkv
    q, k, v = _rand_bf16(rng, (B, T, Hq, D)), _rand_bf16(rng, (B, T, Hkv, D)), _rand_bf16(rng, (B, T, Hkv, D))
    table = torch.from_numpy(rng.standard_normal((B, Hkv, T)).astype(np.float32)).cuda()   # score of every token
    cache = ngc.Cache.allocate(1, B, Hkv, Hq, D, T, with_pos=True)
    ws = ngc.allocate_workspace(cache, T)
    kept = torch.zeros(1, B, Hkv, T, dtype=torch.int32, device="cuda")
    logits = torch.zeros(1, B, Hkv, T, dtype=torch.float32, device="cuda")
    outs = torch.zeros(B, T, Hq, D, dtype=torch.float32, device="cuda")
    death = torch.full((B, Hkv, T), T, dtype=torch.int32, device="cuda")
    scale = 1.0 / np.sqrt(D)
    print("[rollout] append/decode/evict", flush=True)
    for i in range(T):
        if i > 0 and i % period == 0:
            n = cache.len.clone()
            logits[0] = torch.gather(table, 2, cache.pos[0].long().clamp(0, T - 1))
            keep = ((n + 1) // 2).contiguous()
            before = [[set(cache.pos[0, b, h, :int(n[0, b, h])].tolist()) for h in range(Hkv)] for b in range(B)]
            ngc.ngc_evict(cache, -1, logits, keep, ngc.make_params(noise_scale=0.0), T, kept, None, None, ws)
            torch.cuda.synchronize()
            for b in range(B):
                for h in range(Hkv):
                    after = set(cache.pos[0, b, h, :int(cache.len[0, b, h])].tolist())
                    for tok in before[b][h] - after:
                        death[b, h, tok] = i
        pos = torch.full((B,), i, dtype=torch.int32, device="cuda")
        ngc.ngc_cache_append(cache, 0, to_bf16_tensor(k[:, i], "cuda"), to_bf16_tensor(v[:, i], "cuda"), pos, ws)
        o = torch.zeros(B, Hq, D, dtype=torch.float32, device="cuda")
        ngc.ngc_decode_attn(cache, 0, to_bf16_tensor(q[:, i], "cuda"), scale, 0, o, ws)
        outs[:, i] = o
    torch.cuda.synchronize()
    assert all(x == 0 for x in ngc.read_status(ws))
    got = _run(q, k, v, death.cpu().numpy(), Hq, Hkv, D, True, scale)
    assert np.abs(got - outs.cpu().numpy()).max() <= 5e-5


def _sweep_cases():
    rng = np.random.default_rng(4518002)
    out = []
    for i in range(14):
        Hkv = int(rng.integers(1, 4))
        G = int(rng.choice([1, 2, 4, 6, 7]))
        out.append(dict(i=i, T=int(rng.choice([1, 31, 64, 65, 127, 129, 257, 500, 777, 1025])), Hkv=Hkv, Hq=Hkv * G,
                        D=int(rng.choice([64, 128])), period=int(rng.choice([16, 50, 128, 350])),
                        keep=float(rng.choice([0.1, 0.5, 0.9])), per_head=bool(rng.integers(0, 2)),
                        block=int(rng.choice([1, 1, 32])), B=int(rng.integers(1, 3))))
    return out


@pytest.mark.parametrize("c", _sweep_cases(), ids=lambda c: f"{c['i']}-T{c['T']}-D{c['D']}-p{c['period']}")
def test_replay_sweep(c):
    rng = np.random.default_rng(c["i"])
    B, T, Hq, Hkv, D = c["B"], c["T"], c["Hq"], c["Hkv"], c["D"]
    q, k, v = _rand_bf16(rng, (B, T, Hq, D)), _rand_bf16(rng, (B, T, Hkv, D)), _rand_bf16(rng, (B, T, Hkv, D))
    if c["per_head"]:
        death = np.stack([np.stack([_random_death(rng, T, c["period"], c["keep"], c["block"]) for _ in range(Hkv)])
                          for _ in range(B)])
    else:
        death = np.stack([_random_death(rng, T, c["period"], c["keep"], c["block"]) for _ in range(B)])
    scale = 1.0 / np.sqrt(D)
    got = _run(q, k, v, death.astype(np.int32), Hq, Hkv, D, c["per_head"], scale)
    _check(q, k, v, death, Hq, Hkv, D, c["per_head"], scale, got)


@pytest.mark.parametrize("scale", [0.0, -0.125, float("inf"), float("nan")])
def test_replay_rejects_a_scale_that_is_not_positive_and_finite(scale):
    """The kernel takes maxima on raw scores and scales afterwards: the scale has to be positive (ngc.h)."""
    rng = np.random.default_rng(7)
    T, Hq, Hkv, D = 40, 4, 2, 64
    q, k, v = _rand_bf16(rng, (1, T, Hq, D)), _rand_bf16(rng, (1, T, Hkv, D)), _rand_bf16(rng, (1, T, Hkv, D))
    death = np.full((1, T), T, np.int32)
    ngc = _ngc()
    with pytest.raises(ngc.NgcError) as e:
        _run(q, k, v, death, Hq, Hkv, D, False, scale)
    assert e.value.code == ngc.NGC_EINVAL
