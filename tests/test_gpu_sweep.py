"""Seeded sweep over geometries the hand-picked cases do not name: head counts, head dims, block sizes,
noise scales, ragged lengths around tile and workgroup-size boundaries.  Every case runs
evict -> append -> decode attention on the GPU and the same on the oracle."""
import numpy as np
import pytest

import oracle as orc
from paper_2604_18002_amd import synth

from _harness import from_bf16_tensor, host_case, oracle_evict_segment, to_bf16_tensor, upload

pytestmark = pytest.mark.gpu


def _cases():
    rng = np.random.default_rng(20260418)
    out = []
    for i in range(28):
        D = int(rng.choice([64, 128]))
        Hkv = int(rng.integers(1, 5))
        G = int(rng.choice([1, 2, 3, 4, 6, 7, 8, 12, 16]))
        top = int(rng.choice([33, 64, 257, 1000, 2049, 4097, 8192, 9000, 16384]))
        lo = max(1, int(top * rng.uniform(0.05, 1.0)))
        block = int(rng.choice([1, 1, 1, 2, 5, 32, 64]))
        tau = float(rng.choice([1.0, 1.0, 0.0, 0.25]))
        share = int(rng.integers(0, 2))
        keep_num, keep_den = [(1, 2), (1, 3), (2, 5), (9, 10), (1, 50)][int(rng.integers(0, 5))]
        out.append(dict(i=i, D=D, Hkv=Hkv, G=G, lo=lo, top=top, block=block, tau=tau, share=share,
                        keep_num=keep_num, keep_den=keep_den, L=int(rng.integers(1, 3)), B=int(rng.integers(1, 4))))
    return out


@pytest.mark.parametrize("c", _cases(), ids=lambda c: f"{c['i']}-D{c['D']}-G{c['G']}-n{c['top']}-b{c['block']}")
def test_sweep(c):
    import torch
    from paper_2604_18002_amd import binding as ngc
    w = synth.workload(1, L=c["L"], B=c["B"], Hkv=c["Hkv"], Hq=c["Hkv"] * c["G"], D=c["D"], n_lo=c["lo"], n_hi=c["top"],
                       keep_num=c["keep_num"], keep_den=c["keep_den"])
    case = host_case(w, block=c["block"])
    # two spare rows so that a no-op round (K = n) still leaves room for the append, unless that would
    # exceed the entry point's item limit (then K < n anyway)
    cap = w.cap + 2 if (w.cap + 2 + c["block"] - 1) // c["block"] <= 16384 else w.cap
    cache, logits, keep = upload(case, with_pos=True, cap=cap)
    max_keep = max(1, int(case.keep.max()))
    ws = ngc.allocate_workspace(cache, max_keep)
    kept = torch.full((w.L, w.B, w.Hkv, max_keep), -1, dtype=torch.int32, device="cuda")
    sigma = torch.full_like(kept, -1)
    logp = torch.zeros(w.L, w.B, w.Hkv, dtype=torch.float32, device="cuda")
    p = ngc.make_params(block=c["block"], share_heads=c["share"], noise_scale=c["tau"], round=3, seed=w.gumbel_seed)
    print(f"[sweep] {c}", flush=True)
    ngc.ngc_evict(cache, -1, logits, keep, p, max_keep, kept, sigma, logp, ws)
    nk = np.stack([synth.new_token_kv(w, l, 0)[0] for l in range(w.L)])
    nv = np.stack([synth.new_token_kv(w, l, 0)[1] for l in range(w.L)])
    q = np.stack([synth.queries(w, l, 9) for l in range(w.L)])
    ngc.ngc_cache_append(cache, -1, to_bf16_tensor(nk, "cuda"), to_bf16_tensor(nv, "cuda"), None, ws)
    out = torch.zeros(w.L, w.B, w.Hq, w.D, dtype=torch.float32, device="cuda")
    scale = 1.0 / np.sqrt(w.D)
    ngc.ngc_decode_attn(cache, -1, to_bf16_tensor(q, "cuda"), scale, 0, out, ws)
    torch.cuda.synchronize()
    assert all(x == 0 for x in ngc.read_status(ws))
    hk, hv = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v)
    hkept, hsig, hlp = kept.cpu().numpy(), sigma.cpu().numpy(), logp.cpu().numpy()
    hlen, hpos, hout = cache.len.cpu().numpy(), cache.pos.cpu().numpy(), out.cpu().numpy()
    for seg in case.segs:
        l, b, h = seg
        okept, osig, olp, ka, va = oracle_evict_segment(case, seg, c["tau"], w.gumbel_seed, 3, c["block"], bool(c["share"]))
        K = okept.size
        assert hkept[l, b, h, :K].tolist() == okept.tolist(), seg
        assert hsig[l, b, h, :K].tolist() == osig.tolist(), seg
        assert hlp[l, b, h] == pytest.approx(olp, rel=1e-4, abs=1e-5), seg
        n_new = ka.shape[0]
        assert hlen[l, b, h] == n_new + 1, seg
        assert hk[l, b, h, :n_new].tobytes() == ka.tobytes() and hv[l, b, h, :n_new].tobytes() == va.tobytes(), seg
        want_pos = orc.compact_i32(np.arange(case.k[seg].shape[0], dtype=np.int32), okept, c["block"])
        assert hpos[l, b, h, :n_new].tolist() == want_pos.tolist(), seg
        kk = np.concatenate([ka, nk[l, b, h][None]])
        vv = np.concatenate([va, nv[l, b, h][None]])
        want = orc.decode_attn(q[l, b, h * w.G:(h + 1) * w.G], kk, vv, scale)
        assert np.abs(hout[l, b, h * w.G:(h + 1) * w.G] - want).max() <= 2e-3, seg
