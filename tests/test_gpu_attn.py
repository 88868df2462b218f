"""GPU parity of decode attention (and of the whole evict -> append -> attend
sequence) against the CPU oracle, through the C ABI.

Tolerance: 2e-3 max-abs (bf16 inputs, fp32 scores / softmax / accumulation;
the kernel's own rounding is ~1e-5, see the split of P into two bf16 parts)."""
import numpy as np
import pytest

import oracle as orc
from paper_2604_18002_amd import synth

from _harness import from_bf16_tensor, host_case, oracle_evict_segment, to_bf16_tensor, upload

pytestmark = pytest.mark.gpu

ATOL = 2e-3


def _ngc():
    from paper_2604_18002_amd import binding
    binding.load_library()
    return binding


def _attend(ngc, cache, q_u16, layer, scale, hint=0, ws=None):
    import torch
    ws = ws if ws is not None else ngc.allocate_workspace(cache, 1)
    q = to_bf16_tensor(q_u16, "cuda")
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    print(f"[attn] layer={layer} q={tuple(q.shape)} cap={cache.k.shape[3]} hint={hint}", flush=True)
    ngc.ngc_decode_attn(cache, layer, q, scale, hint, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), ws


def _oracle_attend(w, hk, hv, hlen, q_u16, l, scale):
    """hk, hv: host copies [L,B,Hkv,cap,D]; q_u16 [B,Hq,D] -> fp32 [B,Hq,D]."""
    out = np.zeros((w.B, w.Hq, w.D), np.float32)
    G = w.G
    for b in range(w.B):
        for h in range(w.Hkv):
            n = int(hlen[l, b, h])
            out[b, h * G:(h + 1) * G] = orc.decode_attn(q_u16[b, h * G:(h + 1) * G], hk[l, b, h, :n],
                                                        hv[l, b, h, :n], scale)
    return out


@pytest.mark.parametrize("idx,over", [
    (0, {}),                                             # D = 64, G = 4, n = 512
    (1, {}),                                             # D = 128, G = 6, ragged 1024..2048
    (3, dict(L=2, B=5, n_lo=33, n_hi=700)),              # G = 7, short ragged
    (1, dict(B=3, n_lo=1, n_hi=70)),                     # tiny lengths incl. partial tiles
    (0, dict(B=7, Hq=32, Hkv=2, n_lo=100, n_hi=1000)),   # G = 16, D = 64
    (1, dict(B=2, Hq=2, Hkv=2, n_lo=3000, n_hi=5000)),   # G = 1, long
])
def test_dense_attention_parity(idx, over):
    ngc = _ngc()
    w = synth.workload(idx, **over)
    case = host_case(w)
    cache, _, _ = upload(case)
    hk, hv, hlen = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v), cache.len.cpu().numpy()
    scale = 1.0 / np.sqrt(w.D)
    qs = np.stack([synth.queries(w, l) for l in range(w.L)])          # [L,B,Hq,D]
    got_all, ws = _attend(ngc, cache, qs, -1, scale)
    for l in range(w.L):
        want = _oracle_attend(w, hk, hv, hlen, qs[l], l, scale)
        assert np.abs(got_all[l] - want).max() <= ATOL, f"all-layers call, layer {l}"
        got_one, _ = _attend(ngc, cache, qs[l], l, scale, ws=ws)
        assert np.abs(got_one - want).max() <= ATOL, f"single-layer call, layer {l}"
    assert all(x == 0 for x in ngc.read_status(ws))


def test_split_count_does_not_change_the_result():
    # the length hint only steers the split; results agree to fp32 reassociation
    ngc = _ngc()
    w = synth.workload(1, B=2, n_lo=2048, n_hi=2048)
    case = host_case(w)
    cache, _, _ = upload(case)
    q = synth.queries(w, 0)
    scale = 1.0 / np.sqrt(w.D)
    ref, ws = _attend(ngc, cache, q, 0, scale, hint=0)
    for hint in (1, 256, 512, 1024, 2047):
        got, _ = _attend(ngc, cache, q, 0, scale, hint=hint, ws=ws)
        assert np.abs(got - ref).max() <= 2e-5, hint


def test_peaked_softmax_and_large_scores():
    # one key nearly parallel to the query: softmax weight ~1 on a single row,
    # plus large score magnitudes; exercises the two-part P and the running max
    ngc = _ngc()
    w = synth.workload(1, B=2, n_lo=600, n_hi=900)
    case = host_case(w)
    q = synth.queries(w, 0)
    for (l, b, h) in case.segs:
        k = synth.bf16_bits_to_f32(case.k[(l, b, h)])
        qf = synth.bf16_bits_to_f32(q[b, h * w.G])
        k[137] = 4.0 * qf
        k[5] = 3.9 * qf
        case.k[(l, b, h)] = synth.f32_to_bf16_bits(k)
    cache, _, _ = upload(case)
    hk, hv, hlen = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v), cache.len.cpu().numpy()
    for scale in (1.0 / np.sqrt(w.D), 1.0):
        got, ws = _attend(ngc, cache, q, 0, scale)
        want = _oracle_attend(w, hk, hv, hlen, q, 0, scale)
        assert np.all(np.isfinite(got))
        assert np.abs(got - want).max() <= ATOL, scale


def test_permutation_of_retained_rows():
    import torch
    ngc = _ngc()
    w = synth.workload(1, B=2, n_lo=777, n_hi=777)
    case = host_case(w)
    cache, _, _ = upload(case)
    q = synth.queries(w, 0)
    scale = 1.0 / np.sqrt(w.D)
    a, ws = _attend(ngc, cache, q, 0, scale)
    perm = torch.from_numpy(np.random.default_rng(1).permutation(777)).cuda()
    cache.k[:, :, :, :777] = cache.k[:, :, :, perm]
    cache.v[:, :, :, :777] = cache.v[:, :, :, perm]
    b, _ = _attend(ngc, cache, q, 0, scale, ws=ws)
    assert np.abs(a - b).max() <= 2e-5


def test_empty_segment_gives_zeros_and_is_counted():
    ngc = _ngc()
    w = synth.workload(0, B=3)
    case = host_case(w)
    cache, _, _ = upload(case)
    cache.len[0, 1, :] = 0
    q = synth.queries(w, 0)
    got, ws = _attend(ngc, cache, q, 0, 0.125)
    assert np.array_equal(got[1], np.zeros_like(got[1]))
    assert np.all(np.isfinite(got))
    assert ngc.read_status(ws)[ngc.STATUS_EMPTY_ATTN] == w.Hkv


@pytest.mark.parametrize("idx,over", [(0, {}), (1, dict(B=6)), (4, dict(L=1, B=2))])
def test_evict_append_attend_sequence(idx, over):
    """The whole step: sample + compact, append the next token, attend."""
    import torch
    ngc = _ngc()
    w = synth.workload(idx, **over)
    case = host_case(w)
    cache, logits, keep = upload(case)
    max_keep = int(case.keep.max())
    ws = ngc.allocate_workspace(cache, max_keep)
    kept = torch.zeros(w.L, w.B, w.Hkv, max_keep, dtype=torch.int32, device="cuda")
    sigma = torch.zeros_like(kept)
    logp = torch.zeros(w.L, w.B, w.Hkv, dtype=torch.float32, device="cuda")
    p = ngc.make_params(noise_scale=1.0, round=0, seed=w.gumbel_seed)
    print(f"[step] workload={w.name} evict -> append -> attend", flush=True)
    ngc.ngc_evict(cache, -1, logits, keep, p, max_keep, kept, sigma, logp, ws)
    new = [synth.new_token_kv(w, l, 0) for l in range(w.L)]
    nk, nv = np.stack([x[0] for x in new]), np.stack([x[1] for x in new])
    ngc.ngc_cache_append(cache, -1, to_bf16_tensor(nk, "cuda"), to_bf16_tensor(nv, "cuda"), None, ws)
    qs = np.stack([synth.queries(w, l, 1) for l in range(w.L)])
    scale = 1.0 / np.sqrt(w.D)
    got, _ = _attend(ngc, cache, qs, -1, scale, hint=max_keep + 1, ws=ws)
    # oracle: same steps on the host copies
    for l in range(w.L):
        for b in range(w.B):
            for h in range(w.Hkv):
                _, _, _, k_after, v_after = oracle_evict_segment(case, (l, b, h), 1.0, w.gumbel_seed, 0)
                kk = np.concatenate([k_after, nk[l, b, h][None]])
                vv = np.concatenate([v_after, nv[l, b, h][None]])
                want = orc.decode_attn(qs[l, b, h * w.G:(h + 1) * w.G], kk, vv, scale)
                diff = np.abs(got[l, b, h * w.G:(h + 1) * w.G] - want).max()
                assert diff <= ATOL, ((l, b, h), diff)
    assert all(x == 0 for x in ngc.read_status(ws))


def test_one_very_long_segment_uses_the_maximum_split():
    """A single sequence of 65024 rows: 2 segments, so every segment is cut into the maximum number of splits
    (64) and merged; both layouts' entry points, against the oracle."""
    import torch
    ngc = _ngc()
    w = synth.workload(3, L=1, B=1, Hkv=2, Hq=14, n_lo=65024, n_hi=65024)
    case = host_case(w)
    cache, _, _ = upload(case)
    q = synth.queries(w, 0, 5)
    scale = 1.0 / np.sqrt(w.D)
    got, ws = _attend(ngc, cache, q, 0, scale, hint=0)
    want = _oracle_attend(w, from_bf16_tensor(cache.k), from_bf16_tensor(cache.v), cache.len.cpu().numpy(), q, 0, scale)
    assert np.abs(got - want).max() <= 2e-3
    # the same rows seen as a paged cache with an identity table: bit-identical to the contiguous call
    P = 128
    mp = w.cap // P                                    # 65024 = 508 pages of 128 rows
    nseg = w.Hkv
    table = (torch.arange(nseg, dtype=torch.int32, device="cuda")[:, None] * mp +
             torch.arange(mp, dtype=torch.int32, device="cuda")[None]).view(1, 1, w.Hkv, mp).contiguous()
    pc = ngc.PagedCache(cache.k.view(nseg * mp, P, w.D), cache.v.view(nseg * mp, P, w.D), None, table, cache.len,
                        torch.zeros(nseg * mp, dtype=torch.int32, device="cuda"),
                        torch.zeros(1, dtype=torch.int32, device="cuda"), w.Hq)
    out = torch.zeros(1, w.Hq, w.D, dtype=torch.float32, device="cuda")
    ngc.ngc_paged_decode_attn(pc, 0, to_bf16_tensor(q, "cuda"), scale, 0, out, ws)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), got)


@pytest.mark.parametrize("idx,over", [
    (0, {}),                                             # one workgroup per segment
    (1, dict(B=3, n_lo=31, n_hi=97)),                    # appended row opens a new tile for some segments (n = 32, 64, 96)
    (1, dict(B=2, n_lo=3000, n_hi=4000)),                # split segments: the last workgroup to finish stores the length
    (3, dict(L=2, B=4, n_lo=1500, n_hi=2600)),           # G = 7, two layers, ragged, split
])
def test_decode_step_equals_append_then_attend_and_the_oracle(idx, over):
    """ngc_decode_step (one launch) against ngc_cache_append + ngc_decode_attn on a copy of the cache, bit for bit
    (cache bytes, lengths, positions, outputs, log-sum-exp), and against the oracle on the grown cache."""
    import torch
    ngc = _ngc()
    w = synth.workload(idx, **over)
    case = host_case(w)
    cache, _, _ = upload(case, with_pos=True, cap=w.cap + 8)       # room for the appended rows
    ref = ngc.Cache(cache.k.clone(), cache.v.clone(), cache.len.clone(), cache.pos.clone(), cache.Hq)
    scale = 1.0 / np.sqrt(w.D)
    ws = ngc.allocate_workspace(cache, 1)
    ws_ref = ngc.allocate_workspace(ref, 1)
    for step in range(3):                                # lengths grow across tile boundaries step by step
        for l in range(w.L):
            nk, nv = synth.new_token_kv(w, l, step)
            q = synth.queries(w, l, 10 + step)
            tk, tv, tq = to_bf16_tensor(nk, "cuda"), to_bf16_tensor(nv, "cuda"), to_bf16_tensor(q, "cuda")
            new_pos = torch.full((w.B,), 100000 + step, dtype=torch.int32, device="cuda")
            out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float32, device="cuda")
            lse = torch.full((w.B, w.Hq), float("nan"), dtype=torch.float32, device="cuda")
            out_ref, lse_ref = torch.zeros_like(out), torch.zeros_like(lse)
            print(f"[step] workload={w.name} step={step} layer={l}", flush=True)
            ngc.ngc_decode_step(cache, l, tk, tv, new_pos, tq, scale, 0, out, ws, lse_out=lse)
            ngc.ngc_cache_append(ref, l, tk, tv, new_pos, ws_ref)
            ngc.ngc_decode_attn(ref, l, tq, scale, 0, out_ref, ws_ref, lse_out=lse_ref)
            torch.cuda.synchronize()
            assert torch.equal(cache.len, ref.len)
            assert torch.equal(out, out_ref) and torch.equal(lse, lse_ref)
            hk, hv, hlen = from_bf16_tensor(cache.k), from_bf16_tensor(cache.v), cache.len.cpu().numpy()
            want = _oracle_attend(w, hk, hv, hlen, q, l, scale)
            assert np.abs(out.cpu().numpy() - want).max() <= ATOL
            for b in range(w.B):
                for h in range(w.Hkv):
                    n = int(hlen[l, b, h])
                    assert n == case.k[(l, b, h)].shape[0] + step + 1
                    assert hk[l, b, h, n - 1].tobytes() == nk[b, h].tobytes()
                    assert hv[l, b, h, n - 1].tobytes() == nv[b, h].tobytes()
    assert torch.equal(cache.k, ref.k) and torch.equal(cache.v, ref.v) and torch.equal(cache.pos, ref.pos)
    assert all(x == 0 for x in ngc.read_status(ws))
    # the tickets of every segment are back at zero
    nseg = w.L * w.B * w.Hkv
    assert int(ws[ngc.STATUS_WORDS * 4:ngc.STATUS_WORDS * 4 + 12 * nseg].view(torch.int32).abs().sum()) == 0


def test_decode_step_on_a_full_segment_attends_without_appending():
    import torch
    ngc = _ngc()
    w = synth.workload(1, B=2, n_lo=640, n_hi=640)
    case = host_case(w)
    cache, _, _ = upload(case, cap=640)                 # every segment is full
    q = synth.queries(w, 0)
    nk, nv = synth.new_token_kv(w, 0, 0)
    scale = 1.0 / np.sqrt(w.D)
    ws = ngc.allocate_workspace(cache, 1)
    out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.float32, device="cuda")
    before = cache.k.clone()
    ngc.ngc_decode_step(cache, 0, to_bf16_tensor(nk, "cuda"), to_bf16_tensor(nv, "cuda"), None, to_bf16_tensor(q, "cuda"),
                        scale, 0, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(cache.k, before) and int(cache.len.min()) == 640 and int(cache.len.max()) == 640
    assert ngc.read_status(ws)[ngc.STATUS_APPEND_FULL] == w.B * w.Hkv
    want = _oracle_attend(w, from_bf16_tensor(cache.k), from_bf16_tensor(cache.v), cache.len.cpu().numpy(), q, 0, scale)
    assert np.abs(out.cpu().numpy() - want).max() <= ATOL
