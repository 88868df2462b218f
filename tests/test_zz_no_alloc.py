"""ngc_decode_attn_static: the decode-attention entry point for callers that
cannot allocate (no workspace argument: the split partials live in a fixed
array inside the library).  It must return what ngc_decode_attn returns, call
after call, also when a call with a smaller input follows a larger one."""
import ctypes as C

import numpy as np
import pytest

from paper_2604_18002_amd import synth

from _harness import host_case, to_bf16_tensor, upload

pytestmark = pytest.mark.gpu


def _case(idx, **over):
    import torch
    w = synth.workload(idx, **over)
    case = host_case(w)
    cache, _, _ = upload(case)
    q = to_bf16_tensor(synth.queries(w, 0), "cuda")
    return w, cache, q


def _both(ngc, w, cache, q, hint):
    """(workspace entry point, static entry point) through the C ABI, same inputs."""
    import torch
    lib = ngc.load_library()
    scale = 1.0 / np.sqrt(w.D)
    view = cache.view()
    stream = torch.cuda.current_stream().cuda_stream
    ws = ngc.allocate_workspace(cache, 1)
    ref = torch.full((w.B, w.Hq, w.D), 7.0, dtype=torch.float32, device="cuda")
    ref_lse = torch.zeros(w.B, w.Hq, dtype=torch.float32, device="cuda")
    rc = lib.ngc_decode_attn(C.byref(view), 0, q.data_ptr(), scale, hint, ref.data_ptr(), ref_lse.data_ptr(),
                             ws.data_ptr(), ws.numel(), stream)
    assert rc == 0
    got = torch.full_like(ref, -7.0)
    got_lse = torch.zeros_like(ref_lse)
    status = torch.zeros(ngc.STATUS_WORDS, dtype=torch.int32, device="cuda")
    rc = lib.ngc_decode_attn_static(C.byref(view), 0, q.data_ptr(), scale, hint, got.data_ptr(), got_lse.data_ptr(),
                                    status.data_ptr(), stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert status.cpu().tolist() == ngc.read_status(ws)
    # the Python binding of the same entry point (marshalling only) gives the same bits
    again = torch.full_like(ref, -9.0)
    ngc.ngc_decode_attn_static(cache, 0, q, scale, hint, again)
    torch.cuda.synchronize()
    assert torch.equal(again, got)
    return ref.cpu().numpy(), got.cpu().numpy(), ref_lse.cpu().numpy(), got_lse.cpu().numpy()


def test_static_entry_point_matches_the_workspace_one_twice_in_a_row():
    from paper_2604_18002_amd import binding as ngc
    ngc.load_library()
    # first call: 4 segments of 3000..4000 rows -> every segment is split and merged through the scratch array
    print("[static] large call: B=2, 3000..4000 rows, split partials in the fixed array", flush=True)
    w1, cache1, q1 = _case(1, B=2, n_lo=3000, n_hi=4000)
    ref, got, ref_lse, got_lse = _both(ngc, w1, cache1, q1, 0)
    assert np.all(np.isfinite(got))
    assert np.abs(got - ref).max() <= 2e-3
    assert np.array_equal(got, ref)            # same kernels, same split: the same bits
    assert np.array_equal(got_lse, ref_lse)
    # second call, smaller input, straight after: fewer segments, fewer rows, fewer splits
    print("[static] small call: B=1, 600..700 rows", flush=True)
    w2, cache2, q2 = _case(1, B=1, n_lo=600, n_hi=700)
    ref, got, ref_lse, got_lse = _both(ngc, w2, cache2, q2, 0)
    assert np.abs(got - ref).max() <= 2e-3
    assert np.array_equal(got, ref)
    assert np.array_equal(got_lse, ref_lse)
    # and a split case again after the small one (the array still holds the first call's partials)
    print("[static] split call after the small one: B=3, 2000..2600 rows, hint", flush=True)
    w3, cache3, q3 = _case(1, B=3, n_lo=2000, n_hi=2600)
    ref, got, _, _ = _both(ngc, w3, cache3, q3, 2600)
    assert np.array_equal(got, ref)


def test_static_entry_point_rejects_what_does_not_fit():
    """A launch whose partials exceed the fixed array is refused on the host with NGC_ENOSPC (nothing is enqueued)."""
    import torch
    from paper_2604_18002_amd import binding as ngc
    lib = ngc.load_library()
    # 128 segments per layer, 2 workgroups each, 16 query heads per KV head at D = 128:
    # 256 * 16 * 130 * 4 bytes = 2.13 MB of partials, more than the 2 MiB array
    A = 0x10000   # made-up aligned device address: the call is refused before anything is enqueued
    c = ngc.ngc_cache(A, A, A, None, 2, 32, 4, 64, 128, 2048)
    assert 4096 + 128 * 2 * 16 * 130 * 4 > ngc.STATIC_SCRATCH_BYTES
    rc = lib.ngc_decode_attn_static(C.byref(c), 0, A, 0.1, 0, A, None, None, torch.cuda.current_stream().cuda_stream)
    assert rc == ngc.NGC_ENOSPC
    assert "fixed scratch" in ngc.strerror(rc)


def test_static_entry_point_serves_caches_of_different_geometry_one_after_the_other():
    """The array's layout does not depend on the cache: a call with many segments after one with few (and back)
    finds its tickets at zero, not on the other call's partials."""
    from paper_2604_18002_amd import binding as ngc
    ngc.load_library()
    for over in (dict(B=2, n_lo=3000, n_hi=4000), dict(B=16, n_lo=900, n_hi=1100), dict(B=1, n_lo=2000, n_hi=2100),
                 dict(B=24, n_lo=700, n_hi=1300), dict(B=3, n_lo=3000, n_hi=3100)):
        print(f"[static] geometry {over}", flush=True)
        w, cache, q = _case(1, **over)
        ref, got, ref_lse, got_lse = _both(ngc, w, cache, q, 0)
        assert np.all(np.isfinite(got))
        assert np.array_equal(got, ref)
        assert np.array_equal(got_lse, ref_lse)
