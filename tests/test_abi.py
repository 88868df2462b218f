"""The C-ABI library loads and exports every entry point that include/ngc.h
declares; host-side argument checks that need no GPU; host schedule logic."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2604_18002_amd import _build, schedule

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header="ngc.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ngc_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(_build.LIB_PATH):
        _build.build()
    from paper_2604_18002_amd import binding
    return binding.load_library()


def test_header_and_binding_name_the_same_entry_points():
    from paper_2604_18002_amd import binding
    assert _declared() == sorted(binding.EXPORTS)


def test_library_exports_every_declared_symbol(lib):
    for name in _declared():
        assert hasattr(lib, name), name


def test_probe_library_exports_what_its_header_declares(lib):
    """include/ngc_probe.h is the boundary of the second, measurement-only library."""
    from paper_2604_18002_amd import probe
    assert os.listdir(os.path.join(ROOT, "include")) == ["ngc.h", "ngc_probe.h"] or \
        sorted(os.listdir(os.path.join(ROOT, "include"))) == ["ngc.h", "ngc_probe.h"]
    assert _declared("ngc_probe.h") == sorted(probe.EXPORTS)
    plib = probe.load_library()
    for name in _declared("ngc_probe.h"):
        assert hasattr(plib, name), name
    # host-side argument checks, no GPU needed
    assert plib.ngc_probe_stream(1, None, None, 16, None) == -1
    assert plib.ngc_probe_copy_shape(0x1000, 0x2000, 1 << 20, 384, 4, 8, 0, None) == -1
    assert plib.ngc_probe_compact(0x1000, 0x2000, 0x3000, 0x4000, 1, 100, 200, 256, 4, 0, None) == -1


def test_version_and_strerror(lib):
    from paper_2604_18002_amd import binding
    assert lib.ngc_version() >= 100
    assert binding.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert isinstance(binding.strerror(code), str) and binding.strerror(code)


def test_struct_layout_matches_the_header():
    from paper_2604_18002_amd import binding
    # ngc_cache: 4 pointers + 6 int32; ngc_evict_params: 2 int32, float, u32, u64, u32, 3 int32
    assert C.sizeof(binding.ngc_cache) == 4 * 8 + 6 * 4
    assert C.sizeof(binding.ngc_evict_params) == 40
    assert binding.ngc_evict_params.seed.offset == 16
    assert binding.ngc_evict_params.layer_base.offset == 28 and binding.ngc_evict_params.seq_base.offset == 32


def test_host_side_argument_checks_need_no_gpu(lib):
    from paper_2604_18002_amd import binding
    c = binding.ngc_cache(None, None, None, None, 1, 1, 2, 8, 64, 512)
    p = binding.make_params()
    # null cache pointers are rejected before anything touches a device
    assert lib.ngc_evict(C.byref(c), -1, None, None, C.byref(p), 1, None, None, None, None, 0, None) == binding.NGC_EINVAL
    assert lib.ngc_decode_attn(C.byref(c), 0, None, 0.125, 0, None, None, None, 0, None) == binding.NGC_EINVAL
    assert lib.ngc_subset_logprob(None, None, None, None, 1, 1, 1, None, None, 0, None) == binding.NGC_EINVAL
    assert lib.ngc_workspace_bytes(C.byref(c), 256) >= binding.STATUS_WORDS * 4 + 2 * 2 * 4


def test_paged_struct_and_argument_checks_need_no_gpu(lib):
    from paper_2604_18002_amd import binding
    assert C.sizeof(binding.ngc_paged_cache) == 7 * 8 + 8 * 4
    A = 0x10000                      # a made-up, 16-byte aligned device address: the host side never reads it
    def pc(**kw):
        f = dict(k_pool=A, v_pool=A, pos_pool=None, table=A, len=A, free_stack=A, free_count=A,
                 L=2, B=3, Hkv=2, Hq=12, D=128, page_rows=32, max_pages=64, num_pages=1000)
        f.update(kw)
        return binding.ngc_paged_cache(*[f[k] for k, _ in binding.ngc_paged_cache._fields_])
    good = pc()
    need = lib.ngc_paged_workspace_bytes(C.byref(good))
    assert need >= binding.STATUS_WORDS * 4 + 2 * 4 * 12
    p32 = binding.make_params(block=32)
    def evict(cache, params=p32, stride=64, ws=A, ws_bytes=None, max_keep=8):
        return lib.ngc_paged_evict(C.byref(cache), -1, A, stride, A, C.byref(params), max_keep, A, None, None,
                                   ws, need if ws_bytes is None else ws_bytes, None)
    assert evict(pc(page_rows=48)) == binding.NGC_EINVAL                  # not a power of two
    assert evict(pc(page_rows=16)) == binding.NGC_EINVAL                  # below the 32-row tile
    assert evict(pc(D=96)) == binding.NGC_EINVAL
    assert evict(pc(Hq=13)) == binding.NGC_EINVAL                         # not a multiple of Hkv
    assert evict(pc(table=None)) == binding.NGC_EINVAL
    assert evict(pc(k_pool=A + 8)) == binding.NGC_EINVAL                  # misaligned pool
    assert evict(pc(max_pages=20000)) == binding.NGC_EUNSUPPORTED
    assert evict(good, params=binding.make_params(block=1)) == binding.NGC_EINVAL        # items are pages
    assert evict(good, stride=63) == binding.NGC_EINVAL                   # logit rows would overlap
    assert evict(good, params=binding.make_params(block=32, flags=binding.EVICT_UNORDERED)) == binding.NGC_EUNSUPPORTED
    assert evict(good, params=binding.make_params(block=32, flags=binding.EVICT_POOL_HEADS)) == binding.NGC_EUNSUPPORTED
    assert evict(good, ws_bytes=64) == binding.NGC_ENOSPC
    assert evict(good, max_keep=0) == binding.NGC_EINVAL
    assert lib.ngc_paged_append(C.byref(good), 5, A, A, None, A, need, None) == binding.NGC_EINVAL     # no such layer
    assert lib.ngc_paged_append(C.byref(good), 0, A + 4, A, None, A, need, None) == binding.NGC_EINVAL
    assert lib.ngc_paged_decode_attn(C.byref(good), -1, A, 0.1, 0, A, None, A, 16, None) == binding.NGC_ENOSPC
    assert lib.ngc_paged_decode_attn(C.byref(pc(page_rows=24)), -1, A, 0.1, 0, A, None, A, need, None) == binding.NGC_EINVAL
    assert lib.ngc_paged_score_keys(C.byref(good), -1, A, None, 20, 0.1, 0, 32, A, A, need, None) == binding.NGC_EUNSUPPORTED
    assert lib.ngc_paged_score_keys(C.byref(good), -1, A, A, 5, 0.1, binding.SCORE_NO_CAUSAL, 32, A, A, need, None) \
        == binding.NGC_EINVAL


def test_contiguous_argument_checks_need_no_gpu(lib):
    from paper_2604_18002_amd import binding
    A = 0x10000
    def cache(**kw):
        f = dict(k=A, v=A, len=A, pos=None, L=2, B=3, Hkv=2, Hq=12, D=128, cap=4096)
        f.update(kw)
        return binding.ngc_cache(*[f[k] for k, _ in binding.ngc_cache._fields_])
    good = cache()
    need = lib.ngc_workspace_bytes(C.byref(good), 100)
    p = binding.make_params()
    def evict(c, params=p, ws_bytes=None, max_keep=100):
        return lib.ngc_evict(C.byref(c), -1, A, A, C.byref(params), max_keep, A, None, None, A,
                             need if ws_bytes is None else ws_bytes, None)
    assert evict(cache(D=80)) == binding.NGC_EINVAL
    assert evict(cache(Hq=34)) == binding.NGC_EINVAL                      # more than 16 query heads per KV head
    assert evict(cache(v=A + 2)) == binding.NGC_EINVAL
    assert evict(cache(cap=70000)) == binding.NGC_EUNSUPPORTED            # more items than a segment's LDS holds
    assert evict(good, params=binding.make_params(block=0)) == binding.NGC_EINVAL
    assert evict(good, params=binding.make_params(block=2, flags=binding.EVICT_UNORDERED)) == binding.NGC_EUNSUPPORTED
    assert evict(good, params=binding.make_params(flags=binding.EVICT_POOL_HEADS), ws_bytes=need) == binding.NGC_ENOSPC
    assert evict(good, ws_bytes=8) == binding.NGC_ENOSPC
    assert lib.ngc_cache_append(C.byref(good), 2, A, A, None, A, need, None) == binding.NGC_EINVAL
    assert lib.ngc_decode_attn(C.byref(good), -1, A, float("nan"), 0, A, None, A, need, None) == binding.NGC_EINVAL
    assert lib.ngc_decode_attn(C.byref(good), -1, A, 0.1, -5, A, None, A, need, None) == binding.NGC_EINVAL
    assert lib.ngc_score_keys(C.byref(good), -1, A, None, 0, 0.1, 0, 1, A, A, need, None) == binding.NGC_EINVAL
    huge = cache(cap=1 << 24)                                             # 4 GiB per segment: beyond 32-bit offsets
    assert lib.ngc_decode_attn(C.byref(huge), -1, A, 0.1, 0, A, None, A, 1 << 40, None) == binding.NGC_EUNSUPPORTED
    assert lib.ngc_score_keys(C.byref(huge), -1, A, None, 5, 0.1, 0, 1, A, A, 1 << 40, None) == binding.NGC_EUNSUPPORTED
    assert lib.ngc_subset_logprob_backward(A, A, A, A, 4, 10, 10, 40000, None, A, A, need, None) == binding.NGC_EUNSUPPORTED
    assert lib.ngc_replay_attn(A, A, A, A, 1, 70000, 12, 2, 128, 0, 0.1, A, A, 1 << 30, None) != binding.NGC_OK


def test_workspace_grows_with_the_geometry(lib):
    from paper_2604_18002_amd import binding
    small = binding.ngc_cache(None, None, None, None, 1, 1, 2, 8, 64, 512)
    big = binding.ngc_cache(None, None, None, None, 28, 128, 4, 28, 128, 8192)
    a, b = lib.ngc_workspace_bytes(C.byref(small), 256), lib.ngc_workspace_bytes(C.byref(big), 3277)
    assert 0 < a < b < 1 << 30


# ------------------------------------------------------------- schedule ----

def test_keep_counts_match_the_scalar_rule():
    n = np.array([0, 1, 2, 512, 4096, 4097, 8192])
    for num, den in ((1, 2), (1, 3), (2, 5), (1, 1)):
        got = schedule.keep_counts(n, num, den)
        assert got.tolist() == [schedule.keep_count(int(x), num, den) for x in n]
    assert schedule.keep_count(4096, 1, 3) == 1366 and schedule.keep_count(8192, 2, 5) == 3277


def test_budget_split_sums_and_caps():
    w = np.array([1.0, 1.3, 0.6, 1.1])
    s = schedule.split_budget(21846, w, np.full(4, 16384))
    assert s.sum() == 21846 and (s >= 1).all() and (s <= 16384).all()
    assert len(set(s.tolist())) == 4                       # the heads really differ
    s = schedule.split_budget(10, np.ones(4), np.array([1, 100, 100, 100]))
    assert s[0] == 1 and (s <= [1, 100, 100, 100]).all()


def test_trajectories():
    # fraction rule: steady state delta / eps (Appendix A.2); budget rule: budget + delta
    assert schedule.trajectory(256, 256, 1, 2, 30)[-1] == 512
    t = schedule.trajectory(4096, 256, 1, 3, 6, rule="budget")
    assert t == [4096, 1366 + 256, 1366 + 256, 1366 + 256, 1366 + 256, 1366 + 256]
    # memory saving at 50 % eviction with cadence 256 and ~1k-token completions is a bit over 2x
    assert 2.0 < schedule.peak_reduction(100, 1024, 256, 1, 2) < 2.8


# ------------------------------------------------ independence of the two sides ----

def test_product_and_oracle_do_not_know_each_other():
    """The HIP path and the oracle share no code: neither imports, includes or loads the other; only the
    seeded input generators (synth, which holds none of the method's arithmetic) serve both."""
    import os
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2604_18002_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".c", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "ngc_oracle" not in text and "libngc_oracle" not in text, f
    for f in os.listdir(os.path.join(root, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(root, "oracle", f)).read()
            assert "paper_2604_18002_amd" not in text, f
            assert "libngc.so" not in text and "hip" not in text.lower().replace("relationship", ""), f
    # the header is the only thing the C ABI shares, and the oracle does not include it
    assert '#include "ngc.h"' not in open(os.path.join(root, "oracle", "ngc_oracle.c")).read()
    # synth holds generators only: none of the method's building blocks is named there
    segments = open(os.path.join(pkg, "synth.py")).read().split('"""')[0::2]          # text outside docstrings
    synth_code = "\n".join(line.split("#")[0] for seg in segments for line in seg.split("\n")).lower()
    for word in ("gumbel(", "philox", "softmax(", "logsumexp", "argsort", "topk", "exp("):
        assert word not in synth_code, word


def test_missing_library_is_an_error_not_a_fallback(tmp_path):
    from paper_2604_18002_amd import binding
    with pytest.raises(RuntimeError, match="missing"):
        binding.load_library(str(tmp_path / "no_such_libngc.so"))
