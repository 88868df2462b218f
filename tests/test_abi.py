"""The C-ABI library loads and exports every entry point that include/ngc.h
declares; host-side argument checks that need no GPU; host schedule logic."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2604_18002_amd import _build, schedule

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ngc.h")).read()
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


def test_version_and_strerror(lib):
    from paper_2604_18002_amd import binding
    assert lib.ngc_version() >= 100
    assert binding.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert isinstance(binding.strerror(code), str) and binding.strerror(code)


def test_struct_layout_matches_the_header():
    from paper_2604_18002_amd import binding
    # ngc_cache: 4 pointers + 6 int32; ngc_evict_params: 2 int32, float, u32, u64, 2 u32
    assert C.sizeof(binding.ngc_cache) == 4 * 8 + 6 * 4
    assert C.sizeof(binding.ngc_evict_params) == 32
    assert binding.ngc_evict_params.seed.offset == 16


def test_host_side_argument_checks_need_no_gpu(lib):
    from paper_2604_18002_amd import binding
    c = binding.ngc_cache(None, None, None, None, 1, 1, 2, 8, 64, 512)
    p = binding.make_params()
    # null cache pointers are rejected before anything touches a device
    assert lib.ngc_evict(C.byref(c), -1, None, None, C.byref(p), 1, None, None, None, None, 0, None) == binding.NGC_EINVAL
    assert lib.ngc_decode_attn(C.byref(c), 0, None, 0.125, 0, None, None, None, 0, None) == binding.NGC_EINVAL
    assert lib.ngc_subset_logprob(None, None, None, None, 1, 1, 1, None, None, 0, None) == binding.NGC_EINVAL
    assert lib.ngc_workspace_bytes(C.byref(c), 256) >= binding.STATUS_WORDS * 4 + 2 * 2 * 4


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
