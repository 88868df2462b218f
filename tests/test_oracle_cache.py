"""Pins for the oracle's compaction, decode attention and cache-size schedule."""
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import softmax

import oracle as orc
from paper_2604_18002_amd import synth


# ------------------------------------------------------------ compaction ---

def test_compaction_is_boolean_mask_indexing():
    rng = np.random.default_rng(20)
    n, D = 300, 64
    rows = rng.integers(0, 65536, size=(n, D), dtype=np.uint16)
    pos = np.arange(n, dtype=np.int32) * 3 + 1
    mask = rng.random(n) < 0.4
    kept = np.flatnonzero(mask).astype(np.int32)
    assert orc.compact_rows(rows, kept).tobytes() == rows[mask].tobytes()
    assert orc.compact_i32(pos, kept).tolist() == pos[mask].tolist()


def test_compaction_keep_all_and_prefix():
    rng = np.random.default_rng(21)
    rows = rng.integers(0, 65536, size=(50, 8), dtype=np.uint16)
    assert orc.compact_rows(rows, np.arange(50)).tobytes() == rows.tobytes()
    assert orc.compact_rows(rows, np.arange(17)).tobytes() == rows[:17].tobytes()
    assert orc.compact_rows(rows, np.zeros(0, np.int32)).shape == (0, 8)
    # greedy selection on decreasing logits keeps the prefix, so nothing moves
    s = -np.arange(50, dtype=np.float32)
    kept, _ = orc.evict_select(s, 20, 0.0, 0, 0, 0, 0, 0)
    assert orc.compact_rows(rows, kept).tobytes() == rows[:20].tobytes()


def test_compaction_of_blocks():
    # items are blocks of 4 rows; 10 rows -> blocks of sizes 4, 4, 2
    rows = np.arange(10 * 2, dtype=np.uint16).reshape(10, 2)
    got = orc.compact_rows(rows, [0, 2], block=4)
    assert got.tolist() == rows[[0, 1, 2, 3, 8, 9]].tolist()
    got = orc.compact_rows(rows, [1], block=4)
    assert got.tolist() == rows[4:8].tolist()
    assert orc.compact_i32(np.arange(10), [1, 2], block=4).tolist() == [4, 5, 6, 7, 8, 9]


def test_unordered_compaction_by_hand_and_as_a_set():
    # n = 8, keep {1, 2, 5, 7}: K = 4, holes among slots 0..3 are 0 and 3, tails are 5 and 7
    rows = (np.arange(8, dtype=np.uint16)[:, None] * 10 + np.arange(3, dtype=np.uint16)[None]).astype(np.uint16)
    got = orc.compact_rows_unordered(rows, [1, 2, 5, 7])
    assert got.tolist() == rows[[5, 1, 2, 7]].tolist()
    # nothing beyond K kept: nothing moves; everything kept: nothing moves
    assert orc.compact_rows_unordered(rows, [0, 1, 2]).tolist() == rows[:3].tolist()
    assert orc.compact_rows_unordered(rows, np.arange(8)).tolist() == rows.tolist()
    # same multiset of rows as the ordered compaction, rows below K that are kept do not move
    rng = np.random.default_rng(22)
    n, D, K = 500, 4, 180
    big = rng.integers(0, 65536, size=(n, D), dtype=np.uint16)
    big[:, 0] = np.arange(n)                      # make rows distinct and traceable
    kept = np.sort(rng.permutation(n)[:K]).astype(np.int32)
    a, b = orc.compact_rows(big, kept), orc.compact_rows_unordered(big, kept)
    assert sorted(map(tuple, a.tolist())) == sorted(map(tuple, b.tolist()))
    stay = kept[kept < K]
    assert b[stay].tolist() == big[stay].tolist()
    moved = int((b[:, 0] != np.arange(K)).sum())
    assert moved == int((kept >= K).sum())        # exactly the tails move


# ------------------------------------------------------------- attention ---

def _dense_reference(q, k, v, scale):
    """Dense softmax attention from library routines, fp64."""
    qf = synth.bf16_bits_to_f32(q).astype(np.float64)
    kf = synth.bf16_bits_to_f32(k).astype(np.float64)
    vf = synth.bf16_bits_to_f32(v).astype(np.float64)
    p = softmax(qf @ kf.T * scale, axis=-1)
    return p @ vf


def _rand_bf16(rng, shape, sd=1.0):
    return synth.f32_to_bf16_bits((sd * rng.standard_normal(shape)).astype(np.float32))


@pytest.mark.parametrize("G,D,n", [(4, 64, 257), (6, 128, 100), (7, 128, 1), (1, 32, 33)])
def test_keep_everything_is_dense_attention(G, D, n):
    rng = np.random.default_rng(30 + n)
    q, k, v = _rand_bf16(rng, (G, D)), _rand_bf16(rng, (n, D)), _rand_bf16(rng, (n, D))
    scale = 1.0 / np.sqrt(D)
    got = orc.decode_attn(q, k, v, scale)
    want = _dense_reference(q, k, v, scale)
    assert np.abs(got - want).max() < 1e-6          # fp32 rounding of the output only
    assert got.dtype == np.float32


def test_attention_over_kept_rows_only():
    # evict, compact, attend == dense attention restricted to the kept set
    rng = np.random.default_rng(31)
    G, D, n, K = 4, 64, 200, 71
    q, k, v = _rand_bf16(rng, (G, D)), _rand_bf16(rng, (n, D)), _rand_bf16(rng, (n, D))
    s = rng.standard_normal(n).astype(np.float32)
    kept, _ = orc.evict_select(s, K, 1.0, 3, 0, 0, 0, 0)
    got = orc.decode_attn(q, orc.compact_rows(k, kept), orc.compact_rows(v, kept), 0.125)
    want = _dense_reference(q, k[kept], v[kept], 0.125)
    assert np.abs(got - want).max() < 1e-6


def test_permutation_invariance():
    rng = np.random.default_rng(32)
    G, D, n = 6, 128, 150
    q, k, v = _rand_bf16(rng, (G, D)), _rand_bf16(rng, (n, D)), _rand_bf16(rng, (n, D))
    perm = rng.permutation(n)
    a = orc.decode_attn(q, k, v, 0.0884)
    b = orc.decode_attn(q, k[perm], v[perm], 0.0884)
    assert np.abs(a - b).max() < 1e-6
    # permuting K without V is a different function: the test above is not vacuous
    c = orc.decode_attn(q, k[perm], v, 0.0884)
    assert np.abs(a - c).max() > 1e-3


def test_attention_special_cases():
    rng = np.random.default_rng(33)
    G, D, n = 3, 64, 40
    q, k, v = _rand_bf16(rng, (G, D)), _rand_bf16(rng, (n, D)), _rand_bf16(rng, (n, D))
    vf = synth.bf16_bits_to_f32(v).astype(np.float64)
    # one row: the output is that row of V exactly
    one = orc.decode_attn(q, k[:1], v[:1], 0.125)
    assert np.array_equal(one, np.broadcast_to(synth.bf16_bits_to_f32(v[:1]), (G, D)))
    # all K rows equal, or q = 0, or scale = 0: uniform weights -> mean of V
    same = orc.decode_attn(q, np.repeat(k[:1], n, 0), v, 0.125)
    assert np.abs(same - vf.mean(0)).max() < 1e-6
    zero_q = orc.decode_attn(np.zeros_like(q), k, v, 0.125)
    assert np.abs(zero_q - vf.mean(0)).max() < 1e-6
    assert np.abs(orc.decode_attn(q, k, v, 0.0) - vf.mean(0)).max() < 1e-6
    # the scale multiplies the scores (1/sqrt(d_h) in the paper): doubling q's
    # exponent equals doubling the scale
    q2 = synth.f32_to_bf16_bits(2.0 * synth.bf16_bits_to_f32(q))
    assert np.abs(orc.decode_attn(q2, k, v, 0.125) - orc.decode_attn(q, k, v, 0.25)).max() < 1e-6
    # nothing retained
    assert np.array_equal(orc.decode_attn(q, k[:0], v[:0], 0.125), np.zeros((G, D), np.float32))


def test_attention_large_scores_do_not_overflow():
    rng = np.random.default_rng(34)
    q, k, v = _rand_bf16(rng, (2, 64), 30.0), _rand_bf16(rng, (50, 64), 30.0), _rand_bf16(rng, (50, 64))
    got = orc.decode_attn(q, k, v, 1.0)
    want = _dense_reference(q, k, v, 1.0)
    assert np.all(np.isfinite(got))
    assert np.abs(got - want).max() < 1e-6


# -------------------------------------------------------------- schedule ---

def test_keep_count_is_a_clamped_ceiling():
    assert orc.keep_count(4096, 1, 3) == 1366
    assert orc.keep_count(512, 1, 2) == 256
    assert orc.keep_count(8192, 2, 5) == 3277
    assert orc.keep_count(4097, 2, 5) == 1639
    assert orc.keep_count(1, 1, 3) == 1
    assert orc.keep_count(0, 1, 3) == 0
    assert orc.keep_count(7, 1, 1) == 7


@pytest.mark.parametrize("delta,num,den", [(256, 1, 2), (256, 2, 3), (350, 1, 2), (1024, 1, 3), (512, 3, 5)])
def test_cache_size_converges_to_delta_over_eps(delta, num, den):
    # Appendix A.2: c_{t+1} = (1 - eps) c_t + delta has the fixed point delta / eps
    star = orc.steady_state(delta, num, den)
    assert star == Fraction(delta * den, den - num)
    sizes = orc.trajectory_fraction(delta, delta, num, den, 80)
    for a, b in zip(sizes, sizes[1:]):
        exact = Fraction(num, den) * a + delta
        assert 0 <= b - exact < 1                       # the recursion, up to the ceiling
    assert abs(sizes[-1] - star) <= den / (den - num) + 1   # converged to within the rounding slack
    assert max(sizes) <= float(star) + den / (den - num) + 1


def test_paper_example_half_eviction():
    # eviction rate 1/2 with cadence 256: the steady state before a round is 512
    assert orc.steady_state(256, 1, 2) == 512
    assert orc.trajectory_fraction(256, 256, 1, 2, 30)[-1] == 512


def test_decode_lse_is_library_logsumexp():
    from scipy.special import logsumexp
    rng = np.random.default_rng(35)
    G, D, n = 5, 64, 123
    q, k = _rand_bf16(rng, (G, D)), _rand_bf16(rng, (n, D))
    qf = synth.bf16_bits_to_f32(q).astype(np.float64)
    kf = synth.bf16_bits_to_f32(k).astype(np.float64)
    want = logsumexp(qf @ kf.T * 0.125, axis=1)
    assert np.abs(orc.decode_lse(q, k, 0.125) - want).max() < 1e-12
    assert np.isneginf(orc.decode_lse(q, k[:0], 0.125)).all()
