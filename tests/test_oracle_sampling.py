"""Pins for the oracle's sampling half: the counter generator, the defined
logarithm, the Gumbel variate, the perturbed keys and the top-K selection.

None of these tests compares the oracle with itself: each checks it against a
published vector, a library routine, a closed form or a theorem.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------- Philox ----

def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_published_vectors():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = orc.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want


def test_item_word_counter_layout():
    # item t uses counter (t//4, b, l*65536 + hsel, round), key = seed halves, word t%4
    seed, rnd, l, b, h = 0x0123456789ABCDEF, 7, 3, 11, 2
    for t in (0, 1, 2, 3, 4, 5, 1023, 65537):
        blk = orc.philox4x32_10([t // 4, b, (l << 16) | h, rnd], [seed & 0xFFFFFFFF, seed >> 32])
        assert orc.item_word(seed, rnd, l, b, h, t) == int(blk[t % 4])
    # every coordinate matters
    base = orc.item_word(seed, rnd, l, b, h, 5)
    assert orc.item_word(seed + 1, rnd, l, b, h, 5) != base
    assert orc.item_word(seed, rnd + 1, l, b, h, 5) != base
    assert orc.item_word(seed, rnd, l + 1, b, h, 5) != base
    assert orc.item_word(seed, rnd, l, b + 1, h, 5) != base
    assert orc.item_word(seed, rnd, l, b, h + 1, 5) != base


def test_item_words_are_uniform():
    # 2^16 words: byte histogram chi-square and mean of the top bit
    words = np.array([orc.item_word(99, 0, 0, 0, 0, t) for t in range(1 << 16)], dtype=np.uint64)
    counts = np.bincount((words >> 24).astype(np.int64), minlength=256)
    chi2 = ((counts - 256.0) ** 2 / 256.0).sum()
    assert stats.chi2.sf(chi2, 255) > 1e-3
    counts = np.bincount((words & 0xFF).astype(np.int64), minlength=256)
    chi2 = ((counts - 256.0) ** 2 / 256.0).sum()
    assert stats.chi2.sf(chi2, 255) > 1e-3


# ---------------------------------------------------------- defined log ----

def test_defined_log_matches_libm():
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        np.exp(rng.uniform(-25, 4, 4000)),             # the range -log(u) and u live in
        1.0 - np.exp(rng.uniform(-23, -1, 2000)),      # just below 1 (upper Gumbel tail)
        np.array([1.0, 2.0, 0.5, math.sqrt(2), math.sqrt(0.5), 1.4142135623730951, 1.4142135623730954,
                  2.0 ** -33, 23.0, 1 - 2.0 ** -33]),
    ])
    for x in xs:
        got = orc.defined_log(float(x))
        want = math.log(x)
        assert got == pytest.approx(want, rel=4e-15, abs=1e-300), x
    assert orc.defined_log(1.0) == 0.0


def test_gumbel_is_minus_log_minus_log():
    for r in (0, 1, 12345, 2 ** 31, 2 ** 32 - 2, 2 ** 32 - 1):
        u = (r + 0.5) / 2.0 ** 32
        want = -math.log(-math.log(u)) if r < 2 ** 32 - 1000 else -math.log(-math.log1p(-(1 - u)))
        assert orc.gumbel_u32(r) == pytest.approx(want, rel=1e-13)
    # range of the variate: u in [2^-33, 1 - 2^-33]
    assert orc.gumbel_u32(0) == pytest.approx(-math.log(33 * math.log(2)), rel=1e-13)
    assert orc.gumbel_u32(2 ** 32 - 1) == pytest.approx(33 * math.log(2), rel=1e-9)


def test_gumbel_moments():
    g = np.array([orc.gumbel_u32(orc.item_word(5, 0, 0, 0, 0, t)) for t in range(100000)])
    assert g.mean() == pytest.approx(0.5772156649, abs=0.02)          # Euler-Mascheroni
    assert g.var() == pytest.approx(math.pi ** 2 / 6, abs=0.05)
    # Kolmogorov-Smirnov against the Gumbel CDF exp(-exp(-x))
    assert stats.kstest(g, lambda x: np.exp(-np.exp(-x))).pvalue > 1e-3


# ------------------------------------------------------- perturbed keys ----

def test_keys_formula_and_tau_zero():
    rng = np.random.default_rng(2)
    s = rng.standard_normal(37).astype(np.float32)
    seed, rnd, l, b, h = 42, 3, 1, 2, 1
    k1 = orc.perturbed_keys(s, 1.0, seed, rnd, l, b, h)
    k2 = orc.perturbed_keys(s, 0.5, seed, rnd, l, b, h)
    for t in range(37):
        g = orc.gumbel_u32(orc.item_word(seed, rnd, l, b, h, t))
        assert k1[t] == np.float32(float(s[t]) + g)
        assert k2[t] == np.float32(float(s[t]) + 0.5 * g)
    k0 = orc.perturbed_keys(s, 0.0, seed, rnd, l, b, h)
    assert k0.tobytes() == s.tobytes()
    # another round is another draw; the same round is the same draw
    assert orc.perturbed_keys(s, 1.0, seed, rnd + 1, l, b, h).tobytes() != k1.tobytes()
    assert orc.perturbed_keys(s, 1.0, seed, rnd, l, b, h).tobytes() == k1.tobytes()
    # a prefix of a segment draws the same noise as the whole segment
    assert orc.perturbed_keys(s[:9], 1.0, seed, rnd, l, b, h).tobytes() == k1[:9].tobytes()


# -------------------------------------------------------------- select -----

def test_zero_noise_is_sorted_topk():
    rng = np.random.default_rng(3)
    for n, K in ((1, 1), (7, 3), (64, 64), (100, 1), (513, 200), (4096, 1366)):
        s = rng.standard_normal(n).astype(np.float32)
        if n > 10:
            s[5] = s[1]          # a tie
            s[n - 1] = s[1]
        kept, sigma = orc.evict_select(s, K, 0.0, 1, 0, 0, 0, 0)
        order = np.argsort(-s.astype(np.float64), kind="stable")   # library routine
        assert sigma.tolist() == order[:K].tolist()
        assert kept.tolist() == sorted(order[:K].tolist())


def test_select_boundaries():
    s = np.array([0.5, -1.0, 3.0, 3.0, -0.0, 0.0, -np.inf, 2.0], np.float32)
    kept, sigma = orc.select(s, 8)
    assert kept.tolist() == list(range(8))
    # ties by index; +0 above -0; -inf last
    assert sigma.tolist() == [2, 3, 7, 0, 5, 4, 1, 6]
    kept, sigma = orc.select(s, 1)
    assert kept.tolist() == [2] and sigma.tolist() == [2]
    kept, sigma = orc.select(s, 0)
    assert kept.size == 0 and sigma.size == 0
    with pytest.raises(ValueError):
        orc.select(np.array([1.0, np.nan], np.float32), 1)
    with pytest.raises(ValueError):
        orc.select(s, 9)


def test_kept_is_sorted_sigma():
    rng = np.random.default_rng(4)
    s = rng.standard_normal(777).astype(np.float32)
    kept, sigma = orc.evict_select(s, 300, 1.0, 9, 1, 2, 3, 0)
    assert sorted(sigma.tolist()) == kept.tolist()
    assert len(set(sigma.tolist())) == 300
    keys = orc.perturbed_keys(s, 1.0, 9, 1, 2, 3, 0)
    assert np.all(np.diff(keys[sigma]) <= 0)
    assert keys[sigma].min() >= np.delete(keys, kept).max()


# --------------------- the theorem the method leans on (Sec. 4.3, Eq. 2) ---

def _pl_prob(s, seq):
    """Probability of an ordered draw without replacement, straight from the
    definition of sequential sampling (not from the oracle)."""
    w = np.exp(np.asarray(s, np.float64))
    p, rem = 1.0, w.sum()
    for i in seq:
        p *= w[i] / rem
        rem -= w[i]
    return p


def test_gumbel_max_frequencies_are_softmax():
    s = np.array([0.3, -1.2, 1.5, 0.0, 0.7], np.float32)
    N = 120000
    counts = np.zeros(5)
    for r in range(N):
        _, sigma = orc.evict_select(s, 1, 1.0, 1234, r, 0, 0, 0)
        counts[sigma[0]] += 1
    p = np.exp(s.astype(np.float64))
    p /= p.sum()
    chi2 = ((counts - N * p) ** 2 / (N * p)).sum()
    assert stats.chi2.sf(chi2, 4) > 1e-3


def test_gumbel_topk_frequencies_are_plackett_luce():
    import itertools
    s = np.array([0.9, -0.4, 0.2, 1.4, -1.0], np.float32)
    K, N = 3, 240000
    seqs = list(itertools.permutations(range(5), K))
    index = {q: i for i, q in enumerate(seqs)}
    counts = np.zeros(len(seqs))
    for r in range(N):
        # spread the draws over rounds, sequences and heads so every counter coordinate is exercised
        _, sigma = orc.evict_select(s, K, 1.0, 777, r % 1000, 0, r // 1000, r % 3)
        counts[index[tuple(sigma.tolist())]] += 1
    p = np.array([_pl_prob(s, q) for q in seqs])
    assert p.sum() == pytest.approx(1.0, abs=1e-12)
    chi2 = ((counts - N * p) ** 2 / (N * p)).sum()
    assert stats.chi2.sf(chi2, len(seqs) - 1) > 1e-3
    # and the oracle's Eq. 2 is the log of that probability
    for q in seqs[::7]:
        assert orc.logprob_literal(s, q) == pytest.approx(math.log(_pl_prob(s, q)), rel=1e-12)


def test_noise_scale_flattens_the_choice():
    # tau -> large makes every item (nearly) equally likely: not a pin of the
    # paper, a sanity check that tau multiplies the noise and not the logit
    s = np.array([3.0, 0.0, 0.0, 0.0], np.float32)
    N = 20000
    first = sum(int(orc.evict_select(s, 1, 50.0, 5, r, 0, 0, 0)[1][0] == 0) for r in range(N)) / N
    p = math.exp(3 / 50.0) / (math.exp(3 / 50.0) + 3)
    assert first == pytest.approx(p, abs=0.015)


# ------------------------------------------------------ pooled over heads ---

def test_pooled_selection_is_one_topk_over_all_heads():
    rng = np.random.default_rng(6)
    heads = [rng.standard_normal(n).astype(np.float32) for n in (50, 80, 65)]
    heads[1][:10] += 4.0                                  # one head clearly more important
    kept, sigma, cat, sig_idx = orc.evict_select_pooled(heads, 60, 0.0, 1, 0, 0, 0)
    order = np.argsort(-cat.astype(np.float64), kind="stable")[:60]      # library top-k over the concatenation
    assert sig_idx.tolist() == order.tolist()
    offs = [0, 50, 130]
    want = [sorted(int(i - offs[h]) for i in order if offs[h] <= i < offs[h] + len(heads[h])) for h in range(3)]
    assert [k.tolist() for k in kept] == want
    assert sum(k.size for k in kept) == 60 and kept[1].size > kept[0].size
    assert sigma[0] == (1, int(np.argmax(heads[1])))
    # with noise: every item keeps the noise of its own head, so a single head pooled alone is the per-head sample
    k1, s1, _, _ = orc.evict_select_pooled([heads[0]], 20, 1.0, 9, 2, 3, 4)
    k0, s0 = orc.evict_select(heads[0], 20, 1.0, 9, 2, 3, 4, 0)
    assert k1[0].tolist() == k0.tolist() and [t for _, t in s1] == s0.tolist()
