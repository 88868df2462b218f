"""Pins for the oracle's subset log-probability (Eq. 2 of the paper)."""
import itertools
import math

import numpy as np
import pytest
from scipy.special import gammaln, log_softmax, logsumexp

import oracle as orc


@pytest.mark.parametrize("n", [1, 2, 3, 5, 7, 8])
def test_ordered_probabilities_sum_to_one(n):
    rng = np.random.default_rng(n)
    s = (2.0 * rng.standard_normal(n)).astype(np.float32)
    for K in range(0, n + 1):
        if n == 8 and K not in (0, 1, 2, 3, 8):
            continue            # 8!/(8-K)! grows fast; the ends and small K cover the n=8 case
        total = 0.0
        for seq in itertools.permutations(range(n), K):
            total += math.exp(orc.logprob_literal(s, seq))
        assert total == pytest.approx(1.0, abs=1e-10), (n, K)


def test_single_pick_is_log_softmax():
    rng = np.random.default_rng(10)
    s = rng.standard_normal(50).astype(np.float32)
    ls = log_softmax(s.astype(np.float64))
    for t in (0, 7, 49):
        assert orc.logprob_literal(s, [t]) == pytest.approx(ls[t], rel=1e-13)
        assert orc.logprob_suffix(s, [t]) == pytest.approx(ls[t], rel=1e-13)


def test_equal_logits_closed_form():
    # every ordered K-sequence of n equally likely items has probability (n-K)!/n!
    for n, K in ((5, 2), (40, 40), (1000, 333), (4096, 1366)):
        s = np.full(n, 0.37, np.float32)
        sigma = np.random.default_rng(n).permutation(n)[:K]
        want = gammaln(n - K + 1) - gammaln(n + 1)
        assert orc.logprob_suffix(s, sigma) == pytest.approx(want, rel=1e-12)
        if n * K <= 2_000_000:
            assert orc.logprob_literal(s, sigma) == pytest.approx(want, rel=1e-12)


def test_two_step_example_by_hand():
    # n = 3, picks (2, 0): p = e^{s2}/(e^{s0}+e^{s1}+e^{s2}) * e^{s0}/(e^{s0}+e^{s1})
    s = np.array([0.5, -1.0, 2.0], np.float32)
    e = np.exp(s.astype(np.float64))
    want = math.log(e[2] / e.sum()) + math.log(e[0] / (e[0] + e[1]))
    assert orc.logprob_literal(s, [2, 0]) == pytest.approx(want, rel=1e-13)
    # the order matters (it is the probability of a sequence, not of a set)
    other = math.log(e[0] / e.sum()) + math.log(e[2] / (e[1] + e[2]))
    assert orc.logprob_literal(s, [0, 2]) == pytest.approx(other, rel=1e-13)
    assert abs(want - other) > 1e-3


def test_shift_invariance_and_literal_equals_suffix():
    rng = np.random.default_rng(11)
    for n, K in ((9, 9), (300, 120), (2048, 1024)):
        s = rng.standard_normal(n).astype(np.float64)
        sigma = rng.permutation(n)[:K]
        a = orc.logprob_literal(s.astype(np.float32), sigma)
        b = orc.logprob_suffix(s.astype(np.float32), sigma)
        assert a == pytest.approx(b, rel=1e-12)
        # shift by a power of two so that the fp32 logits shift exactly
        s32 = (np.round(s * 1024) / 1024).astype(np.float32)
        c = orc.logprob_suffix(s32, sigma)
        d = orc.logprob_suffix(s32 + np.float32(8.0), sigma)
        assert c == pytest.approx(d, rel=1e-12)


def test_against_independent_numpy_evaluation():
    # Eq. 2 re-evaluated with scipy's logsumexp over explicit remaining sets
    rng = np.random.default_rng(12)
    n, K = 200, 77
    s = (3 * rng.standard_normal(n)).astype(np.float32)
    sigma = rng.permutation(n)[:K]
    alive = np.ones(n, bool)
    want = 0.0
    for j in sigma:
        want += float(s[j]) - logsumexp(s[alive].astype(np.float64))
        alive[j] = False
    assert orc.logprob_literal(s, sigma) == pytest.approx(want, rel=1e-13)
    assert orc.logprob_suffix(s, sigma) == pytest.approx(want, rel=1e-13)


def test_heavy_tails_do_not_cancel():
    # a few huge logits picked first: the removed mass is ~1 after two picks; the
    # reverse running sum must still agree with the literal form
    rng = np.random.default_rng(13)
    n, K = 500, 200
    s = rng.standard_normal(n).astype(np.float32)
    s[[3, 100, 250]] = [38.0, 31.0, 25.0]
    keys = s.copy()
    order = np.argsort(-keys, kind="stable")[:K]
    a = orc.logprob_literal(s, order)
    b = orc.logprob_suffix(s, order)
    assert a == pytest.approx(b, rel=1e-12)
    assert np.isfinite(a)


def test_full_permutation_of_everything():
    # K = n: the unpicked mass is zero and the last factor is exactly 1
    s = np.array([0.1, 0.2, -0.3, 1.0], np.float32)
    e = np.exp(s.astype(np.float64))
    seq = [3, 1, 0, 2]
    want, rem = 0.0, e.sum()
    for i in seq:
        want += math.log(e[i] / rem)
        rem -= e[i]
    assert orc.logprob_literal(s, seq) == pytest.approx(want, rel=1e-12)
    assert orc.logprob_suffix(s, seq) == pytest.approx(want, rel=1e-12)
    assert orc.logprob_suffix(s, []) == 0.0


# ------------------------------------------------ gradient of Eq. 2 --------

def test_gradient_matches_finite_differences():
    rng = np.random.default_rng(14)
    n, K = 12, 5
    s = np.round(rng.standard_normal(n) * 64) / 64            # exactly representable in fp32
    sigma = rng.permutation(n)[:K]
    g = orc.logprob_grad(s.astype(np.float32), sigma)
    h = 2.0 ** -9                                             # exact step in fp32 at this magnitude
    for t in range(n):
        up, dn = s.copy(), s.copy()
        up[t] += h
        dn[t] -= h
        fd = (orc.logprob_literal(up.astype(np.float32), sigma) -
              orc.logprob_literal(dn.astype(np.float32), sigma)) / (2 * h)
        assert g[t] == pytest.approx(fd, abs=2e-5)


def test_gradient_invariants():
    rng = np.random.default_rng(15)
    n, K = 300, 120
    s = (2 * rng.standard_normal(n)).astype(np.float32)
    sigma = rng.permutation(n)[:K]
    g = orc.logprob_grad(s, sigma)
    assert g.sum() == pytest.approx(0.0, abs=1e-10)           # adding a constant to all logits changes nothing
    unpicked = np.setdiff1d(np.arange(n), sigma)
    assert (g[unpicked] < 0).all()                            # raising an unpicked logit lowers the probability
    # K = 1: one-hot minus softmax
    g1 = orc.logprob_grad(s, sigma[:1])
    want = -np.exp(log_softmax(s.astype(np.float64)))
    want[sigma[0]] += 1.0
    assert np.abs(g1 - want).max() < 1e-14
    # the last pick of a full permutation has zero gradient contribution beyond itself
    assert orc.logprob_grad(s[:5], [0, 1, 2, 3, 4]).sum() == pytest.approx(0.0, abs=1e-12)


# ------------------------------------------------ eviction loss (Eq. 4) ----

def test_lmem_by_hand():
    # one layer, one head, one prompt of two rollouts: rewards 1 and 0 -> advantages +1/2, -1/2.
    # rollout 0 fired two rounds (log-probs -1, -3), rollout 1 one round (-4; its second entry is unused)
    lp = np.array([[[[-1.0], [-4.0]]], [[[-3.0], [99.0]]]])          # [R=2, L=1, B=2, H=1]
    per_layer, total = orc.lmem(lp, [2, 1], [1.0, 0.0], group=2)
    want = -0.5 * (((-1.0 - 3.0) / 2) * 0.5 + (-4.0) * (-0.5))       # -(1/G) sum_i mean_t(logp) * A_i
    assert per_layer.tolist() == pytest.approx([want]) and total == pytest.approx(want)
    assert want == pytest.approx(-0.5)


def test_lmem_invariants():
    rng = np.random.default_rng(16)
    R, L, B, H, G = 5, 3, 8, 2, 4
    lp = -10.0 * rng.random((R, L, B, H))
    rounds = rng.integers(0, R + 1, size=B)
    rounds[0] = 0                                                    # a rollout that ended before its first round
    reward = rng.integers(0, 2, size=B).astype(np.float64)
    per_layer, total = orc.lmem(lp, rounds, reward, G)
    assert total == pytest.approx(per_layer.sum())
    # advantages are centred per prompt: a bonus to every rollout of a prompt changes nothing
    shifted = reward.copy()
    shifted[:G] += 3.0
    assert orc.lmem(lp, rounds, shifted, G)[1] == pytest.approx(total, abs=1e-12)
    assert orc.advantages(reward, G).reshape(-1, G).sum(axis=1) == pytest.approx(np.zeros(B // G), abs=1e-15)
    # equal rewards: no signal
    assert orc.lmem(lp, rounds, np.ones(B), G)[1] == 0.0
    # entries of rounds that never fired do not matter
    junk = lp.copy()
    for i in range(B):
        junk[rounds[i]:, :, i, :] = 1e6
    assert orc.lmem(junk, rounds, reward, G)[1] == pytest.approx(total, abs=1e-12)
    # the loss is linear in the log-probabilities: d loss / d logp[t, l, i, h] = -A_i / (B * rounds_i)
    adv = orc.advantages(reward, G)
    t, l, i, h = 1, 2, int(np.flatnonzero(rounds >= 2)[0]), 1
    bumped = lp.copy()
    bumped[t, l, i, h] += 1.0
    assert orc.lmem(bumped, rounds, reward, G)[1] - total == pytest.approx(-adv[i] / (B * rounds[i]), abs=1e-12)
    # vectorised numpy evaluation of the same formula
    w = np.where(np.arange(R)[:, None] < rounds[None, :], 1.0 / np.maximum(rounds, 1)[None, :], 0.0)   # [R, B]
    want = -(lp * w[:, None, :, None] * adv[None, None, :, None]).sum(axis=(0, 2, 3)) / B
    assert per_layer == pytest.approx(want, abs=1e-12)


def test_masked_entries():
    """Entries with logit -inf (masked keys): never picked, they drop out of every sum; picked, the sequence has
    probability zero.  Pinned to scipy's log-softmax (K = 1), to the same problem with the masked entries deleted,
    to the limit of very negative finite logits, and to the enumeration still summing to one."""
    s = np.array([0.3, -np.inf, 1.2, -0.7, -np.inf, 0.1], np.float32)
    ls = log_softmax(s.astype(np.float64))
    for t in range(s.size):
        assert orc.logprob_literal(s, [t]) == ls[t] or orc.logprob_literal(s, [t]) == pytest.approx(ls[t], rel=1e-13)
    assert orc.logprob_literal(s, [1]) == -np.inf and orc.logprob_suffix(s, [4]) == -np.inf
    # masked entries that are not picked change nothing: same value as with those entries deleted
    finite = np.array([0, 2, 3, 5])
    dense = s[finite]
    for seq in ((2, 0), (3, 1, 0), (0, 1, 2, 3)):
        full_seq = [int(finite[i]) for i in seq]
        assert orc.logprob_literal(s, full_seq) == pytest.approx(orc.logprob_literal(dense, seq), rel=1e-13)
        assert orc.logprob_suffix(s, full_seq) == pytest.approx(orc.logprob_suffix(dense, seq), rel=1e-13)
    # picked after every finite entry (also where only masked entries are left, the 0/0 case): -inf, never NaN
    for seq in ([0, 2, 3, 5, 1], [0, 2, 3, 5, 1, 4], [2, 1]):
        assert orc.logprob_literal(s, seq) == -np.inf
        assert orc.logprob_suffix(s, seq) == -np.inf
    # limit: a very negative finite logit in place of -inf gives a hugely negative value
    t = s.copy()
    t[[1, 4]] = -1e30
    assert orc.logprob_suffix(t, [2, 1]) < -1e29
    # the probabilities of all ordered pairs still sum to one
    total = sum(math.exp(orc.logprob_literal(s, seq)) for seq in itertools.permutations(range(s.size), 2))
    assert total == pytest.approx(1.0, abs=1e-12)
    # an all-masked segment: any pick has log-probability -inf
    m = np.full(5, -np.inf, np.float32)
    assert orc.logprob_literal(m, [3]) == -np.inf and orc.logprob_suffix(m, [0, 1]) == -np.inf


def test_selection_puts_masked_entries_last():
    """Masked entries are taken only after every finite one, lowest index first, with or without noise."""
    s = np.array([0.3, -np.inf, 1.2, -0.7, -np.inf, 0.1, -np.inf], np.float32)
    for tau in (0.0, 1.0):
        kept, sigma = orc.evict_select(s, 6, tau, 99, 0, 0, 0, 0)
        assert sorted(sigma[:4].tolist()) == [0, 2, 3, 5]
        assert sigma[4:].tolist() == [1, 4]
        assert kept.tolist() == [0, 1, 2, 3, 4, 5]
    kept, sigma = orc.evict_select(np.full(9, -np.inf, np.float32), 4, 1.0, 5, 0, 0, 0, 0)
    assert kept.tolist() == [0, 1, 2, 3] and sigma.tolist() == [0, 1, 2, 3]
