"""Pins for the oracle's key scoring and block coarsening (Sec. 4.2)."""
import numpy as np
import pytest
from scipy.special import softmax

import oracle as orc
from paper_2604_18002_amd import synth


def _rand_bf16(rng, shape, sd=1.0):
    return synth.f32_to_bf16_bits((sd * rng.standard_normal(shape)).astype(np.float32))


def _f(x):
    return synth.bf16_bits_to_f32(x).astype(np.float64)


def test_single_query_single_head_is_one_softmax_row():
    rng = np.random.default_rng(40)
    n, D = 77, 64
    q, k = _rand_bf16(rng, (1, 1, D)), _rand_bf16(rng, (n, D))
    got = orc.score_keys(q, k, 0.125, causal=True)        # the one query is the last token: sees all rows
    want = softmax(_f(k) @ _f(q[0, 0]) * 0.125)
    assert np.abs(got - want).max() < 1e-14


def test_scores_are_an_average_of_distributions():
    rng = np.random.default_rng(41)
    n, D, w, G = 300, 128, 5, 6
    q, k = _rand_bf16(rng, (w, G, D)), _rand_bf16(rng, (n, D))
    for causal in (True, False):
        psi = orc.score_keys(q, k, 1 / np.sqrt(D), causal)
        assert psi.sum() == pytest.approx(1.0, abs=1e-12)
        assert (psi >= 0).all()


def test_against_library_softmax_with_causal_window():
    rng = np.random.default_rng(42)
    n, D, w, G = 40, 32, 5, 3
    q, k = _rand_bf16(rng, (w, G, D)), _rand_bf16(rng, (n, D))
    scale = 0.2
    want = np.zeros(n)
    for j in range(w):
        vis = n - w + j + 1
        for g in range(G):
            want[:vis] += softmax(_f(k[:vis]) @ _f(q[j, g]) * scale)
    want /= w * G
    assert np.abs(orc.score_keys(q, k, scale, True) - want).max() < 1e-14
    # the newest key is seen by the newest query only
    assert orc.score_keys(q, k, scale, True)[n - 1] <= 1.0 / w + 1e-12
    # without the causal window every query sees everything
    full = sum(softmax(_f(k) @ _f(q[j, g]) * scale) for j in range(w) for g in range(G)) / (w * G)
    assert np.abs(orc.score_keys(q, k, scale, False) - full).max() < 1e-14


def test_single_query_matches_the_attention_oracle():
    # with one-hot value rows the attention output *is* the probability vector
    rng = np.random.default_rng(43)
    n, D, G = 48, 64, 4
    q, k = _rand_bf16(rng, (1, G, D)), _rand_bf16(rng, (n, D))
    v = synth.f32_to_bf16_bits(np.eye(n, D, dtype=np.float32))
    probs = orc.decode_attn(q[0], k, v, 0.125)[:, :n].astype(np.float64)      # [G, n]
    assert np.abs(orc.score_keys(q, k, 0.125, True) - probs.mean(0)).max() < 1e-7


def test_short_cache_and_window_longer_than_cache():
    rng = np.random.default_rng(44)
    D = 32
    q, k = _rand_bf16(rng, (5, 2, D)), _rand_bf16(rng, (3, D))
    psi = orc.score_keys(q, k, 0.3, True)      # only the last 3 of the 5 queries have a row to see
    assert psi.sum() == pytest.approx(3 / 5, abs=1e-12)
    assert orc.score_keys(q, k[:0], 0.3, True).size == 0


def test_block_means():
    rng = np.random.default_rng(45)
    psi = rng.random(100)
    for b in (1, 7, 32, 100, 128):
        s = orc.block_means(psi, b)
        N = (100 + b - 1) // b
        want = np.array([psi[j * b:(j + 1) * b].mean() for j in range(N)])
        assert np.abs(s - want).max() < 1e-15
        sizes = np.array([min(b, 100 - j * b) for j in range(N)])
        assert (s * sizes).sum() == pytest.approx(psi.sum(), rel=1e-13)
