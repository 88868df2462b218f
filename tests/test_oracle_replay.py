"""Pins for the oracle's replay-mask attention (Sec. 4.5, Appendix A.3)."""
import os

import numpy as np
import pytest
from scipy.special import softmax

import oracle as orc
from paper_2604_18002_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_bf16(rng, shape):
    return synth.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def _f(x):
    return synth.bf16_bits_to_f32(x).astype(np.float64)


def test_figure_example_of_the_paper():
    rows = {}
    with open(os.path.join(GOLDEN, "replay_mask_fig2.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            i, js = line.split(":")
            rows[int(i)] = [int(x) for x in js.split()]
    # round 1 over alive {0..4} drops 1 and 3; round 2 over alive {0,2,4,5,6,7} drops 2 and 5
    death = orc.replay_death(10, [5, 8], [[1, 0, 1, 0, 1], [1, 0, 1, 0, 1, 1]])
    assert death.tolist() == [10, 5, 8, 5, 10, 8, 10, 10, 10, 10]
    mask = orc.replay_mask(death)
    for i in range(10):
        assert np.flatnonzero(mask[i]).tolist() == rows[i], i


def _appendix_mask(T, period, decisions):
    """The construction of Appendix A.3, written out: blocks of `period` tokens, causal inside a
    block, every query of block r+1 also sees kept_r, diagonal set."""
    M = np.zeros((T, T), bool)
    nblocks = (T + period - 1) // period
    alive = list(range(0, min(period, T)))
    kept = []
    for r in range(nblocks):
        lo, hi = r * period, min((r + 1) * period, T)
        for i in range(lo, hi):
            M[i, lo:i + 1] = True                 # causal within the block
            M[i, kept] = True                     # plus everything kept by the previous round
        if r < len(decisions):
            dec = np.asarray(decisions[r]).astype(bool)
            kept = [tok for tok, keep in zip(alive, dec) if keep]
            alive = kept + list(range(hi, min(hi + period, T)))
    M[np.arange(T), np.arange(T)] = True
    return M


@pytest.mark.parametrize("T,period", [(10, 5), (37, 8), (64, 16), (50, 7)])
def test_death_predicate_equals_the_appendix_construction(T, period):
    rng = np.random.default_rng(T)
    R = (T + period - 1) // period - 1
    boundaries = [(r + 1) * period for r in range(R)]
    decisions, alive = [], 0
    n_alive = 0
    for r in range(R):
        n_alive += period
        dec = rng.random(n_alive) < 0.6
        decisions.append(dec.astype(np.int32))
        n_alive = int(dec.sum())
    death = orc.replay_death(T, boundaries, decisions)
    assert np.array_equal(orc.replay_mask(death), _appendix_mask(T, period, decisions))


def test_replay_row_equals_decoding_over_the_pruned_cache():
    # generate token by token with periodic eviction; the attention each token saw at generation
    # time (decode over the compacted cache) must equal its row of the replay attention
    rng = np.random.default_rng(50)
    T, G, D, period = 45, 3, 32, 10
    q, k, v = _rand_bf16(rng, (T, G, D)), _rand_bf16(rng, (T, D)), _rand_bf16(rng, (T, D))
    scale = 1 / np.sqrt(D)
    alive, boundaries, decisions, rows = [], [], [], []
    for i in range(T):
        if i > 0 and i % period == 0:
            s = rng.standard_normal(len(alive)).astype(np.float32)
            kept, _ = orc.evict_select(s, orc.keep_count(len(alive), 1, 2), 1.0, 5, i // period, 0, 0, 0)
            dec = np.zeros(len(alive), np.int32)
            dec[kept] = 1
            boundaries.append(i)
            decisions.append(dec)
            alive = [alive[j] for j in kept]
        alive.append(i)
        rows.append(orc.decode_attn(q[i], k[alive], v[alive], scale))
    death = orc.replay_death(T, boundaries, decisions)
    got = orc.replay_attn(q, k, v, death, scale)
    assert np.abs(got - np.stack(rows)).max() < 1e-6


def test_no_eviction_is_causal_attention():
    rng = np.random.default_rng(51)
    T, G, D = 30, 2, 16
    q, k, v = _rand_bf16(rng, (T, G, D)), _rand_bf16(rng, (T, D)), _rand_bf16(rng, (T, D))
    got = orc.replay_attn(q, k, v, np.full(T, T, np.int32), 0.25)
    for g in range(G):
        x = _f(q[:, g]) @ _f(k).T * 0.25
        x[np.triu_indices(T, 1)] = -np.inf
        want = softmax(x, axis=1) @ _f(v)
        assert np.abs(got[:, g] - want).max() < 1e-6
