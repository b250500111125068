"""Pins for the oracle's replay distribution (appendix: PLR prioritization, temperature,
staleness coefficient)."""
import numpy as np
import pytest

import oracle


def test_hand_worked_rank_case():
    # scores 0.2, 0.9, 0.5 -> ranks 3, 1, 2; beta = 0.5 -> weights (1/3)^2, 1, (1/2)^2
    p = oracle.replay_distribution([0.2, 0.9, 0.5], [10, 10, 10], now=10, rank=True,
                                   temperature=0.5, staleness_coef=0.3)
    w = np.array([1 / 9, 1.0, 1 / 4])
    assert np.allclose(p, w / w.sum(), rtol=1e-15)          # every level just seen: scores only
    # staleness 4, 0, 6 -> P_C = .4, 0, .6 ; rho = 0.3
    p = oracle.replay_distribution([0.2, 0.9, 0.5], [6, 10, 4], now=10, rank=True,
                                   temperature=0.5, staleness_coef=0.3)
    assert np.allclose(p, 0.7 * w / w.sum() + 0.3 * np.array([0.4, 0.0, 0.6]), rtol=1e-15)


def test_proportional_case_and_degenerate_sums():
    p = oracle.replay_distribution([1.0, 3.0, -2.0, 0.0], [0, 0, 0, 0], now=0, rank=False,
                                   temperature=1.0, staleness_coef=0.5)
    assert np.allclose(p, [0.25, 0.75, 0.0, 0.0])
    p = oracle.replay_distribution([4.0, 1.0], [0, 0], now=0, rank=False, temperature=0.5,
                                   staleness_coef=0.0)
    assert np.allclose(p, [16 / 17, 1 / 17])
    p = oracle.replay_distribution([0.0, -1.0, 0.0], [5, 5, 5], now=5, rank=False, temperature=0.3,
                                   staleness_coef=0.3)
    assert np.allclose(p, 1 / 3)                             # no positive score: uniform
    p = oracle.replay_distribution([0.0, -1.0, 0.0], [5, 1, 3], now=5, rank=False, temperature=0.3,
                                   staleness_coef=1.0)
    assert np.allclose(p, [0.0, 4 / 6, 2 / 6])               # staleness only


def test_ranks_by_counting():
    rng = np.random.default_rng(0)
    for K in (1, 2, 17, 64):
        s = rng.integers(0, 6, K).astype(np.float32)          # many ties
        p = oracle.replay_distribution(s, np.zeros(K, np.int32), 0, True, 1.0, 0.0)
        ranks = np.array([1 + sum(1 for j in range(K) if s[j] > s[i] or (s[j] == s[i] and j < i))
                          for i in range(K)])
        h = 1.0 / ranks
        assert np.allclose(p, h / h.sum(), rtol=1e-14)
        assert sorted(ranks) == list(range(1, K + 1))


@pytest.mark.parametrize("rank", [True, False])
def test_invariants_at_buffer_size(rank):
    K = 4000
    rng = np.random.default_rng(1)
    s = rng.random(K).astype(np.float32)
    seen = rng.integers(0, 1000, K).astype(np.int32)
    p = oracle.replay_distribution(s, seen, 1000, rank, 0.3, 0.3)
    assert abs(p.sum() - 1.0) < 1e-12 and (p >= 0).all()
    # relabelling the levels relabels the probabilities (no ties in these scores)
    perm = rng.permutation(K)
    q = oracle.replay_distribution(s[perm], seen[perm], 1000, rank, 0.3, 0.3)
    assert np.allclose(q, p[perm], rtol=1e-12)
    # score part is monotone in the score; a lower temperature sharpens it
    ps = oracle.replay_distribution(s, seen, 1000, rank, 0.3, 0.0)
    order = np.argsort(s)
    assert (np.diff(ps[order]) >= 0).all()
    sharp = oracle.replay_distribution(s, seen, 1000, rank, 0.1, 0.0)
    assert sharp.max() > ps.max()
    # staleness part is linear in the age
    pc = oracle.replay_distribution(s, seen, 1000, rank, 0.3, 1.0)
    assert np.allclose(pc, (1000 - seen) / (1000 - seen).sum(), rtol=1e-12)
    mix = oracle.replay_distribution(s, seen, 1000, rank, 0.3, 0.3)
    assert np.allclose(mix, 0.7 * ps + 0.3 * pc, rtol=1e-12)
