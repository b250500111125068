"""Pins for the oracle's GAE (PPO with generalised advantage estimation, the
paper's appendix on hyperparameters: gamma in {0.995, 0.999}, lambda in
{0.95, 0.98}).  Closed forms, limiting cases, and the explicit double sum
A_t = sum_k (gamma*lambda)^k delta_{t+k} cut at episode ends.
"""
import numpy as np
import pytest

import oracle


def test_constant_reward_and_value_closed_form():
    T, N, g, l = 256, 3, 0.995, 0.98
    r = np.full((T, N), 0.25, np.float32)
    V = np.full((T + 1, N), 0.5, np.float32)
    d = np.zeros((T, N), np.uint8)
    adv, ret = oracle.compute_gae(r, V, d, g, l)
    delta = 0.25 + (g - 1.0) * 0.5
    t = np.arange(T)
    want = delta * (1 - (g * l) ** (T - t)) / (1 - g * l)
    assert np.allclose(adv, want[:, None], rtol=1e-12, atol=1e-13)
    assert np.allclose(ret, adv + 0.5, rtol=0, atol=1e-15)


def _rand(T, N, seed, p_done=0.05):
    rng = np.random.default_rng(seed)
    r = rng.random((T, N), dtype=np.float32)
    V = rng.random((T + 1, N), dtype=np.float32)
    d = (rng.random((T, N)) < p_done).astype(np.uint8)
    return r, V, d


def test_lambda_zero_is_the_td_error():
    r, V, d = _rand(40, 7, 1)
    adv, _ = oracle.compute_gae(r, V, d, 0.99, 0.0)
    nd = 1.0 - d
    want = r.astype(np.float64) + 0.99 * V[1:].astype(np.float64) * nd - V[:-1].astype(np.float64)
    assert np.allclose(adv, want, rtol=0, atol=1e-15)


def test_lambda_one_is_the_discounted_return_minus_value():
    T, N, g = 30, 4, 0.9
    r, V, d = _rand(T, N, 2, p_done=0.0)
    adv, ret = oracle.compute_gae(r, V, d, g, 1.0)
    r, V = r.astype(np.float64), V.astype(np.float64)
    for t in range(T):
        G = sum(g ** k * r[t + k] for k in range(T - t)) + g ** (T - t) * V[T]
        assert np.allclose(adv[t], G - V[t], rtol=0, atol=1e-13)
        assert np.allclose(ret[t], G, rtol=0, atol=1e-13)


def test_all_done_gives_reward_minus_value():
    r, V, _ = _rand(20, 5, 3)
    d = np.ones((20, 5), np.uint8)
    adv, ret = oracle.compute_gae(r, V, d, 0.995, 0.98)
    assert np.allclose(adv, r.astype(np.float64) - V[:-1].astype(np.float64), rtol=0, atol=1e-15)
    assert np.allclose(ret, r.astype(np.float64), rtol=0, atol=1e-15)


@pytest.mark.parametrize("g,l", [(0.995, 0.98), (0.999, 0.95)])
def test_explicit_double_sum_with_episode_cuts(g, l):
    T, N = 64, 6
    r, V, d = _rand(T, N, 4, p_done=0.1)
    adv, _ = oracle.compute_gae(r, V, d, g, l)
    r64, V64 = r.astype(np.float64), V.astype(np.float64)
    for n in range(N):
        delta = [r64[t, n] + (0.0 if d[t, n] else g * V64[t + 1, n]) - V64[t, n] for t in range(T)]
        for t in range(T):
            acc, w = 0.0, 1.0
            for k in range(t, T):
                acc += w * delta[k]
                if d[k, n]:
                    break                 # nothing beyond an episode end leaks back
                w *= g * l
            assert abs(adv[t, n] - acc) < 1e-12


def test_a_done_in_the_middle_decouples_the_two_halves():
    T, N = 50, 3
    r, V, d = _rand(T, N, 6, p_done=0.0)
    d[24] = 1
    adv, _ = oracle.compute_gae(r, V, d, 0.995, 0.98)
    r2, V2 = r.copy(), V.copy()
    r2[25:] += 1.0                         # change everything after the cut
    V2[25:] *= 0.5
    adv2, _ = oracle.compute_gae(r2, V2, d, 0.995, 0.98)
    assert (adv[:25] == adv2[:25]).all()
    assert not np.allclose(adv[25:], adv2[25:])


@pytest.mark.parametrize("reward,peak", [(0.5, 20.0), (1.0, 40.0)])
def test_dense_rewards_reach_the_geometric_limit(reward, peak):
    """Dense rewards, no episode ends, V = 0: A_t = r (1 - (gamma lambda)^(T-t)) / (1 - gamma lambda),
    which climbs to r / (1 - 0.995 * 0.98) = 40.16 r -- the largest magnitudes the recurrence
    produces with the paper's gamma and lambda."""
    T, N, g, l = 512, 2, 0.995, 0.98
    r = np.full((T, N), reward, np.float32)
    V = np.zeros((T + 1, N), np.float32)
    d = np.zeros((T, N), np.uint8)
    adv, ret = oracle.compute_gae(r, V, d, g, l)
    gl = g * l
    want = reward * (1 - gl ** (T - np.arange(T))) / (1 - gl)
    assert np.allclose(adv, want[:, None], rtol=1e-12, atol=0)
    assert (ret == adv).all()
    assert peak < adv.max() < 1.01 * peak * 1.004 + 0.2
