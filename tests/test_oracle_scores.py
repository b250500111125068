"""Pins for the oracle's replay scores (Appendix: PLR scoring functions MaxMC and PVL)."""
import numpy as np

import oracle


def _rand(T, N, seed, p_done=0.05):
    rng = np.random.default_rng(seed)
    r = rng.random((T, N), dtype=np.float32)
    v = rng.random((T + 1, N), dtype=np.float32)
    d = (rng.random((T, N)) < p_done).astype(np.uint8)
    a = (rng.random((T, N), dtype=np.float32) - 0.5).astype(np.float32)
    return r, v, d, a


def test_constant_reward_closed_form():
    T, N, g, r0, vT = 40, 3, 0.9, 0.25, 2.0
    r = np.full((T, N), r0, np.float32)
    v = np.zeros((T + 1, N), np.float32)
    v[T] = vT
    d = np.zeros((T, N), np.uint8)
    a = np.zeros((T, N), np.float32)
    rmax, maxmc, pvl = oracle.replay_scores(r, v, d, a, g)
    G0 = r0 * (1 - g ** T) / (1 - g) + g ** T * vT            # geometric series + bootstrap
    GT1 = r0 + g * vT                                          # last step's return
    assert np.allclose(rmax, max(G0, GT1), rtol=0, atol=1e-12)
    assert np.allclose(maxmc, rmax, atol=1e-12)                # all V_t (t < T) are zero
    assert (pvl == 0).all()


def test_done_cuts_the_return_and_prior_best_counts():
    # one env, rewards 0 except a 1 at t=2 where the episode ends; values zero, bootstrap 5
    T, g = 6, 0.5
    r = np.zeros((T, 1), np.float32); r[2, 0] = 1
    d = np.zeros((T, 1), np.uint8); d[2, 0] = 1
    v = np.zeros((T + 1, 1), np.float32); v[T, 0] = 5
    a = np.array([[0.5], [-1.0], [2.0], [0.0], [-0.25], [1.5]], np.float32)
    rmax, maxmc, pvl = oracle.replay_scores(r, v, d, a, g)
    # second episode: G_5 = 0 + .5*5 = 2.5 ; first: G_2 = 1, G_1 = .5, G_0 = .25
    assert rmax[0] == 2.5
    assert pvl[0] == (0.5 + 2.0 + 1.5) / 6
    rmax, maxmc, _ = oracle.replay_scores(r, v, d, a, g, rmax=np.array([7.0], np.float32))
    assert rmax[0] == 7.0 and maxmc[0] == 7.0
    rmax, _, _ = oracle.replay_scores(r, v, d, a, g, rmax=np.array([-3.0], np.float32))
    assert rmax[0] == 2.5
    # all returns negative and no prior best: the best is the largest of them, not zero
    rmax, _, _ = oracle.replay_scores(-np.ones((T, 1), np.float32), 0 * v, d, a, g)
    assert rmax[0] == -1.0


def test_returns_agree_with_gae_at_lambda_one():
    # with lambda = 1 the GAE advantage is the Monte Carlo return minus the value
    T, N, g = 64, 50, 0.97
    r, v, d, a = _rand(T, N, 4)
    adv, ret = oracle.compute_gae(r, v, d, g, 1.0)
    rmax, maxmc, pvl = oracle.replay_scores(r, v, d, a, g)
    assert np.allclose(rmax, ret.max(axis=0), rtol=0, atol=1e-12)
    assert np.allclose(maxmc, ret.max(axis=0) - v[:T].astype(np.float64).mean(axis=0), atol=1e-12)
    assert np.allclose(pvl, np.maximum(a.astype(np.float64), 0).mean(axis=0), atol=1e-15)


def test_each_env_is_scored_on_its_own():
    T, N, g = 30, 8, 0.99
    r, v, d, a = _rand(T, N, 6)
    whole = oracle.replay_scores(r, v, d, a, g)
    for n in (0, 3, 7):
        one = oracle.replay_scores(r[:, n:n + 1], v[:, n:n + 1], d[:, n:n + 1], a[:, n:n + 1], g)
        for x, y in zip(whole, one):
            assert x[n] == y[0]
