"""GPU parity of the replay scores (best Monte Carlo return, MaxMC, PVL) against the
oracle, within 1e-6 of the largest magnitude of each output (the oracle works in double,
the library rounds once to float32, whose spacing is 6e-8 relative), through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_12716_amd import binding, workloads as wl
from parity_util import gpu_student, note, to_gpu

pytestmark = pytest.mark.gpu
TOL = 1e-6


def check(r, v, d, a, gamma, rmax=None, what=""):
    note(f"replay scores {what} T={r.shape[0]} N={r.shape[1]} gamma={gamma} prior={rmax is not None}")
    g_rmax = None if rmax is None else to_gpu(rmax)
    out = binding.replay_scores(to_gpu(r), to_gpu(v), to_gpu(d), to_gpu(a), gamma, g_rmax)
    torch.cuda.synchronize()
    ref = oracle.replay_scores(r, v, d, a, gamma, rmax)
    for name, x, y in zip(("rmax", "maxmc", "pvl"), out, ref):
        err = np.abs(x.cpu().numpy().astype(np.float64) - y).max()
        assert err <= TOL * max(1.0, np.abs(y).max()), f"{what} {name}: error {err}"
    if rmax is not None:
        assert out[0].data_ptr() == g_rmax.data_ptr()          # updated in place


def rand_inputs(T, N, seed, p_done=0.02):
    rng = np.random.default_rng(seed)
    r = rng.random((T, N), dtype=np.float32)
    v = rng.random((T + 1, N), dtype=np.float32)
    d = (rng.random((T, N)) < p_done).astype(np.uint8)
    a = (rng.random((T, N), dtype=np.float32) - 0.5).astype(np.float32)
    return r, v, d, a


@pytest.mark.parametrize("T,N", [(1, 1), (256, 4096), (512, 8192), (33, 65), (1000, 32), (256, 32768),
                                 (16, 64), (17, 63), (257, 100)])
@pytest.mark.parametrize("gamma", [0.995, 0.9])
def test_shapes(T, N, gamma):
    r, v, d, a = rand_inputs(T, N, T + N)
    check(r, v, d, a, gamma, what="random")
    prior = (np.random.default_rng(1).random(N) * 8 - 2).astype(np.float32)
    check(r, v, d, a, gamma, rmax=prior, what="random+prior")


def test_on_a_rollout_of_the_maze():
    w = wl.config(2)
    env = gpu_student(w)
    reward, done, _ = env.step(to_gpu(w.actions), want_obs=False)
    values = np.random.default_rng(2).random((w.T + 1, w.N), dtype=np.float32)
    adv, _ = binding.compute_gae(reward, to_gpu(values), done, 0.995, 0.98)
    check(reward.cpu().numpy(), values, done.cpu().numpy(), adv.cpu().numpy(), 0.995, what="C2 rollout")


def test_degenerate_inputs():
    T, N = 40, 70
    r, v, d, a = rand_inputs(T, N, 9)
    check(-r, v, d, a, 0.99, what="negative rewards")                 # best return below zero
    check(r, v, np.ones_like(d), a, 0.99, what="every step ends an episode")
    check(r, v, np.zeros_like(d), a, 1.0, what="no discount, no ends")
    check(r, v, d, -np.abs(a), 0.99, what="no positive advantage")


def test_error_paths():
    t = torch.zeros((4, 8), device="cuda:0")
    with pytest.raises(binding.MazeError):
        binding.replay_scores(t, torch.zeros((4, 8), device="cuda:0"), t.to(torch.uint8), t, 0.99)
