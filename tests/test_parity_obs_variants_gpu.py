"""GPU parity of the observation variants (occluded view, type/colour/state encoding)
against the oracle, byte for byte, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_12716_amd import binding, workloads as wl
from parity_util import (DEV, assert_rollout_equal, assert_state_equal, cpu_student, gpu_student, note,
                         to_gpu)

pytestmark = pytest.mark.gpu
MODES = [(0, 1), (1, 0), (1, 1)]


def run_variant(w, encoding, occlusion):
    note(f"obs variant enc={encoding} occ={occlusion} {w.name}: N={w.N} {w.H}x{w.W} k={w.view}")
    env, o = gpu_student(w), cpu_student(w)
    env.set_obs_mode(encoding, occlusion)
    o.set_obs_mode(encoding, occlusion)
    assert (env.render_obs().cpu().numpy() == o.render_obs()).all(), "initial observation differs"
    out = env.step(to_gpu(w.actions))
    torch.cuda.synchronize()
    ref = o.step(w.actions, w.T)
    assert_rollout_equal(out, ref, w.name)
    assert_state_equal(env, o)
    return env, o


@pytest.mark.parametrize("encoding,occlusion", MODES)
def test_config_2_full_size(encoding, occlusion):
    run_variant(wl.config(2, T=64), encoding, occlusion)


@pytest.mark.parametrize("encoding,occlusion", MODES)
def test_config_3_sampled_steps(encoding, occlusion):
    # full batch of config 3, a short rollout: the oracle renders every step
    run_variant(wl.config(3, T=6), encoding, occlusion)


@pytest.mark.parametrize("encoding,occlusion", MODES)
def test_config_3_full_size_full_rollout(encoding, occlusion):
    """The launch bench.py times for the variant rows: 32768 envs x 256 steps, i.e. the kernels with
    128 (typed bytes alone), 64 (occluded with typed bytes) and 32 (occluded alone) envs per workgroup
    through 32 full blocks of 8 steps, the double-buffered stage buffers and 16 refills of the action ring; every byte compared."""
    run_variant(wl.config(3), encoding, occlusion)


@pytest.mark.parametrize("T", [7, 8, 9, 16, 17, 33])
@pytest.mark.parametrize("encoding,occlusion", MODES)
def test_64_env_workgroups_around_block_boundaries(encoding, occlusion, T):
    # 16384 envs: 64 envs per workgroup with typed bytes, 32 for the occluded view alone; rollout
    # lengths around the 8-step blocks
    # and the action ring's 16- and 32-step refills; short episodes so that resets are frequent
    w = wl.student_random(f"variant-16384-T{T}", 1000 + T, N=16384, T=T, n_walls=50, max_steps=11)
    run_variant(w, encoding, occlusion)


@pytest.mark.parametrize("N,T", [(4096 + 96, 9), (4096 + 96, 40), (8192, 17), (4096, 8), (4096, 70), (48, 131)])
@pytest.mark.parametrize("encoding,occlusion", MODES)
def test_small_workgroups_around_block_boundaries(encoding, occlusion, N, T):
    # more than 4096 envs: 32 envs per workgroup (views and records take two steps per pass);
    # up to 4096: 16 per workgroup (four steps per pass, action ring refilled every 64 steps)
    w = wl.student_random(f"variant-{N}-T{T}", 1500 + N + T, N=N, T=T, n_walls=50, max_steps=11)
    run_variant(w, encoding, occlusion)


@pytest.mark.parametrize("T", [8, 17, 41])
@pytest.mark.parametrize("encoding,occlusion", MODES)
def test_largest_workgroups_around_block_boundaries(encoding, occlusion, T):
    # 32768 envs: 128 envs per workgroup (two dynamics waves) for typed bytes alone, 64 with occlusion
    # and typed bytes, 32 with occlusion alone
    w = wl.student_random(f"variant-32768-T{T}", 2000 + T, N=32768, T=T, n_walls=40, max_steps=9)
    run_variant(w, encoding, occlusion)


def test_large_workgroups_with_a_ragged_tail_and_two_calls():
    # 32768 + 64 + 7 envs: the large workgroups, then one launch of 32-env workgroups whose last
    # one is partly filled; the rollout split into two calls (the state carries over)
    w = wl.student_random("variant-ragged", 77, N=32768 + 64 + 7, T=26, n_walls=50, max_steps=15)
    for enc, occ in MODES:
        note(f"ragged two-call enc={enc} occ={occ}")
        env, o = gpu_student(w), cpu_student(w)
        env.set_obs_mode(enc, occ)
        o.set_obs_mode(enc, occ)
        acts = to_gpu(w.actions)
        for t0, t1 in ((0, 10), (10, 26)):
            out = env.step(acts[t0:t1].contiguous())
            assert_rollout_equal(out, o.step(w.actions[t0:t1], t1 - t0), f"steps {t0}..{t1}")
        assert_state_equal(env, o)


@pytest.mark.parametrize("encoding,occlusion", MODES)
def test_perfect_mazes_view_7(encoding, occlusion):
    run_variant(wl.config(5, N=512, T=40), encoding, occlusion)


@pytest.mark.parametrize("H,W,k,nw", [(13, 13, 3, 30), (7, 19, 5, 40), (20, 9, 7, 50), (30, 30, 9, 200),
                                      (1, 6, 3, 2), (40, 12, 5, 100)])
def test_other_shapes(H, W, k, nw):
    # 272 envs: 256 in the tiled kernel (when k is 3, 5 or 7), 16 in the per-cell kernel
    w = wl.student_random(f"variant-{H}x{W}-k{k}", 3 * H + W + k, N=272, H=H, W=W, view=k, T=30,
                          n_walls=nw, max_steps=12)
    for enc, occ in MODES:
        run_variant(w, enc, occ)


@pytest.mark.parametrize("encoding,occlusion", MODES)
def test_single_steps_in_a_policy_loop(encoding, occlusion):
    w = wl.config(2, T=24)
    env, o = gpu_student(w), cpu_student(w)
    env.set_obs_mode(encoding, occlusion)
    o.set_obs_mode(encoding, occlusion)
    acts = to_gpu(w.actions)
    for t in range(w.T):
        out = env.step(acts[t:t + 1])
        assert_rollout_equal(out, o.step(w.actions[t:t + 1], 1), f"step {t}")
    assert (env.render_obs().cpu().numpy() == o.render_obs()).all()
    assert_state_equal(env, o)


def test_levels_outside_the_preconditions():
    w = wl.student_random("variant-odd", 97, N=384, H=13, W=13, view=5, T=40, n_walls=55, max_steps=20)
    n = np.arange(w.N)
    third = w.N // 3
    w.walls[n[:third], w.goal_xy[:third, 1], w.goal_xy[:third, 0]] = 1
    w.walls[n[third:2 * third], w.agent_xy[third:2 * third, 1], w.agent_xy[third:2 * third, 0]] = 1
    w.goal_xy[2 * third:] = w.agent_xy[2 * third:]
    for enc, occ in MODES:
        run_variant(w, enc, occ)


def test_switching_back_restores_the_default():
    w = wl.config(2, T=16)
    env, o = run_variant(w, 1, 1)
    env.set_obs_mode(0, 0)
    o.set_obs_mode(0, 0)
    assert (env.render_obs().cpu().numpy() == o.render_obs()).all()
    out = env.step(to_gpu(w.actions))
    assert_rollout_equal(out, o.step(w.actions, w.T), "default again")
    with pytest.raises(binding.MazeError):
        env.set_obs_mode(2, 0)
    with pytest.raises(binding.MazeError):
        env.set_obs_mode(0, -1)
