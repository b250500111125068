"""maze_rollout_static -- the entry point for callers that cannot allocate device memory --
against maze_reset_to_levels + maze_step on an env with its own workspace (same kernels, so
every output must be identical) and against the oracle, through the C ABI.  Two calls in a
row share the library's static device array; the second is smaller, so whatever the first
left behind must not leak into it."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2311_12716_amd import binding, workloads as wl
from parity_util import DEV, assert_rollout_equal, cpu_student, gpu_student, note, to_gpu

pytestmark = pytest.mark.gpu


def static_rollout(w):
    N, T, k = w.N, w.T, w.view
    reward = torch.full((T, N), -7.0, dtype=torch.float32, device=DEV)
    done = torch.full((T, N), 9, dtype=torch.uint8, device=DEV)
    obs = torch.full((T, N, k, k, 3), 5, dtype=torch.int8, device=DEV)
    binding.maze_rollout_static(w.H, w.W, k, w.max_steps, to_gpu(w.walls), to_gpu(w.agent_xy),
                                to_gpu(w.agent_dir), to_gpu(w.goal_xy), to_gpu(w.actions), reward, done, obs)
    torch.cuda.synchronize()
    return reward, done, obs


def check(w):
    note(f"static rollout {w.name}: N={w.N} {w.H}x{w.W} k={w.view} T={w.T}")
    got = static_rollout(w)
    env = gpu_student(w)
    want = env.step(to_gpu(w.actions))
    torch.cuda.synchronize()
    for a, b, what in zip(got, want, ("reward", "done", "obs")):
        assert torch.equal(a, b), f"{what} differs from maze_reset_to_levels + maze_step"
    assert_rollout_equal(got, cpu_student(w).step(w.actions, w.T), w.name)


def test_two_calls_in_a_row_the_second_smaller():
    check(wl.student_random("static-large", 11, N=4096 + 64 + 9, T=40, n_walls=50, max_steps=25))
    check(wl.student_random("static-small", 12, N=200, H=9, W=11, view=3, T=19, n_walls=20, max_steps=7))
    # larger again, other word size (51 x 51 with view 7: 64-bit rows)
    check(wl.config(5, N=96, T=24))
    # a view size the store-layout kernels do not take
    check(wl.student_random("static-k9", 13, N=70, H=10, W=10, view=9, T=12, n_walls=30, max_steps=6))


def test_config_3_full_size_fits():
    w = wl.config(3, T=24)
    got = static_rollout(w)
    env = gpu_student(w)
    want = env.step(to_gpu(w.actions))
    for a, b in zip(got, want):
        assert torch.equal(a, b)


def test_limits_and_errors():
    lib = binding.load_library()
    n = ctypes.c_size_t(0)
    # 16 MiB of packed levels and state: 8192 perfect mazes of 51 x 51 fit, 8320 do not
    assert lib.maze_workspace_bytes(8192, 51, 51, 7, ctypes.byref(n)) == 0 and n.value <= 16 << 20
    w = wl.student_random("static-too-many", 14, N=64, T=2)
    big_n = 50000                                          # 18.2 MB of workspace at 13 x 13, view 5
    assert lib.maze_workspace_bytes(big_n, 13, 13, 5, ctypes.byref(n)) == 0 and n.value > 16 << 20
    one = torch.zeros(1, dtype=torch.int8, device=DEV).data_ptr()
    # the size check comes before any pointer is used
    assert lib.maze_rollout_static(big_n, 13, 13, 5, 250, one, one, one, one, one, 2, one, one, one, None) == -3
    assert lib.maze_rollout_static(64, 13, 13, 5, 250, None, one, one, one, one, 2, one, one, one, None) == -2
    assert lib.maze_rollout_static(64, 13, 13, 4, 250, one, one, one, one, one, 2, one, one, one, None) == -1
    assert lib.maze_rollout_static(64, 13, 13, 5, 0, one, one, one, one, one, 2, one, one, one, None) == -1
    assert lib.maze_rollout_static(64, 13, 13, 5, 250, one, one, one, one, one, 0, one, one, one, None) == -1
    # and a good call still works afterwards
    check(w)
