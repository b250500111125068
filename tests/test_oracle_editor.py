"""Pins for the oracle's teacher design env (Section 2.2: the teacher's decision
process is an environment of its own whose final instance becomes the student's
level).  Scripted cases worked out by hand, and set-level invariants computed
from the raw action lists with Python sets.
"""
import numpy as np
import pytest

import oracle


def run(actions, H=13, W=13, n_walls=50, dirs=None):
    actions = np.asarray(actions, np.int32)
    T, N = actions.shape
    e = oracle.EditorOracle(N, H, W, n_walls)
    e.reset(np.zeros(N, np.int8) if dirs is None else dirs)
    obs, t, done = e.step(actions, T)
    return e, obs, t, done


def test_all_actions_equal():
    # one wall placed 50 times, removed by the agent, goal pushed to the next cell
    a = np.full((52, 1), 17, np.int32)
    e, obs, t, done = run(a, dirs=np.array([2], np.int8))
    lv = e.get_levels()
    assert lv.walls.sum() == 0
    assert tuple(lv.agent_xy[0]) == (17 % 13, 17 // 13) and lv.agent_dir[0] == 2
    assert tuple(lv.goal_xy[0]) == (18 % 13, 18 // 13)
    assert list(t[:, 0]) == list(range(1, 53))
    assert list(done[:, 0]) == [0] * 51 + [1]
    # observation history: wall visible from step 1 to 50, agent from 51, goal at 52
    y, x = 17 // 13, 17 % 13
    assert (obs[:50, 0, y, x] == [1, 0, 0]).all()
    assert (obs[50, 0, y, x] == [0, 0, 1]).all() and obs[50].sum() == 1
    assert (obs[51, 0, y, x] == [0, 0, 1]).all() and (obs[51, 0, y, x + 1] == [0, 1, 0]).all()
    assert obs[51].sum() == 2


def test_goal_wraps_past_the_last_cell():
    a = np.zeros((52, 1), np.int32)
    a[:50, 0] = np.arange(50) + 60
    a[50, 0] = 168
    a[51, 0] = 168
    e, obs, t, done = run(a)
    lv = e.get_levels()
    assert tuple(lv.agent_xy[0]) == (12, 12) and tuple(lv.goal_xy[0]) == (0, 0)
    assert lv.walls.sum() == 50


def test_out_of_range_actions_are_clamped():
    a = np.zeros((4, 1), np.int32)
    a[:, 0] = [-5, 10 ** 6, -1, 999]
    e, obs, t, done = run(a, H=3, W=4, n_walls=2)
    lv = e.get_levels()
    # walls at cell 0 and 11; agent at 0 clears that wall; goal at 11 clears the other
    assert lv.walls.sum() == 0
    assert tuple(lv.agent_xy[0]) == (0, 0) and tuple(lv.goal_xy[0]) == (3, 2)


def test_steps_after_the_goal_change_nothing():
    rng = np.random.default_rng(3)
    a = rng.integers(0, 12, size=(9, 5), dtype=np.int32)
    e, obs, t, done = run(a, H=3, W=4, n_walls=3)
    assert (t[4:] == 5).all() and (done[4:] == 1).all() and (done[:4] == 0).all()
    assert (obs[4:] == obs[4]).all()


@pytest.mark.parametrize("H,W,nw", [(13, 13, 50), (5, 8, 12), (9, 4, 20)])
def test_set_level_invariants_on_random_actions(H, W, nw):
    N = 400
    rng = np.random.default_rng(12)
    a = rng.integers(0, H * W, size=(nw + 2, N), dtype=np.int32)
    dirs = rng.integers(0, 4, size=N, dtype=np.int8)
    e, obs, t, done = run(a, H=H, W=W, n_walls=nw, dirs=dirs)
    lv = e.get_levels()
    for n in range(N):
        placed = set(a[:nw, n].tolist())
        agent = int(a[nw, n])
        goal = int(a[nw + 1, n])
        if goal == agent:
            goal = (goal + 1) % (H * W)
        want = placed - {agent, goal}
        got = set(np.nonzero(lv.walls[n].ravel())[0].tolist())
        assert got == want
        assert tuple(lv.agent_xy[n]) == (agent % W, agent // W)
        assert tuple(lv.goal_xy[n]) == (goal % W, goal // W)
        assert lv.agent_dir[n] == dirs[n]
    assert (lv.walls.sum((1, 2)) <= nw).all()
    # obs channels over time: walls only grow during the wall phase, one agent, one goal at the end
    assert (obs[:nw, :, :, :, 1:].sum() == 0)
    assert (np.diff(obs[:nw, :, :, :, 0].sum((2, 3)).astype(int), axis=0) >= 0).all()
    assert (obs[nw:, :, :, :, 2].sum((2, 3)) == 1).all()
    assert (obs[nw + 1, :, :, :, 1].sum((1, 2)) == 1).all()
    assert (obs[nw + 1].sum(-1) <= 1).all()          # never two things in one cell
    assert (obs[-1, :, :, :, 0] == lv.walls).all()


def test_designed_levels_are_valid_student_levels():
    H, W, nw, N = 13, 13, 50, 300
    rng = np.random.default_rng(5)
    a = rng.integers(0, H * W, size=(nw + 2, N), dtype=np.int32)
    e, *_ = run(a)
    lv = e.get_levels()
    m = oracle.MazeOracle(N, H, W, 5, 250)
    m.reset_to_levels(lv.walls, lv.agent_xy, lv.agent_dir, lv.goal_xy)
    back = m.get_levels()
    assert (back.walls == lv.walls).all() and (back.agent_xy == lv.agent_xy).all()
    assert (back.goal_xy == lv.goal_xy).all() and (back.agent_dir == lv.agent_dir).all()
    n = np.arange(N)
    assert (lv.walls[n, lv.agent_xy[:, 1], lv.agent_xy[:, 0]] == 0).all()
    assert (lv.walls[n, lv.goal_xy[:, 1], lv.goal_xy[:, 0]] == 0).all()
    assert (lv.agent_xy != lv.goal_xy).any(1).all()
