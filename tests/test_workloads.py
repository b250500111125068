"""Checks of the synthetic input generators (they hold no method arithmetic)."""
from collections import deque

import numpy as np

from paper_2311_12716_amd import workloads as wl


def test_random_levels_are_valid():
    w = wl.config(2, N=512)
    n = np.arange(w.N)
    assert w.walls.shape == (512, 13, 13) and w.walls.dtype == np.int8
    assert (w.walls[n, w.agent_xy[:, 1], w.agent_xy[:, 0]] == 0).all()
    assert (w.walls[n, w.goal_xy[:, 1], w.goal_xy[:, 0]] == 0).all()
    assert (w.agent_xy != w.goal_xy).any(1).all()
    cnt = w.walls.sum((1, 2))
    assert cnt.min() >= 0 and cnt.max() <= 60 and len(np.unique(cnt)) > 30
    assert set(np.unique(w.actions)) == {0, 1, 2}
    assert w.values.shape == (257, 512) and w.values.dtype == np.float32
    w3 = wl.config(3, N=64)
    assert (w3.walls.sum((1, 2)) == 50).all()
    w1 = wl.config(1)
    assert w1.N == 32 and w1.T == 1000 and (w1.walls.sum((1, 2)) == 25).all()


def test_generators_are_deterministic():
    a, b = wl.config(3, N=128), wl.config(3, N=128)
    assert (a.walls == b.walls).all() and (a.actions == b.actions).all()
    e, f = wl.config(4, N=64), wl.config(4, N=64)
    assert (e.actions == f.actions).all() and e.actions.min() >= 0 and e.actions.max() < 169
    assert e.T == 52


def test_perfect_mazes_are_spanning_trees():
    w = wl.config(5, N=16)
    assert w.H == w.W == 51 and w.view == 7 and w.max_steps == 1000 and w.T == 512
    for n in range(w.N):
        g = w.walls[n]
        assert (g == 0).sum() == 2 * 26 * 26 - 1 and (g == 1).sum() == 2601 - 1351
        # flood fill over open cells from the agent reaches every room
        seen = np.zeros_like(g, bool)
        ax, ay = w.agent_xy[n]
        q = deque([(ax, ay)])
        seen[ay, ax] = True
        while q:
            x, y = q.popleft()
            for dx, dy in ((1, 0), (-1, 0), (0, 1), (0, -1)):
                u, v = x + dx, y + dy
                if 0 <= u < 51 and 0 <= v < 51 and not g[v, u] and not seen[v, u]:
                    seen[v, u] = True
                    q.append((u, v))
        assert seen.sum() == 1351
        assert g[w.goal_xy[n, 1], w.goal_xy[n, 0]] == 0
        assert tuple(w.goal_xy[n]) != tuple(w.agent_xy[n])
        assert (w.agent_xy[n] % 2 == 0).all() and (w.goal_xy[n] % 2 == 0).all()
