"""Pins for the oracle's level metrics (wall count, shortest path length).

The metrics are what Section 2.2 (per-level metrics, e.g. number of walls) and
Section 3 (shortest paths, by a matrix-based all-pairs algorithm) describe.  The
breadth-first search of the oracle is pinned against closed forms, against the
matrix recursion the paper names (written separately in the oracle), and against
scipy's graph routines.
"""
import numpy as np
import pytest
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import shortest_path

import oracle
from paper_2311_12716_amd import workloads as wl


def _xy(pairs):
    return np.asarray(pairs, np.int32).reshape(-1, 2)


def test_empty_grid_is_manhattan_distance():
    rng = np.random.default_rng(5)
    H, W, N = 9, 14, 200
    walls = np.zeros((N, H, W), np.int8)
    a = np.stack([rng.integers(0, W, N), rng.integers(0, H, N)], 1).astype(np.int32)
    g = np.stack([rng.integers(0, W, N), rng.integers(0, H, N)], 1).astype(np.int32)
    nw, pl = oracle.level_metrics(walls, a, g)
    assert (nw == 0).all()
    assert (pl == np.abs(a - g).sum(1)).all()


def test_serpentine_corridor_length():
    # rows 1, 3, 5, ... are walls except for one gap that alternates between the right
    # and the left end: the only route snakes through every free row
    H, W = 9, 7
    walls = np.zeros((1, H, W), np.int8)
    for y in range(1, H, 2):
        walls[0, y, :] = 1
        walls[0, y, W - 1 if (y // 2) % 2 == 0 else 0] = 0
    free_rows = (H + 1) // 2
    expect = free_rows * (W - 1) + 2 * (free_rows - 1)      # along each row + through each gap
    end_x = W - 1 if free_rows % 2 == 1 else 0
    nw, pl = oracle.level_metrics(walls, _xy([[0, 0]]), _xy([[end_x, H - 1]]))
    assert nw[0] == (H // 2) * (W - 1)
    assert pl[0] == expect


def test_degenerate_cases():
    H, W = 5, 5
    walls = np.zeros((4, H, W), np.int8)
    a = _xy([[2, 2], [0, 0], [0, 0], [1, 1]])
    g = _xy([[2, 2], [4, 4], [4, 4], [3, 3]])
    walls[1, 3, 4] = walls[1, 4, 3] = 1          # goal walled in
    walls[2, 0, 0] = 1                           # start cell is a wall
    walls[3, 3, 3] = 1                           # goal cell is a wall
    nw, pl = oracle.level_metrics(walls, a, g)
    assert pl.tolist() == [0, -1, -1, -1]
    assert nw.tolist() == [0, 2, 1, 1]


def _grid_graph(w):
    """Adjacency (dense 0/1) over all cells of one level; wall cells are isolated."""
    H, W = w.shape
    A = np.zeros((H * W, H * W), np.int64)
    for y in range(H):
        for x in range(W):
            if w[y, x]:
                continue
            for dx, dy in ((1, 0), (0, 1)):
                nx, ny = x + dx, y + dy
                if nx < W and ny < H and not w[ny, nx]:
                    A[y * W + x, ny * W + nx] = A[ny * W + nx, y * W + x] = 1
    return A


@pytest.mark.parametrize("H,W,seed", [(7, 7, 1), (6, 9, 2), (13, 13, 3)])
def test_random_levels_against_scipy(H, W, seed):
    w = wl.student_random("m", seed, 40, H, W, 5, 50, 4, n_walls=int(0.4 * H * W))
    nw, pl = oracle.level_metrics(w.walls, w.agent_xy, w.goal_xy)
    assert (nw == (w.walls != 0).reshape(40, -1).sum(1)).all()
    seen_unreachable = False
    for n in range(40):
        A = _grid_graph(w.walls[n])
        D = shortest_path(csr_matrix(A), method="D", unweighted=True)
        s = w.agent_xy[n, 1] * W + w.agent_xy[n, 0]
        t = w.goal_xy[n, 1] * W + w.goal_xy[n, 0]
        expect = -1 if np.isinf(D[s, t]) else int(D[s, t])
        seen_unreachable |= expect < 0
        assert pl[n] == expect, n
    assert seen_unreachable                   # the dense random levels include walled-off goals


def test_matrix_recursion_agrees_on_perfect_mazes():
    # a perfect maze is connected, which the matrix recursion needs
    w = wl.student_perfect("m", 9, 6, S=9, view=5, max_steps=100, T=4, with_values=False)
    N, H, W = w.walls.shape
    _, pl = oracle.level_metrics(w.walls, w.agent_xy, w.goal_xy)
    for n in range(N):
        free = np.flatnonzero(w.walls[n].reshape(-1) == 0)
        A = _grid_graph(w.walls[n])[np.ix_(free, free)]
        D = oracle.apsp_seidel(A)
        ref = shortest_path(csr_matrix(A), method="D", unweighted=True)
        assert (D == ref).all()
        idx = {c: i for i, c in enumerate(free)}
        s = idx[w.agent_xy[n, 1] * W + w.agent_xy[n, 0]]
        t = idx[w.goal_xy[n, 1] * W + w.goal_xy[n, 0]]
        assert pl[n] == D[s, t]


def test_matrix_recursion_on_cycle_and_star():
    V = 9
    C = np.zeros((V, V), np.int64)
    for i in range(V):
        C[i, (i + 1) % V] = C[(i + 1) % V, i] = 1
    D = oracle.apsp_seidel(C)
    i, j = np.indices((V, V))
    assert (D == np.minimum((i - j) % V, (j - i) % V)).all()
    S = np.zeros((V, V), np.int64)
    S[0, 1:] = S[1:, 0] = 1
    D = oracle.apsp_seidel(S)
    expect = 2 * (1 - np.eye(V, dtype=np.int64))
    expect[0, 1:] = expect[1:, 0] = 1
    assert (D == expect).all()


def test_path_length_bounds_the_rollout():
    # an agent cannot reach the goal in fewer steps than the path length (turns only add)
    w = wl.student_random("m", 11, 64, 9, 9, 5, 60, 60, n_walls=16)
    _, pl = oracle.level_metrics(w.walls, w.agent_xy, w.goal_xy)
    env = oracle.MazeOracle(64, 9, 9, 5, 60)
    env.reset_to_levels(w.walls, w.agent_xy, w.agent_dir, w.goal_xy)
    reward, done, _ = env.step(w.actions, n_steps=60, want_obs=False)
    first = np.where(reward > 0, np.arange(1, 61)[:, None], 10 ** 6).min(0)
    reached = first < 10 ** 6
    assert (pl[reached] >= 0).all()
    assert (first[reached] >= pl[reached]).all()
    assert not (reward[:, pl < 0] > 0).any()
