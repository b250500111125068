"""Seeded synthetic inputs for the maze hot path.

This module only draws random inputs (levels, actions, value estimates).  It
holds none of the method's arithmetic and imports neither the HIP binding nor
the CPU oracle; both sides consume the identical numpy arrays it returns.

The paper trains on random mazes with up to ~60 wall blocks on a 13x13 interior
("randomly sampled wall, goal, and agent positions", Section 3), rollouts of
256 steps, GAE with gamma 0.995 and lambda 0.98 (hyperparameter table).  No
public dataset is involved: every workload here is generated from a seed.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class StudentWorkload:
    name: str
    N: int
    H: int
    W: int
    view: int
    max_steps: int
    T: int
    walls: np.ndarray       # int8 [N,H,W]
    agent_xy: np.ndarray    # int32 [N,2]
    agent_dir: np.ndarray   # int8 [N]
    goal_xy: np.ndarray     # int32 [N,2]
    actions: np.ndarray     # int8 [T,N] in {0,1,2}
    values: np.ndarray | None = None   # float32 [T+1,N] in [0,1)
    gamma: float = 0.995
    lam: float = 0.98
    extra: dict = field(default_factory=dict)


@dataclass
class EditorWorkload:
    name: str
    N: int
    H: int
    W: int
    n_walls: int
    T: int
    actions: np.ndarray         # int32 [T,N] in [0,H*W)
    agent_dir_init: np.ndarray  # int8 [N]


def random_levels(rng: np.random.Generator, N: int, H: int, W: int, n_walls):
    """Uniform random levels: agent, goal and walls on distinct cells.

    n_walls is an int or an int array [N] (walls per env).  One permutation of
    the H*W cells per env: entry 0 is the agent, entry 1 the goal, the next
    n_walls entries are walls.
    """
    cells = H * W
    n_walls = np.broadcast_to(np.asarray(n_walls, dtype=np.int64), (N,))
    if n_walls.max(initial=0) + 2 > cells:
        raise ValueError("too many walls for the grid")
    perm = rng.permuted(np.tile(np.arange(cells, dtype=np.int32), (N, 1)), axis=1)
    agent = perm[:, 0]
    goal = perm[:, 1]
    rank = np.arange(cells)[None, :]
    is_wall_slot = (rank >= 2) & (rank < 2 + n_walls[:, None])
    walls = np.zeros((N, cells), np.int8)
    rows = np.broadcast_to(np.arange(N)[:, None], perm.shape)
    walls[rows[is_wall_slot], perm[is_wall_slot]] = 1
    agent_xy = np.stack([agent % W, agent // W], axis=1).astype(np.int32)
    goal_xy = np.stack([goal % W, goal // W], axis=1).astype(np.int32)
    agent_dir = rng.integers(0, 4, size=N, dtype=np.int8)
    return walls.reshape(N, H, W), agent_xy, agent_dir, goal_xy


def perfect_mazes(rng: np.random.Generator, N: int, S: int):
    """N perfect mazes on an SxS interior (S odd), randomized depth-first search.

    Rooms sit on even (x,y); a passage between two adjacent rooms opens the odd
    cell between them.  All envs advance their own DFS in lock step (one push or
    pop per iteration), so the loop runs 2*rooms-1 times whatever N is.
    Returns walls int8 [N,S,S] and the (x,y) of every room [R*R,2].
    """
    if S % 2 != 1:
        raise ValueError("perfect mazes need an odd side")
    R = (S + 1) // 2
    rooms = R * R
    walls = np.ones((N, S, S), np.int8)
    visited = np.zeros((N, R, R), bool)
    stack = np.zeros((N, rooms, 2), np.int32)
    sp = np.zeros(N, np.int64)
    idx = np.arange(N)
    start = rng.integers(0, R, size=(N, 2), dtype=np.int32)
    stack[idx, 0] = start
    visited[idx, start[:, 1], start[:, 0]] = True
    walls[idx, 2 * start[:, 1], 2 * start[:, 0]] = 0
    sp[:] = 1
    dxy = np.array([[1, 0], [0, 1], [-1, 0], [0, -1]], np.int32)
    while True:
        live = sp > 0
        if not live.any():
            break
        li = idx[live]
        cur = stack[li, sp[li] - 1]                       # [L,2] room coords
        nb = cur[:, None, :] + dxy[None, :, :]            # [L,4,2]
        inside = (nb >= 0).all(-1) & (nb < R).all(-1)
        nbc = np.clip(nb, 0, R - 1)
        free = inside & ~visited[li[:, None], nbc[..., 1], nbc[..., 0]]
        nfree = free.sum(1)
        # uniformly pick one of the free neighbours (if any)
        pick_rank = (rng.random(len(li)) * np.maximum(nfree, 1)).astype(np.int64)
        order = np.cumsum(free, axis=1) - 1
        chosen = free & (order == pick_rank[:, None])
        has = nfree > 0
        k = chosen.argmax(1)
        # push
        pi = li[has]
        nxt = nb[has, k[has]]
        c = cur[has]
        visited[pi, nxt[:, 1], nxt[:, 0]] = True
        walls[pi, 2 * nxt[:, 1], 2 * nxt[:, 0]] = 0
        walls[pi, c[:, 1] + nxt[:, 1], c[:, 0] + nxt[:, 0]] = 0   # cell between = mean of 2c, 2n
        stack[pi, sp[pi]] = nxt
        sp[pi] += 1
        # pop
        sp[li[~has]] -= 1
    yy, xx = np.meshgrid(np.arange(R), np.arange(R), indexing="ij")
    room_xy = np.stack([2 * xx.ravel(), 2 * yy.ravel()], axis=1).astype(np.int32)
    return walls, room_xy


def student_random(name, seed, N, H=13, W=13, view=5, max_steps=250, T=256, n_walls=50,
                   n_walls_max=None, with_values=False):
    """Random-maze student workload (the DR-style level distribution)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if n_walls_max is not None:
        nw = rng.integers(0, n_walls_max + 1, size=N)
    else:
        nw = n_walls
    walls, agent_xy, agent_dir, goal_xy = random_levels(rng, N, H, W, nw)
    actions = rng.integers(0, 3, size=(T, N), dtype=np.int8)
    values = rng.random((T + 1, N), dtype=np.float32) if with_values else None
    return StudentWorkload(name, N, H, W, view, max_steps, T, walls, agent_xy, agent_dir, goal_xy,
                           actions, values)


def student_perfect(name, seed, N, S=51, view=7, max_steps=1000, T=512, with_values=True):
    """Perfect-maze student workload: agent and goal on two distinct rooms."""
    rng = np.random.Generator(np.random.PCG64(seed))
    walls, room_xy = perfect_mazes(rng, N, S)
    rooms = len(room_xy)
    a = rng.integers(0, rooms, size=N)
    g = (a + 1 + rng.integers(0, rooms - 1, size=N)) % rooms
    agent_xy = room_xy[a].copy()
    goal_xy = room_xy[g].copy()
    agent_dir = rng.integers(0, 4, size=N, dtype=np.int8)
    actions = rng.integers(0, 3, size=(T, N), dtype=np.int8)
    values = rng.random((T + 1, N), dtype=np.float32) if with_values else None
    return StudentWorkload(name, N, S, S, view, max_steps, T, walls, agent_xy, agent_dir, goal_xy,
                           actions, values)


def editor_random(name, seed, N, H=13, W=13, n_walls=50):
    rng = np.random.Generator(np.random.PCG64(seed))
    T = n_walls + 2
    actions = rng.integers(0, H * W, size=(T, N), dtype=np.int32)
    agent_dir_init = rng.integers(0, 4, size=N, dtype=np.int8)
    return EditorWorkload(name, N, H, W, n_walls, T, actions, agent_dir_init)


# The five benchmark configurations.  `scale` shrinks N (and only N) for quick
# CPU-side checks; the shapes, wall counts and step counts stay the real ones.
def config(i: int, N: int | None = None, T: int | None = None):
    if i == 1:
        return student_random("C1:32env-13x13-25walls-1000steps", 101, N or 32, n_walls=25,
                              T=T or 1000)
    if i == 2:
        return student_random("C2:4096env-13x13-0..60walls-256steps+gae", 202, N or 4096,
                              n_walls_max=60, T=T or 256, with_values=True)
    if i == 3:
        return student_random("C3:32768env-13x13-50walls-256steps", 303, N or 32768, n_walls=50,
                              T=T or 256)
    if i == 4:
        return editor_random("C4:editor-32768env-13x13-52steps", 404, N or 32768)
    if i == 5:
        return student_perfect("C5:8192env-51x51-perfect-512steps+gae", 505, N or 8192,
                               T=T or 512)
    raise ValueError("config index must be 1..5")
