"""CPU oracle for the batched maze hot path -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``maze_oracle.c`` (plain C, one env at a time,
byte-per-cell grids, rewards and GAE in double).  Only the tests, the smoke
check and the ``cpu_baseline`` leg of the benchmark may import this package;
the product (the HIP library and its binding) never does, and this package
imports nothing of the product.

The C file is compiled with gcc into ``liboracle.so`` next to it (``build()``);
if the library is missing it is built on first use.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "maze_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile maze_oracle.c with gcc (no contraction, IEEE arithmetic)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", tmp, _SRC]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def _p(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _req(a, dtype, shape=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_num_threads(n: int) -> None:
    _load().orc_set_num_threads(ctypes.c_int(int(n)))


@dataclass
class Levels:
    """A batch of levels: the free parameters of the maze (Section 2.2)."""
    walls: np.ndarray      # int8 [N,H,W], 1 = wall
    agent_xy: np.ndarray   # int32 [N,2] start (x,y)
    agent_dir: np.ndarray  # int8 [N] start heading 0..3
    goal_xy: np.ndarray    # int32 [N,2]


class MazeOracle:
    """Batched student maze: reset to given levels, step, render."""

    def __init__(self, N: int, H: int, W: int, view: int, max_steps: int):
        if view % 2 != 1:
            raise ValueError("view must be odd")
        self.N, self.H, self.W, self.view, self.max_steps = N, H, W, view, max_steps
        self.levels: Levels | None = None
        self.encoding, self.occlusion = 0, 0

    def set_obs_mode(self, encoding: int, occlusion: int) -> None:
        """encoding 0 = one-hot (wall, goal, empty), 1 = (type, colour, state); occlusion
        0 = the whole window, 1 = cells behind walls are unseen (Section 3, MiniGrid-based)."""
        if self.view > 31:
            raise ValueError("view too large for the variants")
        self.encoding, self.occlusion = int(encoding), int(occlusion)

    def reset_to_levels(self, walls, agent_xy, agent_dir, goal_xy) -> None:
        N, H, W = self.N, self.H, self.W
        self.levels = Levels(_req(walls, np.int8, (N, H, W)).copy(),
                             _req(agent_xy, np.int32, (N, 2)).copy(),
                             _req(agent_dir, np.int8, (N,)).copy(),
                             _req(goal_xy, np.int32, (N, 2)).copy())
        self.xy = self.levels.agent_xy.copy()
        self.dir = self.levels.agent_dir.copy()
        self.t = np.zeros(N, np.int32)

    def render_obs(self) -> np.ndarray:
        L, k = self.levels, self.view
        obs = np.empty((self.N, k, k, 3), np.int8)
        if self.encoding or self.occlusion:
            _load().orc_maze_render_variant(self.N, self.H, self.W, k, self.encoding, self.occlusion,
                                            _p(L.walls), _p(L.goal_xy), _p(self.xy), _p(self.dir),
                                            _p(obs))
        else:
            _load().orc_maze_render(self.N, self.H, self.W, k, _p(L.walls), _p(L.goal_xy),
                                    _p(self.xy), _p(self.dir), _p(obs))
        return obs

    def step(self, actions, n_steps: int = 1, want_obs: bool = True):
        """actions int8 [n_steps,N] -> reward f32, done u8 [n_steps,N], obs or None."""
        L, k, N = self.levels, self.view, self.N
        actions = _req(actions, np.int8, (n_steps, N))
        reward = np.empty((n_steps, N), np.float32)
        done = np.empty((n_steps, N), np.uint8)
        obs = np.empty((n_steps, N, k, k, 3), np.int8) if want_obs else None

        def rollout(first, count, obs_out):
            _load().orc_maze_rollout(N, self.H, self.W, k, self.max_steps, count,
                                     _p(L.walls), _p(L.agent_xy), _p(L.agent_dir), _p(L.goal_xy),
                                     _p(self.xy), _p(self.dir), _p(self.t),
                                     _p(actions[first:first + count]), _p(reward[first:first + count]),
                                     _p(done[first:first + count]), _p(obs_out))

        if want_obs and (self.encoding or self.occlusion):
            for s in range(n_steps):              # step, then observe in the chosen variant
                rollout(s, 1, None)
                obs[s] = self.render_obs()
        else:
            rollout(0, n_steps, obs)
        return reward, done, obs

    def get_state(self):
        return self.xy.copy(), self.dir.copy(), self.t.copy()

    def set_state(self, xy=None, direction=None, t=None) -> None:
        """The setter that goes with get_state (Section 2.2: env state getter and setter):
        overwrite position, heading and the episode's step count; the levels stay.  Positions
        are clamped into the interior, headings taken mod 4, step counts clamped to
        [0, max_steps - 1]; a part passed as None is kept."""
        if xy is not None:
            xy = _req(xy, np.int32, (self.N, 2))
            self.xy = np.stack([np.clip(xy[:, 0], 0, self.W - 1), np.clip(xy[:, 1], 0, self.H - 1)],
                               axis=1).astype(np.int32)
        if direction is not None:
            self.dir = (_req(direction, np.int8, (self.N,)).astype(np.int32) & 3).astype(np.int8)
        if t is not None:
            self.t = np.clip(_req(t, np.int32, (self.N,)), 0, self.max_steps - 1).astype(np.int32)

    def get_levels(self) -> Levels:
        L = self.levels
        return Levels(L.walls.copy(), L.agent_xy.copy(), L.agent_dir.copy(), L.goal_xy.copy())


class EditorOracle:
    """Batched teacher design env: n_walls walls, then agent, then goal."""

    def __init__(self, N: int, H: int, W: int, n_walls: int):
        self.N, self.H, self.W, self.n_walls = N, H, W, n_walls

    def reset(self, agent_dir_init) -> None:
        N, H, W = self.N, self.H, self.W
        self.dir_init = _req(agent_dir_init, np.int8, (N,)).copy()
        self.walls = np.empty((N, H, W), np.int8)
        self.agent_xy = np.empty((N, 2), np.int32)
        self.agent_dir = np.empty(N, np.int8)
        self.goal_xy = np.empty((N, 2), np.int32)
        self.t = np.empty(N, np.int32)
        _load().orc_editor_reset(N, H, W, _p(self.walls), _p(self.agent_xy), _p(self.agent_dir),
                                 _p(self.goal_xy), _p(self.t))

    def step(self, actions, n_steps: int = 1, want_obs: bool = True):
        """actions int32 [n_steps,N] -> obs i8 [n_steps,N,H,W,3] (or None), t i32, done u8."""
        N, H, W = self.N, self.H, self.W
        actions = _req(actions, np.int32, (n_steps, N))
        obs = np.empty((n_steps, N, H, W, 3), np.int8) if want_obs else None
        t_out = np.empty((n_steps, N), np.int32)
        done = np.empty((n_steps, N), np.uint8)
        _load().orc_editor_rollout(N, H, W, self.n_walls, n_steps, _p(self.dir_init),
                                   _p(self.walls), _p(self.agent_xy), _p(self.agent_dir),
                                   _p(self.goal_xy), _p(self.t), _p(actions),
                                   _p(obs), _p(t_out), _p(done))
        return obs, t_out, done

    def get_levels(self) -> Levels:
        return Levels(self.walls.copy(), self.agent_xy.copy(), self.agent_dir.copy(),
                      self.goal_xy.copy())

    def set_levels(self, walls, agent_xy, agent_dir, goal_xy) -> None:
        """Load finished levels (Section 2.2: setter of the free parameters); coordinates
        are clamped into the interior, everything else is copied as it is."""
        N, H, W = self.N, self.H, self.W
        self.walls = (_req(walls, np.int8, (N, H, W)) != 0).astype(np.int8)
        hi = np.array([W - 1, H - 1], np.int32)
        self.agent_xy = np.clip(_req(agent_xy, np.int32, (N, 2)), 0, hi).astype(np.int32)
        self.goal_xy = np.clip(_req(goal_xy, np.int32, (N, 2)), 0, hi).astype(np.int32)
        self.agent_dir = (_req(agent_dir, np.int8, (N,)) & 3).astype(np.int8)
        self.dir_init = self.agent_dir.copy()
        self.t = np.full(N, self.n_walls + 2, np.int32)

    def random_levels(self, seed: int, first_id: int = 0) -> None:
        """Replace all levels by levels first_id .. first_id+N-1 of the random generator."""
        N, H, W = self.N, self.H, self.W
        self.walls = np.empty((N, H, W), np.int8)
        self.agent_xy = np.empty((N, 2), np.int32)
        self.agent_dir = np.empty(N, np.int8)
        self.goal_xy = np.empty((N, 2), np.int32)
        self.t = np.empty(N, np.int32)
        self.dir_init = np.empty(N, np.int8)
        _load().orc_editor_random_levels(
            N, H, W, self.n_walls, ctypes.c_uint64(seed), ctypes.c_uint64(first_id), _p(self.walls),
            _p(self.agent_xy), _p(self.agent_dir), _p(self.goal_xy), _p(self.t), _p(self.dir_init))

    def mutate(self, seed: int, first_id: int, n_edits: int) -> None:
        """n_edits random wall flips per level (cells of the agent and the goal are skipped)."""
        _load().orc_editor_mutate(self.N, self.H, self.W, ctypes.c_uint64(seed),
                                  ctypes.c_uint64(first_id), int(n_edits), _p(self.walls),
                                  _p(self.agent_xy), _p(self.goal_xy))


def philox4x32(counter, key) -> np.ndarray:
    """One block of the counter-based generator: 4 counter words, 2 key words -> 4 words."""
    c = np.asarray(counter, np.uint32).copy()
    k = np.asarray(key, np.uint32).copy()
    out = np.empty(4, np.uint32)
    _load().orc_philox4x32(_p(c), _p(k), _p(out))
    return out


def level_draw(seed: int, level_id: int, purpose: int, index: int) -> int:
    f = _load().orc_level_draw
    f.restype = ctypes.c_uint32
    return int(f(ctypes.c_uint64(seed), ctypes.c_uint64(level_id), ctypes.c_uint32(purpose),
                 ctypes.c_uint32(index)))


def draw_below(u: int, n: int) -> int:
    f = _load().orc_draw_below
    f.restype = ctypes.c_uint32
    return int(f(ctypes.c_uint32(u), ctypes.c_uint32(n)))


def compute_gae(rewards, values, dones, gamma: float, lam: float):
    """rewards f32 [T,N], values f32 [T+1,N], dones u8 [T,N] -> (adv, returns) float64 [T,N]."""
    rewards = _req(rewards, np.float32)
    T, N = rewards.shape
    values = _req(values, np.float32, (T + 1, N))
    dones = _req(dones, np.uint8, (T, N))
    adv = np.empty((T, N), np.float64)
    ret = np.empty((T, N), np.float64)
    _load().orc_gae(T, N, ctypes.c_double(gamma), ctypes.c_double(lam),
                    _p(rewards), _p(values), _p(dones), _p(adv), _p(ret))
    return adv, ret


def level_metrics(walls, agent_xy, goal_xy):
    """walls i8 [N,H,W], agent_xy / goal_xy i32 [N,2] -> (n_walls, path_len) int32 [N].

    path_len: fewest moves between 4-neighbours from the start cell to the goal cell
    (-1 if unreachable), by breadth-first search (Section 3, shortest paths).
    """
    walls = _req(walls, np.int8)
    N, H, W = walls.shape
    agent_xy = _req(agent_xy, np.int32, (N, 2))
    goal_xy = _req(goal_xy, np.int32, (N, 2))
    n_walls = np.empty(N, np.int32)
    path_len = np.empty(N, np.int32)
    scratch = np.empty((max(1, num_threads()), 2 * H * W), np.int32)
    _load().orc_level_metrics(N, H, W, _p(walls), _p(agent_xy), _p(goal_xy), _p(n_walls),
                              _p(path_len), _p(scratch))
    return n_walls, path_len


def apsp_seidel(adj: np.ndarray) -> np.ndarray:
    """All-pairs distances of a connected, undirected, unweighted graph by the
    matrix-product recursion the paper names for its shortest paths (Section 3).

    adj: [V,V] 0/1 symmetric, zero diagonal.  Returns int64 [V,V].
    The square of the graph (pairs at distance <= 2) is solved first; a distance is
    then twice the squared graph's distance, minus one when it is odd, and parity is
    read off from how the squared-graph distances of j's neighbours compare with j's.
    """
    A = np.asarray(adj, dtype=np.int64)
    V = A.shape[0]
    if V <= 1:
        return np.zeros((V, V), np.int64)
    off = ~np.eye(V, dtype=bool)
    B = (((A @ A) > 0) | (A > 0)) & off
    if B[off].all():
        return (2 * B - A) * off
    T = apsp_seidel(B.astype(np.int64))
    X = T @ A
    deg = A.sum(axis=0)
    return 2 * T - (X < T * deg[None, :])


def replay_scores(rewards, values, dones, adv, gamma: float, rmax=None):
    """Per-level replay scores of a rollout -> (rmax, maxmc, pvl) float64 [N].

    rewards, adv f32 [T,N]; values f32 [T+1,N]; dones u8 [T,N]; rmax f32 [N] = best
    return seen on each level so far, or None (Appendix: MaxMC and PVL scoring).
    """
    rewards = _req(rewards, np.float32)
    T, N = rewards.shape
    values = _req(values, np.float32, (T + 1, N))
    dones = _req(dones, np.uint8, (T, N))
    adv = _req(adv, np.float32, (T, N))
    rmax_in = None if rmax is None else _req(rmax, np.float32, (N,))
    out = [np.empty(N, np.float64) for _ in range(3)]
    _load().orc_replay_scores(T, N, ctypes.c_double(gamma), _p(rewards), _p(values), _p(dones),
                              _p(adv), _p(rmax_in), _p(out[0]), _p(out[1]), _p(out[2]))
    return tuple(out)


def replay_distribution(scores, last_seen, now: int, rank: bool, temperature: float,
                        staleness_coef: float) -> np.ndarray:
    """Probability of replaying each of the K levels of a buffer -> float64 [K].

    Appendix, hyperparameter tables: prioritization (rank or proportional), temperature
    beta, staleness coefficient rho; the paper cites prior work (prioritized level replay)
    for the formulas, which are, written out per level i:

        h_i  = 1 / rank_i            (rank 1 = highest score; ties: lower index first)
               or max(score_i, 0)    (proportional)
        P_S  = h_i^(1/beta) / sum_j h_j^(1/beta)      (uniform if the sum is 0)
        P_C  = (now - last_seen_i) / sum_j (now - last_seen_j)
        P    = (1 - rho) P_S + rho P_C                (P_S alone if every level was just seen)

    Double arithmetic; the ranks come from one stable sort.
    """
    s = np.asarray(scores, np.float32).astype(np.float64)
    c = np.asarray(last_seen, np.int32).astype(np.int64)
    K = s.shape[0]
    if rank:
        order = np.argsort(-s, kind="stable")        # highest score first, equal scores by index
        ranks = np.empty(K, np.int64)
        ranks[order] = np.arange(1, K + 1)
        h = 1.0 / ranks
    else:
        h = np.where(s > 0.0, s, 0.0)
    w = np.array([math.pow(x, 1.0 / temperature) for x in h])
    tot = math.fsum(w)
    p_s = w / tot if tot > 0.0 else np.full(K, 1.0 / K)
    stale = (int(now) - c).astype(np.float64)
    stot = math.fsum(stale)
    if stot > 0.0:
        return (1.0 - staleness_coef) * p_s + staleness_coef * (stale / stot)
    return p_s
