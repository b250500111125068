"""Pins for the oracle's egocentric render (Section 3: partially observable maze).

Hand-derived crops from tests/golden/obs_crops.txt, plus invariants that hold for
any level: one-hot cells, the agent's own cell, at most one goal, and invariance
under rotating the whole world by a quarter turn.
"""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "obs_crops.txt")
CODE = {"W": (1, 0, 0), "G": (0, 1, 0), "E": (0, 0, 1)}


def parse_cases(path):
    cases, cur, cur_dir = [], None, None
    for raw in open(path):
        line = raw.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0] == "case":
            cur = {"name": tok[1], "crops": {}}
        elif tok[0] == "size":
            cur["H"], cur["W"] = int(tok[1]), int(tok[2])
        elif tok[0] == "view":
            cur["k"] = int(tok[1])
        elif tok[0] == "walls":
            cur["walls"] = [tuple(map(int, t.split(","))) for t in tok[1:]]
        elif tok[0] == "goal":
            cur["goal"] = (int(tok[1]), int(tok[2]))
        elif tok[0] == "agent":
            cur["agent"] = (int(tok[1]), int(tok[2]))
        elif tok[0] == "dir":
            cur_dir = int(tok[1])
            cur["crops"][cur_dir] = []
        elif tok[0] == "end":
            cases.append(cur)
            cur = None
        else:
            cur["crops"][cur_dir].append([CODE[c] for c in tok])
    return cases


CASES = parse_cases(GOLD)


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_hand_crops(case):
    H, W, k = case["H"], case["W"], case["k"]
    walls = np.zeros((1, H, W), np.int8)
    for (x, y) in case["walls"]:
        walls[0, y, x] = 1
    for d, crop in case["crops"].items():
        o = oracle.MazeOracle(1, H, W, k, 250)
        o.reset_to_levels(walls, np.array([case["agent"]], np.int32), np.array([d], np.int8),
                          np.array([case["goal"]], np.int32))
        want = np.array(crop, np.int8)
        assert want.shape == (k, k, 3)
        got = o.render_obs()[0]
        assert (got == want).all(), f"case {case['name']} dir {d}\n{got.argmax(-1)}\n{want.argmax(-1)}"


def _random(seed, N, H, W, k, n_walls):
    from paper_2311_12716_amd import workloads as wl
    w = wl.student_random("obs", seed, N=N, H=H, W=W, view=k, T=1, n_walls=n_walls)
    o = oracle.MazeOracle(N, H, W, k, 250)
    o.reset_to_levels(w.walls, w.agent_xy, w.agent_dir, w.goal_xy)
    return w, o


@pytest.mark.parametrize("H,W,k", [(13, 13, 5), (7, 10, 3), (9, 6, 7)])
def test_render_invariants(H, W, k):
    w, o = _random(5, 500, H, W, k, (H * W) // 3)
    obs = o.render_obs()
    assert set(np.unique(obs)) <= {0, 1}
    assert (obs.sum(-1) == 1).all()                       # one-hot
    assert (obs[:, k - 1, k // 2, 2] == 1).all()          # own cell reads empty
    assert (obs[..., 1].sum((1, 2)) <= 1).all()           # at most one goal cell
    # the goal is shown exactly when it lies inside the view rectangle
    dvec = np.array([[1, 0], [0, 1], [-1, 0], [0, -1]])
    rel = w.goal_xy - w.agent_xy
    f = (rel * dvec[w.agent_dir]).sum(1)
    s = (rel * dvec[(w.agent_dir + 1) % 4]).sum(1)
    inside = (f >= 0) & (f <= k - 1) & (np.abs(s) <= k // 2)
    assert (obs[..., 1].sum((1, 2)) == inside).all()
    n = np.nonzero(inside)[0]
    assert (obs[n, (k - 1) - f[n], s[n] + k // 2, 1] == 1).all()


def test_quarter_turn_of_the_world_leaves_the_view_unchanged():
    S, k = 11, 5
    w, o = _random(9, 300, S, S, k, 35)
    obs = o.render_obs()
    # rotate clockwise on screen (y down): (x,y) -> (S-1-y, x); headings advance by one
    walls_r = np.rot90(w.walls, k=-1, axes=(1, 2)).copy()
    rot = lambda p: np.stack([S - 1 - p[:, 1], p[:, 0]], 1).astype(np.int32)
    o2 = oracle.MazeOracle(w.N, S, S, k, 250)
    o2.reset_to_levels(walls_r, rot(w.agent_xy), (w.agent_dir + 1) % 4, rot(w.goal_xy))
    # make sure the rotation of the wall array is the one stated above
    n = np.arange(w.N)
    a2 = rot(w.agent_xy)
    assert (walls_r[n, a2[:, 1], a2[:, 0]] == w.walls[n, w.agent_xy[:, 1], w.agent_xy[:, 0]]).all()
    g2 = rot(w.goal_xy)
    assert (walls_r[n, g2[:, 1], g2[:, 0]] == 0).all()
    assert (o2.render_obs() == obs).all()


def test_view_matches_wall_lookup_cell_by_cell():
    """Every view cell against a direct lookup in a border-padded copy of the grid."""
    H, W, k = 8, 12, 5
    w, o = _random(21, 200, H, W, k, 30)
    obs = o.render_obs()
    P = k
    padded = np.ones((w.N, H + 2 * P, W + 2 * P), np.int8)
    padded[:, P:P + H, P:P + W] = w.walls
    for n in range(w.N):
        # rotate the padded map so that the agent looks up, then slice
        x, y, d = w.agent_xy[n, 0] + P, w.agent_xy[n, 1] + P, w.agent_dir[n]
        m = padded[n]
        # number of counter-clockwise quarter turns that bring heading d to "up" (3)
        turns = {3: 0, 0: 1, 1: 2, 2: 3}[int(d)]
        mr = np.rot90(m, k=turns)
        hh, ww = m.shape
        px, py = x, y
        for _ in range(turns):          # ccw quarter turn: (x,y) -> (y, ww-1-x)
            px, py, ww, hh = py, ww - 1 - px, hh, ww
        crop = mr[py - (k - 1):py + 1, px - k // 2:px + k // 2 + 1]
        assert crop.shape == (k, k)
        assert (crop == obs[n, :, :, 0]).all()
