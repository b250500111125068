"""Pins for the oracle's observation variants: occluded view and (type, colour, state)
encoding (Section 3: the maze reproduces the MiniGrid mazes of prior work)."""
import os

import numpy as np
import pytest
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import breadth_first_order

import oracle
from paper_2311_12716_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "occlusion_crops.txt")


def load_cases():
    # comment lines start with "# " (a view row may start with '#', but holds no blank)
    lines = [l.rstrip("\n") for l in open(GOLDEN) if l.strip() and not l.startswith("# ")]
    cases, i = [], 0
    while i < len(lines):
        _, name, k = lines[i].split()
        k = int(k)
        cases.append((name, k, lines[i + 1:i + 1 + k], lines[i + 1 + k:i + 1 + 2 * k]))
        i += 1 + 2 * k
    return cases


def level_from_view(k, view, heading):
    """A level whose agent, facing `heading`, sees exactly `view` (plus empty space around)."""
    S = 2 * k + 1
    walls = np.zeros((1, S, S), np.int8)
    ax = ay = k
    dx, dy = [(1, 0), (0, 1), (-1, 0), (0, -1)][heading]
    rx, ry = [(1, 0), (0, 1), (-1, 0), (0, -1)][(heading + 1) % 4]
    goal = [[0, 0]]
    for r in range(k):
        for c in range(k):
            ahead, side = k - 1 - r, c - k // 2
            x, y = ax + ahead * dx + side * rx, ay + ahead * dy + side * ry
            if view[r][c] == "#":
                walls[0, y, x] = 1
            elif view[r][c] == "G":
                goal = [[x, y]]
    o = oracle.MazeOracle(1, S, S, k, 100)
    o.reset_to_levels(walls, np.array([[ax, ay]], np.int32), np.array([heading], np.int8),
                      np.array(goal, np.int32))
    return o


@pytest.mark.parametrize("name,k,view,mask", load_cases(), ids=[c[0] for c in load_cases()])
@pytest.mark.parametrize("heading", [0, 1, 2, 3])
def test_hand_derived_masks(name, k, view, mask, heading):
    o = level_from_view(k, view, heading)
    plain = o.render_obs()[0]
    o.set_obs_mode(0, 1)
    occ = o.render_obs()[0]
    expect = np.array([[int(ch) for ch in row] for row in mask])
    assert (occ.sum(-1) == expect).all()                       # one-hot: a seen cell has one channel set
    assert (occ == plain * expect[:, :, None]).all()           # seen cells read as without occlusion


def reachable_mask(wall, k):
    """Independent statement of the rule: cells reachable from the agent's cell in the graph whose
    edges leave seen non-wall cells sideways and to the three touching cells of the next row."""
    idx = lambda r, c: r * k + c
    rows, cols = [], []
    for r in range(k):
        for c in range(k):
            if wall[r, c] and not (r == k - 1 and c == k // 2):
                continue
            for rr, cc in ((r, c - 1), (r, c + 1), (r - 1, c - 1), (r - 1, c), (r - 1, c + 1)):
                if 0 <= rr < k and 0 <= cc < k:
                    rows.append(idx(r, c)); cols.append(idx(rr, cc))
    g = csr_matrix((np.ones(len(rows)), (rows, cols)), shape=(k * k, k * k))
    order = breadth_first_order(g, idx(k - 1, k // 2), directed=True, return_predecessors=False)
    m = np.zeros(k * k, int)
    m[order] = 1
    return m.reshape(k, k)


@pytest.mark.parametrize("k", [3, 5, 7, 9])
def test_masks_against_graph_reachability(k):
    w = wl.student_random(f"occ-{k}", 40 + k, N=300, H=11, W=12, view=k, T=2, n_walls=45)
    o = oracle.MazeOracle(w.N, w.H, w.W, k, w.max_steps)
    o.reset_to_levels(w.walls, w.agent_xy, w.agent_dir, w.goal_xy)
    plain = o.render_obs()
    o.set_obs_mode(0, 1)
    occ = o.render_obs()
    hidden = 0
    for n in range(w.N):
        m = reachable_mask(plain[n, :, :, 0] == 1, k)
        assert (occ[n].sum(-1) == m).all(), n
        hidden += int((m == 0).sum())
    assert hidden > 0


def test_type_colour_state_encoding():
    w = wl.student_random("enc", 77, N=200, H=9, W=9, view=5, T=20, n_walls=25)
    o = oracle.MazeOracle(w.N, w.H, w.W, 5, w.max_steps)
    o.reset_to_levels(w.walls, w.agent_xy, w.agent_dir, w.goal_xy)
    plain = o.render_obs().astype(int)
    assert plain[..., 1].sum() > 0                             # some goals in view
    o.set_obs_mode(1, 0)
    enc = o.render_obs().astype(int)
    assert (enc[..., 0] == 2 * plain[..., 0] + 8 * plain[..., 1] + 1 * plain[..., 2]).all()
    assert (enc[..., 1] == 5 * plain[..., 0] + 1 * plain[..., 1]).all()
    assert (enc[..., 2] == 0).all()
    o.set_obs_mode(0, 1)
    occ = o.render_obs().astype(int)
    o.set_obs_mode(1, 1)
    both = o.render_obs().astype(int)
    seen = occ.sum(-1, keepdims=True)
    assert (both == enc * seen).all()                          # unseen cells are (0, 0, 0)


def test_variant_rollout_is_step_then_observe():
    w = wl.student_random("roll", 78, N=50, H=9, W=9, view=5, T=30, n_walls=25, max_steps=10)
    a = oracle.MazeOracle(w.N, w.H, w.W, 5, w.max_steps)
    b = oracle.MazeOracle(w.N, w.H, w.W, 5, w.max_steps)
    for o in (a, b):
        o.reset_to_levels(w.walls, w.agent_xy, w.agent_dir, w.goal_xy)
    a.set_obs_mode(1, 1)
    r, d, obs = a.step(w.actions, w.T)
    rb, db, _ = b.step(w.actions, w.T, want_obs=False)          # dynamics do not depend on the mode
    assert (r == rb).all() and (d == db).all()
    assert all((x == y).all() for x, y in zip(a.get_state(), b.get_state()))
    b.set_obs_mode(1, 1)
    assert (obs[-1] == b.render_obs()).all()
