"""Pins for the oracle's random level generator and level mutations.

The paper (Section 3; table of baselines; hyperparameter tables) says levels are
randomly sampled and that ACCEL mutates them, but fixes no generator: the readings are
in the oracle's header.  The generator is pinned to the published known-answer vectors
of its algorithm; everything built on it is pinned by invariants and by statistics with
wide margins.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = oracle.philox4x32(v[0:4], v[4:6])
        assert out.tolist() == v[6:10]


def test_draw_indexing():
    seed, lid = 0x0123456789ABCDEF, 0xFEDCBA9876543210
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for purpose in (0, 1):
        for block in (0, 1, 5):
            out = oracle.philox4x32([lid & 0xFFFFFFFF, lid >> 32, block, purpose], key)
            for wd in range(4):
                assert oracle.level_draw(seed, lid, purpose, 4 * block + wd) == int(out[wd])


def test_draw_below():
    assert oracle.draw_below(0, 169) == 0
    assert oracle.draw_below(0xFFFFFFFF, 169) == 168
    assert oracle.draw_below(0x80000000, 169) == 84
    assert oracle.draw_below(0x12345678, 1) == 0
    # floor(u*n / 2^32) for a few exact cases
    for u, n in [(123456789, 1000), (4000000000, 2601), (65536, 65536)]:
        assert oracle.draw_below(u, n) == (u * n) >> 32
    prev = -1
    for u in range(0, 1 << 32, 1 << 24):
        v = oracle.draw_below(u, 50)
        assert v >= prev
        prev = v


def _levels(N, H, W, n_walls, seed, first_id=0):
    ed = oracle.EditorOracle(N, H, W, n_walls)
    ed.random_levels(seed, first_id)
    return ed


def test_random_levels_are_valid_levels():
    N, H, W, nw = 500, 13, 13, 50
    ed = _levels(N, H, W, nw, seed=7)
    lv = ed.get_levels()
    assert (ed.t == nw + 2).all()
    assert set(np.unique(lv.walls)) <= {0, 1}
    n = np.arange(N)
    assert (lv.walls[n, lv.agent_xy[:, 1], lv.agent_xy[:, 0]] == 0).all()
    assert (lv.walls[n, lv.goal_xy[:, 1], lv.goal_xy[:, 0]] == 0).all()
    assert (lv.agent_xy != lv.goal_xy).any(axis=1).all()
    assert ((lv.agent_xy >= 0) & (lv.agent_xy < [W, H])).all()
    assert ((lv.goal_xy >= 0) & (lv.goal_xy < [W, H])).all()
    counts = lv.walls.reshape(N, -1).sum(1)
    assert counts.max() <= nw and counts.min() >= 1
    # 50 draws with repeats over 169 cells leave 169*(1-(168/169)^50) = 43.4 distinct cells on
    # average, minus up to two cleared under the agent and the goal
    assert 41.0 < counts.mean() < 44.0
    assert set(np.unique(lv.agent_dir)) == {0, 1, 2, 3}


def test_random_levels_equal_the_design_episode_under_the_same_draws():
    N, H, W, nw, seed, first = 40, 6, 9, 12, 99, 1000
    ed = _levels(N, H, W, nw, seed, first)
    actions = np.array([[oracle.draw_below(oracle.level_draw(seed, first + n, 0, j), H * W)
                         for n in range(N)] for j in range(nw + 2)], np.int32)
    dirs = np.array([oracle.level_draw(seed, first + n, 0, nw + 2) & 3 for n in range(N)], np.int8)
    ref = oracle.EditorOracle(N, H, W, nw)
    ref.reset(dirs)
    ref.step(actions, nw + 2, want_obs=False)
    a, b = ed.get_levels(), ref.get_levels()
    for x, y in zip((a.walls, a.agent_xy, a.agent_dir, a.goal_xy),
                    (b.walls, b.agent_xy, b.agent_dir, b.goal_xy)):
        assert (x == y).all()


def test_levels_do_not_depend_on_the_batch_they_are_drawn_in():
    H, W, nw, seed = 13, 13, 50, 5
    whole = _levels(64, H, W, nw, seed, first_id=100).get_levels()
    lo = _levels(24, H, W, nw, seed, first_id=100).get_levels()
    hi = _levels(40, H, W, nw, seed, first_id=124).get_levels()
    assert (whole.walls == np.concatenate([lo.walls, hi.walls])).all()
    assert (whole.agent_xy == np.concatenate([lo.agent_xy, hi.agent_xy])).all()
    assert (whole.goal_xy == np.concatenate([lo.goal_xy, hi.goal_xy])).all()
    assert (whole.agent_dir == np.concatenate([lo.agent_dir, hi.agent_dir])).all()
    other = _levels(64, H, W, nw, seed + 1, first_id=100).get_levels()
    assert (whole.walls != other.walls).any(axis=(1, 2)).all()
    big = _levels(2, H, W, nw, seed, first_id=(1 << 32) + 100).get_levels()     # high id word counts
    assert (big.walls[0] != whole.walls[0]).any()


def test_cells_are_drawn_uniformly():
    N, H, W, nw = 4000, 5, 7, 6
    lv = _levels(N, H, W, nw, seed=21).get_levels()
    cells = H * W
    agent = np.bincount(lv.agent_xy[:, 1] * W + lv.agent_xy[:, 0], minlength=cells)
    walls = lv.walls.reshape(N, cells).sum(0)
    # chi-square with 34 degrees of freedom: mean 34, sd 8.2; 80 is > 5 sd out
    for counts in (agent, walls):
        e = counts.sum() / cells
        assert ((counts - e) ** 2 / e).sum() < 80


def test_mutation_invariants():
    N, H, W, nw, seed = 300, 13, 13, 50, 3
    ed = _levels(N, H, W, nw, seed)
    before = ed.get_levels()
    ed.mutate(seed=11, first_id=0, n_edits=0)
    assert (ed.walls == before.walls).all()
    ed.mutate(seed=11, first_id=0, n_edits=20)
    after = ed.get_levels()
    n = np.arange(N)
    assert (after.agent_xy == before.agent_xy).all() and (after.goal_xy == before.goal_xy).all()
    assert (after.walls[n, after.agent_xy[:, 1], after.agent_xy[:, 0]] == 0).all()
    assert (after.walls[n, after.goal_xy[:, 1], after.goal_xy[:, 0]] == 0).all()
    changed = (after.walls != before.walls).reshape(N, -1).sum(1)
    assert changed.max() <= 20
    # 20 flips over 169 cells: a cell flipped an odd number of times differs; ~18 on average
    assert 16.0 < changed.mean() < 19.5
    # the same draws again undo every flip
    ed.mutate(seed=11, first_id=0, n_edits=20)
    assert (ed.walls == before.walls).all()
    # other draws do not
    ed.mutate(seed=12, first_id=0, n_edits=20)
    assert (ed.walls != before.walls).any()


def test_single_mutation_is_the_drawn_cell():
    N, H, W = 50, 4, 6
    ed = oracle.EditorOracle(N, H, W, 3)
    walls = np.zeros((N, H, W), np.int8)
    axy = np.tile(np.array([[0, 0]], np.int32), (N, 1))
    gxy = np.tile(np.array([[5, 3]], np.int32), (N, 1))
    ed.set_levels(walls, axy, np.zeros(N, np.int8), gxy)
    ed.mutate(seed=77, first_id=500, n_edits=1)
    for n in range(N):
        c = oracle.draw_below(oracle.level_draw(77, 500 + n, 1, 0), H * W)
        expect = np.zeros(H * W, np.int8)
        if c not in (0, H * W - 1):
            expect[c] = 1
        assert (ed.walls[n].reshape(-1) == expect).all()


def test_set_levels_round_trip():
    N, H, W = 30, 7, 5
    rng = np.random.default_rng(0)
    walls = (rng.random((N, H, W)) < 0.3).astype(np.int8) * 5          # any non-zero value is a wall
    axy = np.stack([rng.integers(0, W, N), rng.integers(0, H, N)], 1).astype(np.int32)
    gxy = np.stack([rng.integers(0, W, N), rng.integers(0, H, N)], 1).astype(np.int32)
    adir = rng.integers(0, 4, N).astype(np.int8)
    ed = oracle.EditorOracle(N, H, W, 4)
    ed.set_levels(walls, axy, adir, gxy)
    lv = ed.get_levels()
    assert (lv.walls == (walls != 0)).all()
    assert (lv.agent_xy == axy).all() and (lv.goal_xy == gxy).all() and (lv.agent_dir == adir).all()
    assert (ed.t == 6).all()
    ed.set_levels(walls, axy + 100, adir, gxy - 100)                   # clamped into the interior
    assert (ed.agent_xy == [W - 1, H - 1]).all() and (ed.goal_xy == 0).all()
