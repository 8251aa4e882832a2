"""GPU parity tests of the shared-world task (the whole population as agents of one world) against
oracle/forage.py.  The world's arithmetic is binary32 by definition, so a step from a given state
with given actions is compared bit for bit; so is a whole roll-out whose policies ignore their
observations (constant actions).  With observation-driven policies the fp32 policy output differs
from the oracle's in the last bits, so one step is compared at 1e-6 and longer horizons
statistically (a flipped nearest neighbour is a legitimate, discontinuous difference)."""
import numpy as np
import pytest

from oracle import forage
from workloads import CONFIGS, configs as wc, generators as gen
from tests.util import dev, host

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

SEED = 20220509


@pytest.fixture(scope="module")
def evo():
    import paper_2202_05008_amd as e
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return e


def _cp(w):
    return (w["dt"], w["thrust"], w["drag"], w["vmax"], w["radius"], float(w["n_food"]), float(w["n_poison"]))


def _task(evo, w, worlds, pop, pd=None, generation=3, seed=SEED, kind=None):
    kind = evo.EVO_TASK_FORAGE if kind is None else kind
    make = lambda work: evo.make_task_desc(kind, n_rollouts=worlds, reset_seed=seed,
                                           generation=generation, cp=_cp(w), work=work)
    if pd is None:
        return make(None)
    n = evo.rollout_workspace_bytes(make(None), pd, pop)
    assert n > 0
    return make(torch.empty(n, dtype=torch.uint8, device="cuda"))


def _bits(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint32) if a.dtype == np.float32 else a


@pytest.mark.parametrize("pop,worlds,n_food,n_poison,radius", [(130, 3, 5, 7, 0.0625), (1024, 5, 24, 24, 0.03125),
                                                               (2, 1, 1, 1, 0.25), (77, 8, 100, 156, 0.015625),
                                                               (2500, 2, 24, 24, 0.03125),
                                                               (4800, 1, 24, 24, 0.03125)])   # the most that fit
def test_one_step_from_a_given_state_is_bit_exact(evo, pop, worlds, n_food, n_poison, radius):
    w = dict(forage.WORLD_DEFAULT, n_food=n_food, n_poison=n_poison, radius=radius)
    n_items = n_food + n_poison
    rng = np.random.default_rng(pop * 31 + worlds)
    pos = rng.random((worlds, pop, 2), dtype=np.float32)
    vel = (rng.random((worlds, pop, 2), dtype=np.float32) - np.float32(0.5)) * np.float32(2 * w["vmax"])
    act = (rng.standard_normal((worlds, pop, 2)) * 1.2).astype(np.float32)
    counts = rng.integers(0, 6, size=(worlds, n_items)).astype(np.int32)
    # special cases: agents on top of each other (distance 0, index tie-break), on the walls and heading
    # out, and sitting on items of their world (touches)
    if pop >= 16:
        pos[:, 5] = pos[:, 3]
        pos[:, 9] = pos[:, 3]
        pos[:, 7] = (0.0, 1.0)
        vel[:, 7] = (-w["vmax"], w["vmax"])
        act[:, 7] = (-1.0, 1.0)
        for r in range(worlds):
            items = forage.item_positions(SEED, 3, r, counts[r])
            pos[r, 10:10 + min(4, n_items)] = items[:min(4, n_items)]
            pos[r, 14] = items[-1] + np.float32(radius / 2)
            vel[r, 10:15] = 0
            act[r, 10:15] = 0
    td = _task(evo, w, worlds, pop)
    f32, i32 = torch.float32, torch.int32
    obs = torch.empty(worlds, pop, 8, dtype=f32, device="cuda")
    npos, nvel = torch.empty(worlds, pop, 2, dtype=f32, device="cuda"), torch.empty(worlds, pop, 2, dtype=f32, device="cuda")
    reward = torch.full((worlds, pop), 99, dtype=i32, device="cuda")
    hit = torch.full((worlds, n_items), 99, dtype=i32, device="cuda")
    evo.evo_forage_step(td, pop, dev(pos), dev(vel), dev(counts), dev(act), obs, npos, nvel, reward, hit)
    touched = 0
    for r in range(worlds):
        items = forage.item_positions(SEED, 3, r, counts[r])
        want_obs = forage.observe(pos[r], vel[r], items, n_food)
        p, v, rew, h = forage.step(pos[r], vel[r], act[r], items, n_food, w)
        assert np.array_equal(_bits(host(obs)[r]), _bits(want_obs)), "observations of world %d" % r
        assert np.array_equal(_bits(host(npos)[r]), _bits(p)), "positions of world %d" % r
        assert np.array_equal(_bits(host(nvel)[r]), _bits(v)), "velocities of world %d" % r
        assert np.array_equal(host(reward)[r], rew), "rewards of world %d" % r
        assert np.array_equal(host(hit)[r], h.astype(np.int32)), "hits of world %d" % r
        touched += int(np.abs(rew).sum())
    assert touched > 0 or pop < 16, "the case must exercise touches"


def _params_constant_action(pop, dims, rng):
    """Zero weights, the output bias as the action (no output activation): policies that ignore what they see."""
    P = wc.mlp_param_count(dims)
    params = np.zeros((pop, P), dtype=np.float32)
    params[:, -2:] = (rng.random((pop, 2), dtype=np.float32) - np.float32(0.5)) * np.float32(3.0)
    return params


def _run_state(evo, td, pd, params, pop, worlds, n_items, steps, solo=False):
    f32, i32 = torch.float32, torch.int32
    pos = torch.empty(worlds, pop, 2, dtype=f32, device="cuda")
    vel = torch.empty(worlds, pop, 2, dtype=f32, device="cuda")
    reward = torch.empty(worlds, pop, dtype=i32, device="cuda")
    counts = torch.empty((worlds, pop, n_items) if solo else (worlds, n_items), dtype=i32, device="cuda")
    evo.evo_forage_state(td, pd, params, pop, steps, pos, vel, reward, counts)
    fit = torch.empty(pop, dtype=f32, device="cuda")
    evo.rollout(td, pd, params, pop, steps, fit)
    return host(pos), host(vel), host(reward), host(counts), host(fit)


@pytest.mark.parametrize("pop,worlds,H,steps", [(150, 3, 16, 61), (64, 1, 32, 40), (34, 6, 64, 35)])
def test_whole_rollout_with_constant_actions_is_bit_exact(evo, pop, worlds, H, steps):
    w = dict(forage.WORLD_DEFAULT, n_food=9, n_poison=6, radius=0.0625)
    dims, acts = (8, H, H, 2), (evo.EVO_ACT_TANH, evo.EVO_ACT_RELU, evo.EVO_ACT_NONE)
    params = _params_constant_action(pop, dims, np.random.default_rng(H))
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    td = _task(evo, w, worlds, pop, pd)
    pos, vel, reward, counts, fit = _run_state(evo, td, pd, dev(params), pop, worlds, 15, steps)
    want_fit, total, details = forage.rollout(params, dims, acts, SEED, 3, worlds, steps, w, return_details=True)
    for r in range(worlds):
        assert np.array_equal(_bits(pos[r]), _bits(details[r][0])), "positions of world %d" % r
        assert np.array_equal(_bits(vel[r]), _bits(details[r][1])), "velocities of world %d" % r
        assert np.array_equal(counts[r], details[r][2]), "item book of world %d" % r
    assert np.array_equal(reward, total)
    assert np.abs(total).sum() > 20 and max(d[2].max() for d in details) >= 2, "items must be eaten, some twice"
    np.testing.assert_allclose(fit, want_fit, rtol=1e-6, atol=0)


def _random_policies(pop, dims, scale, seed):
    P = wc.mlp_param_count(dims)
    return (np.random.default_rng(seed).standard_normal((pop, P)) * scale).astype(np.float32)


@pytest.mark.parametrize("H,acts", [(32, (1, 1, 1)), (16, (2, 1, 0)), (64, (1, 2, 1))])
def test_one_step_with_the_policy_in_the_loop(evo, H, acts):
    pop, worlds = 200, 2
    w = dict(forage.WORLD_DEFAULT, radius=0.0625)
    dims = (8, H, H, 2)
    params = _random_policies(pop, dims, 0.5, H)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    td = _task(evo, w, worlds, pop, pd)
    pos, vel, reward, counts, fit = _run_state(evo, td, pd, dev(params), pop, worlds, 48, 1)
    _, total, details = forage.rollout(params, dims, acts, SEED, 3, worlds, 1, w, return_details=True)
    for r in range(worlds):
        np.testing.assert_allclose(vel[r], details[r][1], rtol=0, atol=1e-7)
        np.testing.assert_allclose(pos[r], details[r][0], rtol=0, atol=1e-7)
    assert np.array_equal(reward, total)
    assert np.abs(vel).max() > 1e-3, "the policies must act"


def test_short_horizon_with_the_policy_in_the_loop(evo):
    pop, worlds, steps = 256, 2, 20
    w = dict(forage.WORLD_DEFAULT, radius=0.0625)
    dims, acts = (8, 32, 32, 2), (1, 1, 1)
    params = _random_policies(pop, dims, 0.5, 11)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    td = _task(evo, w, worlds, pop, pd)
    pos, vel, reward, counts, fit = _run_state(evo, td, pd, dev(params), pop, worlds, 48, steps)
    want_fit, total, details = forage.rollout(params, dims, acts, SEED, 3, worlds, steps, w, return_details=True)
    want_pos = np.stack([d[0] for d in details])
    close = np.abs(pos - want_pos).max(axis=-1) < 1e-5
    assert close.mean() > 0.97, "agents off the oracle's path: %d of %d" % ((~close).sum(), close.size)
    assert (reward == total).mean() > 0.97
    assert np.abs(total).sum() > 10


def test_long_horizon_population_statistics(evo):
    """300 steps with observation-driven policies: single trajectories part ways (a nearest neighbour that
    flips is a discontinuity), the population's statistics do not: the two fitness vectors have the same mean
    within sampling error and are strongly rank-correlated (what an agent collects is mostly its policy's doing)."""
    from scipy.stats import spearmanr
    pop, worlds, steps = 128, 4, 300
    w = dict(forage.WORLD_DEFAULT, radius=0.0625)
    dims, acts = (8, 32, 32, 2), (1, 1, 1)
    params = _random_policies(pop, dims, 0.7, 23)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    td = _task(evo, w, worlds, pop, pd)
    pos, vel, reward, counts, fit = _run_state(evo, td, pd, dev(params), pop, worlds, 48, steps)
    want = forage.rollout(params, dims, acts, SEED, 3, worlds, steps, w)
    sem = np.sqrt((want.var() + fit.var()) / pop)
    assert abs(fit.mean() - want.mean()) < 4 * sem + 0.05, (fit.mean(), want.mean(), sem)
    assert abs(np.abs(fit).mean() - np.abs(want).mean()) < 0.25 * np.abs(want).mean() + 0.1
    rho = spearmanr(fit, want).correlation
    assert rho > 0.5, rho


def test_full_size_constant_actions_and_properties(evo):
    """The benchmark's configuration (1024 agents, 8 worlds, H = 32): 40 steps of policies that ignore
    their observations bit for bit against the oracle, then the full 500 steps with random policies:
    repeatable, whole-number rewards, everyone inside the square."""
    c = CONFIGS["forage"]
    w = wc.world_dict(c.world)
    n_items = w["n_food"] + w["n_poison"]
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
    td = _task(evo, w, c.n_rollouts, c.pop, pd)
    acts_none = (1, 1, 0)
    pd_none = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, acts_none)
    params = _params_constant_action(c.pop, c.dims, np.random.default_rng(1))
    pos, vel, reward, counts, fit = _run_state(evo, td, pd_none, dev(params), c.pop, c.n_rollouts, n_items, 40)
    want_fit, total, details = forage.rollout(params, c.dims, acts_none, SEED, 3, c.n_rollouts, 40, w, return_details=True)
    for r in range(c.n_rollouts):
        assert np.array_equal(_bits(pos[r]), _bits(details[r][0])) and np.array_equal(counts[r], details[r][2])
    assert np.array_equal(reward, total) and np.abs(total).sum() > 100
    params = dev(_random_policies(c.pop, c.dims, 0.3, 5))
    a = _run_state(evo, td, pd, params, c.pop, c.n_rollouts, n_items, c.steps)
    b = _run_state(evo, td, pd, params, c.pop, c.n_rollouts, n_items, c.steps)
    for x, y in zip(a, b):
        assert np.array_equal(_bits(x), _bits(y)), "two runs of the same roll-out differ"
    pos, vel, reward, counts, fit = a
    assert pos.min() >= 0 and pos.max() <= 1 and np.abs(vel).max() <= w["vmax"]
    np.testing.assert_array_equal(fit * c.n_rollouts, reward.sum(axis=0).astype(np.float32))
    assert counts.min() > 0, "over 500 steps every item of every world is eaten at some point"


def test_errors_are_reported(evo):
    w = forage.WORLD_DEFAULT
    good = evo.make_policy_desc(evo.EVO_POLICY_MLP, (8, 32, 32, 2), (1, 1, 1))
    fit = torch.empty(64, dtype=torch.float32, device="cuda")
    params = torch.zeros(64, wc.mlp_param_count((8, 32, 32, 2)), dtype=torch.float32, device="cuda")
    td = _task(evo, w, 2, 64, good)
    for dims in [(8, 32, 16, 2), (5, 32, 32, 2), (8, 48, 48, 2), (8, 32, 32, 1)]:
        bad = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, (1, 1, 1))
        with pytest.raises(evo.EvoError):
            evo.rollout(td, bad, params, 64, 5, fit)
    with pytest.raises(evo.EvoError):                    # no workspace
        evo.rollout(_task(evo, w, 2, 64), good, params, 64, 5, fit)
    with pytest.raises(evo.EvoError):                    # no poison
        evo.rollout(_task(evo, dict(w, n_poison=0), 2, 64), good, params, 64, 5, fit)
    big = torch.zeros(6000, params.shape[1], dtype=torch.float32, device="cuda")
    with pytest.raises(evo.EvoError):                    # more agents than the staging area holds
        evo.rollout(_task(evo, w, 2, 6000, good), good, big, 6000, 5, torch.empty(6000, dtype=torch.float32, device="cuda"))
    evo.rollout(td, good, params, 64, 5, fit)            # and the good case still runs
    assert torch.isfinite(fit).all()


# ---- the single-agent form: every member alone in its own copy of each world, one launch per episode ----

@pytest.mark.parametrize("pop,worlds,H,steps,n_food,n_poison", [(13, 3, 16, 60, 9, 6), (8, 1, 32, 45, 24, 24),
                                                                 (5, 6, 64, 35, 3, 40), (1, 1, 32, 30, 1, 1)])
def test_solo_rollout_with_constant_actions_is_bit_exact(evo, pop, worlds, H, steps, n_food, n_poison):
    w = dict(forage.WORLD_DEFAULT, n_food=n_food, n_poison=n_poison, radius=0.125)
    dims, acts = (8, H, H, 2), (evo.EVO_ACT_TANH, evo.EVO_ACT_RELU, evo.EVO_ACT_NONE)
    params = _params_constant_action(pop, dims, np.random.default_rng(H + pop))
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    td = _task(evo, w, worlds, pop, pd, kind=evo.EVO_TASK_FORAGE_SOLO)
    n_items = n_food + n_poison
    pos, vel, reward, counts, fit = _run_state(evo, td, pd, dev(params), pop, worlds, n_items, steps, solo=True)
    want_fit, total, details = forage.rollout_solitary(params, dims, acts, SEED, 3, worlds, steps, w, return_details=True)
    for m in range(pop):
        for r in range(worlds):
            assert np.array_equal(_bits(pos[r, m]), _bits(details[m][r][0][0])), "position of member %d, world %d" % (m, r)
            assert np.array_equal(_bits(vel[r, m]), _bits(details[m][r][1][0]))
            assert np.array_equal(counts[r, m], details[m][r][2]), "item book of member %d, world %d" % (m, r)
    assert np.array_equal(reward, total)
    assert counts.sum() > 0 or n_items < 10, "items must be eaten"
    np.testing.assert_allclose(fit, want_fit, rtol=1e-6, atol=0)


def test_solo_policy_in_the_loop(evo):
    pop, worlds = 24, 2
    w = dict(forage.WORLD_DEFAULT, radius=0.0625)
    dims, acts = (8, 32, 32, 2), (1, 1, 1)
    params = _random_policies(pop, dims, 0.5, 31)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    td = _task(evo, w, worlds, pop, pd, kind=evo.EVO_TASK_FORAGE_SOLO)
    pos, vel, reward, counts, fit = _run_state(evo, td, pd, dev(params), pop, worlds, 48, 1, solo=True)
    _, total, details = forage.rollout_solitary(params, dims, acts, SEED, 3, worlds, 1, w, return_details=True)
    want_pos = np.stack([np.stack([details[m][r][0][0] for m in range(pop)]) for r in range(worlds)])
    want_vel = np.stack([np.stack([details[m][r][1][0] for m in range(pop)]) for r in range(worlds)])
    np.testing.assert_allclose(pos, want_pos, rtol=0, atol=1e-7)
    np.testing.assert_allclose(vel, want_vel, rtol=0, atol=1e-7)
    assert np.array_equal(reward, total) and np.abs(vel).max() > 1e-3
    # 25 steps: most members still on the oracle's path (a flipped nearest item is a legitimate discontinuity)
    pos, vel, reward, counts, fit = _run_state(evo, td, pd, dev(params), pop, worlds, 48, 25, solo=True)
    _, total, details = forage.rollout_solitary(params, dims, acts, SEED, 3, worlds, 25, w, return_details=True)
    want_pos = np.stack([np.stack([details[m][r][0][0] for m in range(pop)]) for r in range(worlds)])
    close = np.abs(pos - want_pos).max(axis=-1) < 1e-5
    assert close.mean() > 0.9 and (reward == total).mean() > 0.9


def test_solo_full_size_properties(evo):
    """1024 members x 8 worlds x 500 steps in one launch: repeatable bit for bit, inside the square, whole-number
    rewards; members with the same policy get the same result (their worlds are identical)."""
    c = CONFIGS["forage"]
    w = wc.world_dict(c.world)
    n_items = w["n_food"] + w["n_poison"]
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
    td = _task(evo, w, c.n_rollouts, c.pop, pd, kind=evo.EVO_TASK_FORAGE_SOLO)
    host_params = _random_policies(c.pop, c.dims, 0.3, 5)
    host_params[1::2] = host_params[0::2]                  # pairs of identical policies
    params = dev(host_params)
    a = _run_state(evo, td, pd, params, c.pop, c.n_rollouts, n_items, c.steps, solo=True)
    b = _run_state(evo, td, pd, params, c.pop, c.n_rollouts, n_items, c.steps, solo=True)
    for x, y in zip(a, b):
        assert np.array_equal(_bits(x), _bits(y)), "two runs of the same roll-out differ"
    pos, vel, reward, counts, fit = a
    assert pos.min() >= 0 and pos.max() <= 1 and np.abs(vel).max() <= w["vmax"]
    np.testing.assert_array_equal(fit * c.n_rollouts, reward.sum(axis=0).astype(np.float32))
    assert np.array_equal(reward[:, 0::2], reward[:, 1::2]) and np.array_equal(_bits(pos[:, 0::2]), _bits(pos[:, 1::2]))
    assert counts.sum() > 0 and np.array_equal(counts[:, :, :w["n_food"]].sum(axis=2) - counts[:, :, w["n_food"]:].sum(axis=2), reward)
