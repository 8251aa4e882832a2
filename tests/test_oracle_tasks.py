"""Pins for oracle/tasks.py: library losses, Lagrangian invariants of the cart-pole
(energy, momentum, small-angle period, the mass-matrix form of its equations), reward and
termination book-keeping by brute force."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import tasks, philox, policy
from workloads import mlp_param_count

CP = tasks.CP_DEFAULT
FREE = (9.82, 0.5, 0.5, 0.6, 0.0, 10.0, 0.01, 2.4)          # no friction


def test_losses_closed_forms_and_torch():
    rng = np.random.default_rng(0)
    logits = rng.standard_normal((3, 11, 5)) * 4
    y = rng.integers(0, 5, size=11)
    want = [-F.cross_entropy(torch.tensor(logits[m]), torch.tensor(y)).item() for m in range(3)]
    np.testing.assert_allclose(tasks.classify_fitness(logits, y), want, rtol=1e-12)
    conf = np.full((1, 4, 3), -50.0)
    conf[0, np.arange(4), [0, 1, 2, 0]] = 50.0
    assert abs(tasks.classify_fitness(conf, [0, 1, 2, 0])[0]) < 1e-30
    np.testing.assert_allclose(tasks.classify_fitness(conf, [1, 1, 2, 0])[0], -25.0, rtol=1e-12)
    big = np.array([[[1e4, 0.0]]])
    assert np.isfinite(tasks.classify_fitness(big, [1])[0])           # stable log-sum-exp
    out = rng.standard_normal((2, 6, 4))
    assert (tasks.regress_fitness(out, out) == 0).all()
    np.testing.assert_allclose(tasks.regress_fitness(out, out + 2.0), -4.0, rtol=1e-12)
    th = rng.standard_normal((3, 9))
    xs = rng.standard_normal(9)
    np.testing.assert_allclose(tasks.sphere_fitness(th, xs), [-np.linalg.norm(t - xs) ** 2 for t in th], rtol=1e-12)
    assert tasks.sphere_fitness(xs[None], xs)[0] == 0.0


def test_equations_of_motion_solve_the_lagrangian_system():
    """Euler-Lagrange equations in mass-matrix form, solved numerically:
       [M+m, m l cos/2; m l cos/2, m l^2/3] [x_dd, th_dd] = [F - b x_d + m l th_d^2 sin/2, m g l sin/2]."""
    g, M, m, l, b, fs = CP[:6]
    rng = np.random.default_rng(1)
    for _ in range(200):
        s = rng.standard_normal(4) * np.array([1, 2, 3, 4])
        a = rng.uniform(-1, 1)
        A = np.array([[M + m, 0.5 * m * l * np.cos(s[2])], [0.5 * m * l * np.cos(s[2]), m * l * l / 3.0]])
        rhs = np.array([fs * a - b * s[1] + 0.5 * m * l * s[3] ** 2 * np.sin(s[2]), 0.5 * m * g * l * np.sin(s[2])])
        want = np.linalg.solve(A, rhs)
        xdd, thdd = tasks.cartpole_derivs(s, a, CP)
        np.testing.assert_allclose([xdd, thdd], want, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(thdd, 3.0 * (g * np.sin(s[2]) - xdd * np.cos(s[2])) / (2.0 * l), rtol=1e-11, atol=1e-12)


def _free_run(s0, dt, T):
    cp = FREE[:6] + (dt, 2.4)
    s = np.array(s0, dtype=np.float64)
    for _ in range(int(round(T / dt))):
        s, _ = tasks.cartpole_step(s, 0.0, cp)
    return s


def test_energy_and_momentum_drift_vanish_with_dt():
    s0 = np.array([0.1, -0.2, np.pi + 0.3, 0.5])
    e0, p0 = tasks.cartpole_energy(s0, FREE), tasks.cartpole_momentum(s0, FREE)
    drifts = []
    for dt in (0.01, 0.005, 0.0025, 1e-4):
        s = _free_run(s0, dt, 2.0)
        drifts.append(tasks.cartpole_energy(s, FREE) - e0)
        assert abs(tasks.cartpole_momentum(s, FREE) - p0) < 30 * dt
    assert abs(drifts[3]) < 1e-3 and abs(drifts[0]) < 0.2
    ratios = [drifts[0] / drifts[1], drifts[1] / drifts[2]]
    assert all(1.6 < r < 2.8 for r in ratios)                 # first-order integrator: error ~ dt
    # the continuous system conserves both exactly: dE/dt = 0 along the vector field
    rng = np.random.default_rng(2)
    for _ in range(50):
        s = rng.standard_normal(4) * np.array([1, 2, 3, 4])
        xdd, thdd = tasks.cartpole_derivs(s, 0.0, FREE)
        h = 1e-6
        f = lambda q: tasks.cartpole_energy(q, FREE)
        vec = np.array([s[1], xdd, s[3], thdd])
        dE = (f(s + h * vec) - f(s - h * vec)) / (2 * h)
        assert abs(dE) < 1e-6 * (1 + abs(f(s)))
        fp = lambda q: tasks.cartpole_momentum(q, FREE)
        assert abs((fp(s + h * vec) - fp(s - h * vec)) / (2 * h)) < 1e-6


def test_small_angle_period_hanging_down():
    g, M, m, l = FREE[:4]
    period = 2 * np.pi * np.sqrt(l * (4 * (M + m) - 3 * m) / (6 * (M + m) * g))
    assert abs(period - 1.003) < 1e-3
    dt = 1e-4
    cp = FREE[:6] + (dt, 2.4)
    s = np.array([0.0, 0.0, np.pi + 1e-3, 0.0])
    crossings, prev = [], s[2] - np.pi
    for i in range(int(2.6 / dt)):
        s, _ = tasks.cartpole_step(s, 0.0, cp)
        cur = s[2] - np.pi
        if prev > 0 >= cur:
            crossings.append(i * dt)
        prev = cur
    assert len(crossings) >= 2
    assert abs((crossings[1] - crossings[0]) - period) < 2e-3


def test_step_observation_reward_conventions():
    s = np.array([0.3, -0.4, 0.7, 1.1])
    nxt, r = tasks.cartpole_step(s, 0.25, CP)
    xdd, thdd = tasks.cartpole_derivs(s, 0.25, CP)
    np.testing.assert_allclose(nxt, [0.3 - 0.004, -0.4 + 0.01 * xdd, 0.7 + 0.011, 1.1 + 0.01 * thdd], rtol=1e-14)
    np.testing.assert_allclose(r, np.cos(nxt[2]) * np.exp(-nxt[0] ** 2), rtol=1e-14)
    np.testing.assert_allclose(tasks.cartpole_obs(s), [0.3, -0.4, np.cos(0.7), np.sin(0.7), 1.1])
    # a positive action pushes the cart to the right; upright pole then falls to the left (theta<0)
    n2, _ = tasks.cartpole_step(np.array([0.0, 0.0, 0.0, 0.0]), 1.0, CP)
    assert n2[1] > 0 and n2[3] < 0
    s0 = tasks.cartpole_reset(5, 3, 16)
    z = philox.block_normals(5, 0, np.arange(16), 3, philox.TAG_RESET)
    np.testing.assert_allclose(s0 - np.array([0, 0, np.pi, 0]), 0.2 * z, atol=1e-15)
    assert s0.shape == (16, 4) and abs(np.cos(s0[:, 2]).mean() + 1) < 0.1    # starts hanging down


def test_rollout_bookkeeping_by_brute_force():
    dims, acts = (5, 3, 1), (1, 1)
    P = mlp_param_count(dims)
    rng = np.random.default_rng(3)
    params = rng.standard_normal((3, P)) * 2.0
    params[2] = 0.0                                   # zero policy: action tanh(0) = 0
    R, steps, seed, gen = 6, 150, 11, 2
    cp = (9.82, 0.5, 0.5, 0.6, 0.1, 10.0, 0.02, 0.5)   # tight track so that episodes terminate
    fit, ret, s_end, alive = tasks.cartpole_rollout(params, dims, acts, seed, gen, R, steps, cp, return_details=True)
    s0 = tasks.cartpole_reset(seed, gen, R)
    assert (~alive).any() and alive.any()
    for m in range(3):
        for r in range(R):
            s = s0[r].copy()
            total, live = 0.0, True
            for _ in range(steps):
                if not live:
                    break
                a = policy.mlp_forward(params[m:m + 1], tasks.cartpole_obs(s)[None], dims, acts)[0, 0, 0]
                s, rew = tasks.cartpole_step(s, a, cp)
                assert abs(rew) <= 1.0
                total += rew
                live = abs(s[0]) <= cp[7]
            np.testing.assert_allclose(ret[m, r], total, rtol=1e-12, atol=1e-12)
            assert live == alive[m, r]
    np.testing.assert_allclose(fit, ret.mean(axis=1))
    assert (np.abs(ret) <= steps).all()
    # zero policy and no friction reproduces the free system
    free = (9.82, 0.5, 0.5, 0.6, 0.0, 10.0, 0.01, 100.0)
    _, _, s_end, _ = tasks.cartpole_rollout(params[2:3], dims, acts, seed, gen, R, 50, free, return_details=True)
    for r in range(R):
        np.testing.assert_allclose(s_end[0, r], _free_run(s0[r], 0.01, 0.5), rtol=1e-12)
    # identical members see identical episodes
    f2 = tasks.cartpole_rollout(np.stack([params[0], params[0]]), dims, acts, seed, gen, R, 40, CP)
    assert f2[0] == f2[1]
