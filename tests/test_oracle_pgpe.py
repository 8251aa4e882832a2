"""Pins for oracle/pgpe.py: invariants of ask, brute-force ranks, the PGPE estimator from
its textbook definition on materialised samples, closed-form expectations, Adam closed
forms, bf16 rounding against a library routine, and convergence on a sphere."""
import numpy as np
import pytest
import torch

from oracle import pgpe, philox


def _state(P, mu=None, sigma=0.1, **kw):
    st = pgpe.PGPEState.create(pgpe.PGPEConfig(P=P, sigma_init=sigma, **kw), mu)
    return st


# ---------------------------------------------------------------- ask
def test_antithetic_pairs():
    P, pop = 37, 10
    st = _state(P)                                   # mu = 0: mirror images are exact negatives
    th = pgpe.ask(st, 123, pop)
    assert (th[0::2].view(np.uint32) ^ th[1::2].view(np.uint32) == 0x80000000).all()
    mu = np.random.default_rng(0).standard_normal(P).astype(np.float32)
    st = _state(P, mu)
    th = pgpe.ask(st, 123, pop).astype(np.float64)
    # each member is rounded once to fp32: the pair misses 2 mu by at most half an ulp of each
    half = 0.5 * (np.spacing(np.abs(th[0::2]).astype(np.float32)) + np.spacing(np.abs(th[1::2]).astype(np.float32)))
    assert (np.abs(th[0::2] + th[1::2] - 2.0 * mu) <= half.astype(np.float64)).all()
    # in exact (fp64) arithmetic the pair sums to 2 mu
    z = philox.pair_noise(123, 1, np.arange(pop // 2), P)
    plus = mu.astype(np.float64) + st.sigma.astype(np.float64) * z
    minus = mu.astype(np.float64) - st.sigma.astype(np.float64) * z
    np.testing.assert_allclose(plus + minus, np.broadcast_to(2.0 * mu, plus.shape), rtol=0, atol=1e-15)


def test_zero_sigma_returns_mu_bit_exact():
    mu = np.random.default_rng(1).standard_normal(50).astype(np.float32)
    st = _state(50, mu, sigma=0.0)
    th = pgpe.ask(st, 9, 6)
    assert (th.view(np.uint32) == mu.view(np.uint32)[None, :]).all()


def test_perturbation_is_sigma_times_noise():
    P = 64
    st = _state(P, sigma=0.25)
    th = pgpe.ask(st, 5, 4)
    z = philox.pair_noise(5, 1, [0, 1], P)
    np.testing.assert_allclose(th[0::2], 0.25 * z, rtol=1e-6)
    assert th.dtype == np.float32


def test_ask_rejects_odd_population_and_uses_generation():
    st = _state(8)
    with pytest.raises(ValueError):
        pgpe.ask(st, 1, 5)
    a = pgpe.ask(st, 1, 4)
    st.t = 2
    b = pgpe.ask(st, 1, 4)
    assert not np.array_equal(a, b)
    rows = pgpe.ask_rows(st, 1, 4, members=[3], cols=[2, 7])
    assert np.array_equal(rows[0], b[3, [2, 7]])


def test_bf16_rounding_against_torch_and_midpoints():
    # exhaustive: every finite bf16 value v and its successor w; the midpoint rounds to the even one
    hi = np.arange(0x0000, 0x7F7F, dtype=np.uint32)
    v = (hi << 16).view(np.float32)
    mid_bits = (hi << 16) | np.uint32(0x8000)
    mid = mid_bits.view(np.float32)
    r = pgpe.round_to_bf16(mid).view(np.uint32) >> 16
    expect = np.where(hi % 2 == 0, hi, hi + 1)
    assert (r == expect).all()
    assert (pgpe.round_to_bf16((mid_bits + 1).view(np.float32)).view(np.uint32) >> 16 == hi + 1).all()
    assert (pgpe.round_to_bf16((mid_bits - 1).view(np.float32)).view(np.uint32) >> 16 == hi).all()
    assert (pgpe.round_to_bf16(v).view(np.uint32) == v.view(np.uint32)).all()
    x = (np.random.default_rng(2).standard_normal(200000) * 10).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(pgpe.round_to_bf16(x), want)
    assert np.array_equal(pgpe.round_to_bf16(-x), -want)


# ---------------------------------------------------------------- centered ranks
def _brute_rank(f):
    key = pgpe.orderable_key(f)
    pop = len(f)
    r = np.zeros(pop, dtype=np.uint32)
    for m in range(pop):
        for j in range(pop):
            if (int(key[j]), j) < (int(key[m]), m):
                r[m] += 1
    return r


@pytest.mark.parametrize("pop", [2, 3, 64, 257])
def test_centered_rank_structure(pop):
    f = np.random.default_rng(pop).standard_normal(pop).astype(np.float32)
    rank, c = pgpe.centered_rank(f)
    assert sorted(rank.tolist()) == list(range(pop))
    lin = np.linspace(-0.5, 0.5, pop)
    assert np.abs(np.sort(c).astype(np.float64) - lin).max() <= np.spacing(np.float32(0.5))
    assert c.dtype == np.float32 and c.min() == -0.5 and c.max() == 0.5
    assert float(np.sort(c) @ np.ones(pop)) == 0.0 or abs(c.astype(np.float64).sum()) < 1e-6
    assert (np.sort(c) == -np.sort(c)[::-1]).all()                       # exactly antisymmetric
    assert (rank == _brute_rank(f)).all()
    assert rank[np.argmax(f)] == pop - 1 and rank[np.argmin(f)] == 0
    # invariant under strictly monotone transforms
    assert (pgpe.centered_rank(np.exp(f / 3) * 7 - 2)[0] == rank).all()
    assert (pgpe.centered_rank(-f)[0] == pop - 1 - rank).all()


def test_centered_rank_ties_and_specials():
    assert (pgpe.centered_rank(np.full(9, 3.0, np.float32))[0] == np.arange(9)).all()
    f = np.array([1.0, -0.0, 0.0, 1.0, -np.inf, np.nan, np.inf, np.nan, -5.0, 0.0], np.float32)
    rank, _ = pgpe.centered_rank(f)
    #        NaN(5) NaN(7) -inf(4) -5(8) -0(1) 0(2) 0(9) 1(0) 1(3) inf(6)
    want = np.empty(10, np.uint32)
    want[[5, 7, 4, 8, 1, 2, 9, 0, 3, 6]] = np.arange(10)
    assert (rank == want).all()
    assert (rank == _brute_rank(f)).all()
    q = np.round(np.random.default_rng(3).standard_normal(200) * 2).astype(np.float32)
    assert (pgpe.centered_rank(q)[0] == _brute_rank(q)).all()
    # key map is monotone in the usual float order
    s = np.sort(np.random.default_rng(4).standard_normal(1000).astype(np.float32))
    assert (np.diff(pgpe.orderable_key(s).astype(np.int64)) >= 0).all()


# ---------------------------------------------------------------- gradient estimator
def _textbook_pgpe(theta, mu, sigma, f):
    """Symmetric-sampling PGPE written with eps = theta+ - mu on materialised samples:
    grad_mu = (1/N) sum_k eps_k (f+ - f-)/2 ; grad_sigma = (1/N) sum_k ((f+ + f-)/2 - b)(eps_k^2 - sigma^2)/sigma."""
    pop, P = theta.shape
    N = pop // 2
    b = sum(f) / pop
    gm = [0.0] * P
    gs = [0.0] * P
    for k in range(N):
        fp, fm = f[2 * k], f[2 * k + 1]
        for i in range(P):
            eps = theta[2 * k, i] - mu[i]
            gm[i] += eps * (fp - fm) / 2.0 / N
            gs[i] += ((fp + fm) / 2.0 - b) * (eps * eps - sigma[i] ** 2) / sigma[i] / N
    return np.array(gm), np.array(gs)


def test_gradient_brute_force_tiny():
    P, pop, seed = 5, 8, 31
    mu = np.random.default_rng(5).standard_normal(P)
    sigma = np.abs(np.random.default_rng(6).standard_normal(P)) + 0.1
    z = philox.pair_noise(seed, 1, np.arange(pop // 2), P)
    theta = np.empty((pop, P))
    theta[0::2] = mu + sigma * z
    theta[1::2] = mu - sigma * z
    f = np.random.default_rng(7).standard_normal(pop)
    gm, gs = pgpe.gradients(z, sigma, f)
    wm, ws = _textbook_pgpe(theta, mu, sigma, f.tolist())
    np.testing.assert_allclose(gm, wm, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(gs, ws, rtol=1e-10, atol=1e-13)


def test_gradient_from_stored_population():
    """The stored-population form against the double loop over members, against the
    regenerating form (exact population in fp64: equal to rounding; population rounded to fp32:
    equal to the rounding of eps), and sigma = 0 gives g_sigma = 0."""
    P, pop, seed = 6, 10, 41
    mu = np.random.default_rng(15).standard_normal(P)
    sigma = np.abs(np.random.default_rng(16).standard_normal(P)) + 0.1
    z = philox.pair_noise(seed, 3, np.arange(pop // 2), P)
    theta = np.empty((pop, P))
    theta[0::2] = mu + sigma * z
    theta[1::2] = mu - sigma * z
    f = np.random.default_rng(17).standard_normal(pop)
    gm, gs = pgpe.gradients_from_population(theta[0::2], mu, sigma, f)
    wm, ws = _textbook_pgpe(theta, mu, sigma, f.tolist())
    np.testing.assert_allclose(gm, wm, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(gs, ws, rtol=1e-10, atol=1e-13)
    rm, rs = pgpe.gradients(z, sigma, f)
    np.testing.assert_allclose(gm, rm, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(gs, rs, rtol=1e-10, atol=1e-13)
    # through tell: a population rounded to fp32 moves the gradient by the rounding of eps only
    P, pop = 301, 16
    mu0 = np.random.default_rng(18).standard_normal(P).astype(np.float32)
    a, b = _state(P, mu0), _state(P, mu0)
    th = pgpe.ask(a, 5, pop)
    pgpe.ask(b, 5, pop)
    f = np.random.default_rng(19).standard_normal(pop).astype(np.float32)
    ga = pgpe.tell(a, f, return_grads=True)
    gb = pgpe.tell(b, f, return_grads=True, stored=th, chunk=100)
    for x, y in zip(ga, gb):
        # theta ~ 1 is stored to half an ulp = 6e-8, eps ~ 0.1: 1e-6 of a term, a few 1e-6 of the rms
        assert np.abs(x - y).max() < 1e-5 * np.sqrt(np.mean(x * x))
    assert np.abs(a.mu - b.mu).max() < 1e-4 and b.t == 2 and b.last is None
    # sigma = 0: the parameter does not move and its sigma gradient is zero
    sg = np.array([0.0, 0.5])
    th = np.array([[1.0, 2.3], [1.0, 1.9]])
    g0, g1 = pgpe.gradients_from_population(th, np.array([1.0, 2.0]), sg, np.array([3.0, 1.0, -2.0, 0.5]))
    assert g0[0] == 0.0 and g1[0] == 0.0 and np.isfinite(g1).all()


def test_gradient_identities():
    P, N = 7, 6
    z = philox.pair_noise(8, 2, np.arange(N), P)
    sigma = np.full(P, 0.3)
    f = np.random.default_rng(8).standard_normal(2 * N)
    gm, gs = pgpe.gradients(z, sigma, f)
    swapped = f.reshape(N, 2)[:, ::-1].reshape(-1)
    gm2, gs2 = pgpe.gradients(z, sigma, swapped)
    np.testing.assert_allclose(gm2, -gm, rtol=1e-12)
    np.testing.assert_allclose(gs2, gs, rtol=1e-12)
    gm3, gs3 = pgpe.gradients(z, sigma, f + 123.0)
    np.testing.assert_allclose(gm3, gm, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(gs3, gs, rtol=1e-9, atol=1e-12)


def test_gradient_expectations_closed_form():
    """Raw fitness: linear f = a.x gives E[g_mu] = sigma^2 a, E[g_sigma] = 0;
    sphere f = -|x|^2 gives E[g_mu] = -2 sigma^2 mu, E[g_sigma] = -2 sigma^3."""
    P, N = 3, 100000
    mu = np.array([0.5, -1.0, 2.0])
    sigma = np.array([0.2, 0.5, 1.0])
    z = philox.pair_noise(2024, 1, np.arange(N), P)
    plus, minus = mu + sigma * z, mu - sigma * z
    a = np.array([1.0, -2.0, 0.5])
    f = np.empty(2 * N)
    f[0::2], f[1::2] = plus @ a, minus @ a
    gm, gs = pgpe.gradients(z, sigma, f)
    tol = 5.0 / np.sqrt(N)
    assert np.abs(gm - sigma ** 2 * a).max() < tol * np.abs(sigma ** 2 * a).max() * 3
    assert np.abs(gs).max() < 1e-9                # (f+ + f-)/2 - b vanishes identically for linear f
    f[0::2], f[1::2] = -(plus ** 2).sum(1), -(minus ** 2).sum(1)
    gm, gs = pgpe.gradients(z, sigma, f)
    assert np.abs(gm - (-2 * sigma ** 2 * mu)).max() < 20 * tol
    assert np.abs(gs - (-2 * sigma ** 3)).max() < 20 * tol
    assert (np.sign(gs) == -1).all()


# ---------------------------------------------------------------- optimiser
def test_adam_first_step_and_constant_gradient():
    g = np.array([1e-3, -2.0, 5e-5, 0.0])
    x, m, v = pgpe.adam_ascent(np.zeros(4), np.zeros(4), np.zeros(4), g, 0.01, 0.9, 0.999, 1e-8, 1)
    np.testing.assert_allclose(x, 0.01 * g / (np.abs(g) + 1e-8), rtol=1e-12)
    x = np.zeros(4)
    m = np.zeros(4)
    v = np.zeros(4)
    for t in range(1, 51):
        x, m, v = pgpe.adam_ascent(x, m, v, g, 0.01, 0.9, 0.999, 1e-8, t)
    np.testing.assert_allclose(x[:3], 0.01 * 50 * np.sign(g[:3]), rtol=3e-4)
    assert x[3] == 0.0


def test_adam_matches_torch_optimizer():
    """torch.optim.Adam minimises; ascent on f equals descent with the negated gradient."""
    rng = np.random.default_rng(9)
    x0 = rng.standard_normal(6)
    p = torch.nn.Parameter(torch.tensor(x0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=0.01, betas=(0.9, 0.999), eps=1e-8)
    x, m, v = x0.copy(), np.zeros(6), np.zeros(6)
    for t in range(1, 8):
        g = rng.standard_normal(6)
        p.grad = torch.tensor(-g)
        opt.step()
        x, m, v = pgpe.adam_ascent(x, m, v, g, 0.01, 0.9, 0.999, 1e-8, t)
        np.testing.assert_allclose(x, p.detach().numpy(), rtol=1e-10, atol=1e-12)


def test_tell_equals_materialised_gradient_and_sigma_rules():
    P, pop, seed = 203, 12, 77
    for rule in (0, 1):
        for shaping in (1, 0):
            mu0 = np.random.default_rng(10).standard_normal(P).astype(np.float32)
            st = _state(P, mu0, sigma_rule=rule, shaping=shaping)
            pgpe.ask(st, seed, pop)
            f = np.random.default_rng(11).standard_normal(pop).astype(np.float32)
            sg0 = st.sigma.astype(np.float64).copy()
            g_mu, g_sg = pgpe.tell(st, f, chunk=64, return_grads=True)
            z = philox.pair_noise(seed, 1, np.arange(pop // 2), P)
            c = pgpe.centered_rank(f)[1] if shaping else f
            wm, ws = pgpe.gradients(z, sg0, c)
            np.testing.assert_allclose(g_mu, wm, rtol=1e-12, atol=1e-15)
            np.testing.assert_allclose(g_sg, ws, rtol=1e-12, atol=1e-15)
            # first Adam step is lr * sign(g) (up to eps)
            np.testing.assert_allclose(st.mu - mu0, 0.01 * np.sign(wm), rtol=0, atol=2e-4)
            assert st.t == 2 and st.last is None
            if rule == 0:
                step = st.sigma.astype(np.float64) - sg0
                np.testing.assert_allclose(step, np.clip(0.1 * ws, -0.2 * sg0, 0.2 * sg0), atol=1e-8)
                assert (np.abs(step) <= 0.2 * sg0 + 1e-8).all() and (st.sigma > 0).all()
            else:
                np.testing.assert_allclose(st.sigma.astype(np.float64) - sg0, 0.1 * np.sign(ws), atol=2e-3)
                assert (st.sigma >= np.float32(1e-8)).all()
    with pytest.raises(RuntimeError):
        pgpe.tell(st, f)


def test_pgpe_converges_on_sphere():
    P = 20
    mu0 = np.full(P, 1.5, np.float32)
    st = _state(P, mu0, lr_mu=0.05)
    hist = []
    for g in range(200):
        th = pgpe.ask(st, 4242, 32)
        f = -(th.astype(np.float64) ** 2).sum(1)
        pgpe.tell(st, f.astype(np.float32))
        hist.append(-(st.mu.astype(np.float64) ** 2).sum())
    assert hist[0] < -40 and hist[-1] > -0.5
    quart = [np.mean(hist[i:i + 50]) for i in range(0, 200, 50)]
    assert quart[0] < quart[1] < quart[2] <= quart[3] + 0.2


def test_clipup_closed_forms():
    """ClipUp pins: first step has length `step` along g; the speed never exceeds max_speed and a
    constant gradient drives it to min(step / (1 - momentum), max_speed); only the direction of the
    gradient matters; a zero gradient only lets the velocity decay."""
    rng = np.random.default_rng(11)
    g = rng.standard_normal(50)
    x0 = rng.standard_normal(50)
    x1, v1 = pgpe.clipup_ascent(x0, np.zeros(50), g, 0.01, 0.9, 0.02)
    np.testing.assert_allclose(x1 - x0, 0.01 * g / np.linalg.norm(g), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(np.linalg.norm(v1), 0.01, rtol=1e-12)
    # scale invariance (any positive factor) and sign equivariance
    x1b, v1b = pgpe.clipup_ascent(x0, np.zeros(50), 7.0 * g, 0.01, 0.9, 0.02)
    np.testing.assert_allclose(v1b, v1, rtol=1e-12, atol=1e-18)
    _, v1c = pgpe.clipup_ascent(x0, np.zeros(50), -g, 0.01, 0.9, 0.02)
    np.testing.assert_allclose(v1c, -v1, rtol=1e-12, atol=1e-18)
    # constant gradient: unclipped speed is the geometric sum step (1 - m^T) / (1 - m); clipped at max_speed
    for max_speed, want in ((1.0, 0.01 * (1 - 0.9 ** 40) / 0.1), (0.02, 0.02)):
        x, v = x0.copy(), np.zeros(50)
        for _ in range(40):
            x, v = pgpe.clipup_ascent(x, v, g, 0.01, 0.9, max_speed)
            assert np.linalg.norm(v) <= max_speed * (1 + 1e-12)
        np.testing.assert_allclose(np.linalg.norm(v), want, rtol=1e-10)
        np.testing.assert_allclose(v / np.linalg.norm(v), g / np.linalg.norm(g), rtol=1e-9, atol=1e-12)
    # zero gradient: no division by zero, the velocity decays by the momentum
    x2, v2 = pgpe.clipup_ascent(x1, v1, np.zeros(50), 0.01, 0.9, 0.02)
    np.testing.assert_allclose(v2, 0.9 * v1, rtol=1e-15)
    np.testing.assert_allclose(x2, x1 + 0.9 * v1, rtol=1e-15)
    # the clip is a projection: a velocity that would be three times too fast comes out at max_speed, same direction
    _, v3 = pgpe.clipup_ascent(x0, np.zeros(50), g, 0.06, 0.9, 0.02)
    np.testing.assert_allclose(v3, 0.02 * g / np.linalg.norm(g), rtol=1e-12, atol=1e-18)


def test_momentum_ascent_closed_form_and_torch():
    rng = np.random.default_rng(12)
    g = rng.standard_normal(20)
    x, v = np.zeros(20), np.zeros(20)
    for T in range(1, 8):
        x, v = pgpe.momentum_ascent(x, v, g, 0.05, 0.9)
        np.testing.assert_allclose(v, 0.05 * g * (1 - 0.9 ** T) / 0.1, rtol=1e-12)
    # torch's SGD keeps the velocity before the learning rate: identical trajectory for a constant rate
    p = torch.zeros(20, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=0.05, momentum=0.9, maximize=True)
    x, v = np.zeros(20), np.zeros(20)
    for it in range(5):
        gi = rng.standard_normal(20)
        p.grad = torch.from_numpy(gi.copy())
        opt.step()
        x, v = pgpe.momentum_ascent(x, v, gi, 0.05, 0.9)
        np.testing.assert_allclose(p.detach().numpy(), x, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("optimizer", [1, 2])
def test_tell_with_other_optimizers_uses_the_same_gradient(optimizer):
    P, pop = 40, 8
    mu0 = np.linspace(-1, 1, P).astype(np.float32)
    a = pgpe.PGPEState.create(pgpe.PGPEConfig(P=P, pop_max=pop), mu0)
    b = pgpe.PGPEState.create(pgpe.PGPEConfig(P=P, pop_max=pop, optimizer=optimizer), mu0)
    f = np.random.default_rng(3).standard_normal(pop).astype(np.float32)
    pgpe.ask(a, 5, pop)
    pgpe.ask(b, 5, pop)
    ga, sa = pgpe.tell(a, f, return_grads=True)
    gb, sb = pgpe.tell(b, f, return_grads=True)
    assert np.array_equal(ga, gb) and np.array_equal(sa, sb)
    assert np.array_equal(a.sigma, b.sigma)          # the sigma rule does not depend on the optimizer of mu
    if optimizer == 1:
        want, vel = pgpe.clipup_ascent(mu0.astype(np.float64), np.zeros(P), gb, b.cfg.lr_mu, b.cfg.momentum, b.cfg.max_speed)
    else:
        want, vel = pgpe.momentum_ascent(mu0.astype(np.float64), np.zeros(P), gb, b.cfg.lr_mu, b.cfg.momentum)
    assert np.array_equal(b.mu, want.astype(np.float32)) and np.array_equal(b.m, vel.astype(np.float32))
    assert not np.array_equal(a.mu, b.mu)
