"""GPU parity: Philox stream (bit-exact), normals, ask, centered ranks (bit-exact), tell.
Every expected value comes from oracle/ on the same seeded inputs."""
import numpy as np
import pytest

from oracle import pgpe as opgpe, philox as ophilox, tasks as otasks
from workloads import generators as gen
from tests.util import adam_ill_conditioned, assert_close, assert_scalar_rel, dev, host

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def evo():
    import paper_2202_05008_amd as e
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return e


def _states(evo, P, pop_max, mu0=None, **kw):
    g = evo.PGPE(evo.make_pgpe_config(P=P, pop_max=pop_max, **kw), mu0)
    o = opgpe.PGPEState.create(opgpe.PGPEConfig(P=P, pop_max=pop_max, **kw), mu0)
    return g, o


@pytest.mark.parametrize("seed,t,k,block0,nblocks,tag", [
    (0, 0, 0, 0, 1, 0), (20220509, 1, 0, 0, 1000, 0), (0x0123456789ABCDEF, 7, 511, 12345, 4099, 1),
    (2 ** 64 - 1, 2 ** 32 - 1, 2 ** 32 - 1, 2 ** 32 - 5, 16, 0xFFFFFFFF)])
def test_philox_words_bit_exact(evo, seed, t, k, block0, nblocks, tag):
    out = torch.zeros(4 * nblocks, dtype=torch.int32, device="cuda")
    evo.evo_philox_u32(seed, t, k, block0, nblocks, tag, out)
    got = host(out).view(np.uint32)
    want = ophilox.philox_u32_stream(seed, t, k, block0, nblocks, tag)
    assert np.array_equal(got, want)


def test_philox_normals(evo):
    nblocks = 1 << 16
    out = torch.zeros(4 * nblocks, dtype=torch.float32, device="cuda")
    evo.evo_philox_normal(99, 3, 17, 0, nblocks, 0, out)
    ref = ophilox.pair_noise(99, 3, [17], 4 * nblocks)[0]
    assert_close(host(out), ref, 1e-5, "normals")
    assert np.abs(host(out)).max() < 5.78


@pytest.mark.parametrize("P,pop", [(676, 64), (9098, 16), (4609, 6), (7, 2), (1, 4), (4096, 10)])
def test_ask_fp32(evo, P, pop):
    mu0 = gen.initial_mu(1, P)
    g, o = _states(evo, P, 64, mu0)
    params = torch.empty(pop, P, dtype=torch.float32, device="cuda")
    g.ask(4242, pop, params)
    ref = opgpe.ask(o, 4242, pop)
    assert_close(host(params), ref, 1e-5, "ask")
    # mirrored members share one draw: each is rounded once, so the pair misses 2 mu by at most
    # half an ulp of each member
    th32 = host(params)
    th = th32.astype(np.float64)
    half = 0.5 * (np.spacing(np.abs(th32[0::2])) + np.spacing(np.abs(th32[1::2]))).astype(np.float64)
    assert (np.abs(th[0::2] + th[1::2] - 2.0 * mu0) <= half).all()


def test_ask_invariants(evo):
    P, pop = 1000, 8
    g, _ = _states(evo, P, 8)                      # mu = 0: exact sign flips
    params = torch.empty(pop, P, dtype=torch.float32, device="cuda")
    g.ask(5, pop, params)
    bits = host(params).view(np.uint32)
    assert ((bits[0::2] ^ bits[1::2]) == 0x80000000).all()
    mu0 = gen.initial_mu(2, P)
    g, _ = _states(evo, P, 8, mu0, sigma_init=0.0)  # sigma = 0: theta = mu bit-exactly
    g.ask(5, pop, params)
    assert (host(params).view(np.uint32) == mu0.view(np.uint32)[None, :]).all()
    # a different generation gives different noise; the same (seed, t) reproduces it bit-exactly
    g, _ = _states(evo, P, 8, mu0)
    a = torch.empty_like(params)
    b = torch.empty_like(params)
    g.ask(5, pop, a)
    g.ask(5, pop, b)
    assert torch.equal(a, b)
    evo.pgpe_set_generation(g.handle, 2)
    g.ask(5, pop, b)
    assert not torch.equal(a, b)


@pytest.mark.parametrize("P,pop", [(86544, 6), (1028, 64), (37, 4)])
def test_ask_bf16(evo, P, pop):
    mu0 = gen.initial_mu(3, P)
    g, o = _states(evo, P, 64, mu0)
    params = torch.empty(pop, P, dtype=torch.bfloat16, device="cuda")
    g.ask(77, pop, params, evo.EVO_BF16)
    got = params.to(torch.float32).cpu().numpy()
    ref = opgpe.ask(o, 77, pop, opgpe.DT_BF16)
    # bf16 rounding of a value that differs in the last fp32 bits may pick the neighbour: allow
    # one bf16 ulp on a tiny fraction, exact elsewhere
    diff = got != ref
    assert diff.mean() < 2e-3
    ref32 = opgpe.ask_rows(o, 77, pop)
    floor = 1e-5 * np.sqrt(np.mean(ref32.astype(np.float64) ** 2))      # fp32 tolerance of the unrounded value
    assert (np.abs(got - ref) <= np.abs(ref) * 2.0 ** -7 + floor).all()      # at most one bf16 ulp apart
    assert (np.abs(got - ref32) <= np.abs(ref32) * 2.0 ** -8 + floor).all()  # half an ulp from the fp32 value


@pytest.mark.parametrize("pop,kind", [(2, "plain"), (64, "plain"), (100, "ties"), (257, "specials"), (1024, "ties"),
                                      (4096, "plain"), (4096, "equal"), (3000, "specials")])
def test_centered_rank_bit_exact(evo, pop, kind):
    if kind == "equal":
        f = np.full(pop, -1.5, np.float32)
    else:
        f = gen.random_fitness(pop + 1, pop, ties=5 if kind == "ties" else 0, specials=kind == "specials")
    rank = torch.empty(pop, dtype=torch.int32, device="cuda")
    shaped = torch.empty(pop, dtype=torch.float32, device="cuda")
    evo.evo_centered_rank(dev(f), pop, rank, shaped)
    want_r, want_c = opgpe.centered_rank(f)
    assert np.array_equal(host(rank).view(np.uint32), want_r)
    assert np.array_equal(host(shaped).view(np.uint32), want_c.view(np.uint32))


def _compare_state(g, o, ill, tol=1e-5):
    keep = ~ill
    for name in ("mu", "sigma", "m", "v"):
        got = host(getattr(g, name))[keep]
        ref = getattr(o, name)[keep]
        assert_close(got, ref, tol, name)


@pytest.mark.parametrize("P,pop,rule,shaping", [(676, 64, 0, 1), (676, 64, 1, 1), (9098, 256, 0, 1), (4609, 10, 0, 0),
                                                (7, 2, 1, 0), (20000, 1024, 0, 1), (131072 + 4, 8, 0, 1)])
def test_tell_against_oracle(evo, P, pop, rule, shaping):
    mu0 = gen.initial_mu(4, P)
    # Adam moves sigma by about lr_sigma per step whatever the gradient's size: keep it well below sigma
    kw = {"lr_sigma": 0.005} if rule == 1 else {}
    g, o = _states(evo, P, pop, mu0, sigma_rule=rule, shaping=shaping, **kw)
    params = torch.empty(pop, P, dtype=torch.float32, device="cuda")
    ill = np.zeros(P, dtype=bool)
    for it in range(3):
        seed = 1000 + it
        g.ask(seed, pop, params)
        opgpe.ask(o, seed, pop)
        f = gen.random_fitness(50 + it, pop, ties=4 if it == 1 else 0)
        fd = dev(f)
        gmu = torch.empty(P, dtype=torch.float32, device="cuda")
        gsg = torch.empty(P, dtype=torch.float32, device="cuda")
        evo.evo_pgpe_gradients(g.handle, fd, gmu, gsg)
        g.tell(fd)
        ref_gmu, ref_gsg = opgpe.tell(o, f, return_grads=True)
        assert_close(host(gmu), ref_gmu, 1e-5, "g_mu")
        assert_close(host(gsg), ref_gsg, 1e-5, "g_sigma")
        # Adam's early steps are sign-like: elements whose gradient is below the fp32 noise floor
        # may flip; they are declared ill-conditioned from the ORACLE's gradient and excluded
        ill |= adam_ill_conditioned(ref_gmu, o.cfg.eps)
        if rule == 1:
            ill |= adam_ill_conditioned(ref_gsg, o.cfg.eps)
        assert ill.mean() < 2e-2
        _compare_state(g, o, ill)
        assert g.generation == o.t == it + 2


@pytest.mark.parametrize("P,pop,optimizer,rule", [(676, 64, 1, 0), (676, 64, 2, 0), (70001, 32, 1, 0), (9098, 256, 1, 1),
                                                  (1 << 18, 8, 1, 0), (7, 2, 2, 1)])
def test_tell_clipup_and_momentum_against_oracle(evo, P, pop, optimizer, rule):
    """ClipUp (two global norms) and momentum ascent in tell, five generations: the velocity builds
    up and, for ClipUp, reaches the speed bound (momentum 0.9, max_speed 1.2 lr_mu: two steps in
    unrelated directions already exceed it)."""
    mu0 = gen.initial_mu(6, P)
    kw = {"lr_sigma": 0.005} if rule == 1 else {}
    g, o = _states(evo, P, pop, mu0, sigma_rule=rule, optimizer=optimizer, max_speed=0.012, **kw)
    params = torch.empty(pop, P, dtype=torch.float32, device="cuda")
    clipped = False
    for it in range(5):
        seed = 2000 + it
        g.ask(seed, pop, params)
        opgpe.ask(o, seed, pop)
        f = gen.random_fitness(80 + it, pop)
        g.tell(dev(f))
        opgpe.tell(o, f)
        assert_close(host(g.mu), o.mu, 1e-5, "mu, generation %d" % (it + 1))
        assert_close(host(g.m), o.m, 1e-5, "velocity, generation %d" % (it + 1))
        assert_close(host(g.sigma), o.sigma, 1e-5, "sigma, generation %d" % (it + 1))
        speed = float(np.linalg.norm(host(g.m).astype(np.float64)))
        if optimizer == 1:
            assert speed <= o.cfg.max_speed * (1 + 1e-5)
            clipped |= speed > o.cfg.max_speed * (1 - 1e-5)
        assert g.generation == o.t == it + 2
    if optimizer == 1:
        assert clipped, "five steps at momentum 0.9 must have hit the speed bound"


def test_clipup_zero_gradient_and_config_errors(evo):
    P, pop = 100, 8
    mu0 = gen.initial_mu(7, P)
    g, o = _states(evo, P, pop, mu0, optimizer=1)
    params = torch.empty(pop, P, dtype=torch.float32, device="cuda")
    g.ask(3, pop, params)
    # raw equal fitness with shaping off gives w = u = 0: the gradient is exactly zero
    g2, o2 = _states(evo, P, pop, mu0, optimizer=1, shaping=0)
    g2.ask(3, pop, params)
    g2.tell(dev(np.full(pop, 2.5, np.float32)))
    assert np.array_equal(host(g2.mu), mu0) and not np.isnan(host(g2.m)).any() and (host(g2.m) == 0).all()
    for bad in ({"optimizer": 3}, {"optimizer": 1, "max_speed": 0.0}, {"optimizer": 2, "momentum": 1.0}):
        with pytest.raises(evo.EvoError):
            evo.PGPE(evo.make_pgpe_config(P=P, pop_max=pop, **bad))


@pytest.mark.parametrize("P,pop", [(676, 64), (10007, 10), (4096, 2), (3, 4), (40000, 38), (16384 + 4, 8)])
def test_ask_sphere_fused_against_oracle(evo, P, pop):
    """ask fused with the sphere fitness (no population in memory) against the oracle's ask followed
    by its sphere fitness; several workgroups per row, ragged ends in P and in the pairs."""
    mu0 = gen.initial_mu(11, P)
    x_star = gen.sphere_target(12, P)
    g, o = _states(evo, P, 64, mu0)
    fit = torch.full((pop,), 7.0, dtype=torch.float32, device="cuda")
    for it in range(2):                       # the second generation runs from an updated mu, sigma
        g.ask_sphere(900 + it, pop, dev(x_star), fit)
        ref = otasks.sphere_fitness(opgpe.ask(o, 900 + it, pop), x_star)
        assert_scalar_rel(host(fit), ref, 1e-5, "fused sphere fitness, generation %d" % (it + 1))
        # the materialised path of the library gives the same values up to the order of the sums
        params = torch.empty(pop, P, dtype=torch.float32, device="cuda")
        h, _ = _states(evo, P, 64, host(g.mu).copy())
        h.sigma.copy_(g.sigma)
        evo.pgpe_set_generation(h.handle, it + 1)
        h.ask(900 + it, pop, params)
        td = evo.make_task_desc(evo.EVO_TASK_SPHERE, P=P, target=dev(x_star))
        td = evo.make_task_desc(evo.EVO_TASK_SPHERE, P=P, target=dev(x_star), work=torch.empty(
            max(evo.rollout_workspace_bytes(td, None, pop), 16), dtype=torch.uint8, device="cuda"))
        fit2 = torch.empty(pop, dtype=torch.float32, device="cuda")
        evo.rollout(td, None, params, pop, 1, fit2)
        assert_scalar_rel(host(fit), host(fit2), 2e-6, "fused against materialised")
        f = gen.random_fitness(60 + it, pop)   # the fused call leaves a pending ask like pgpe_ask
        g.tell(dev(f))
        opgpe.tell(o, f)
        assert g.generation == o.t == it + 2
        g.mu.copy_(dev(o.mu))                  # teacher-forced: the next ask starts from the oracle's state
        g.sigma.copy_(dev(o.sigma))
    with pytest.raises(evo.EvoError):
        g.ask_sphere(1, pop + 1, dev(x_star), fit)


@pytest.mark.parametrize("P,pop,rule,shaping,optimizer", [(676, 64, 0, 1, 0), (9098, 256, 1, 1, 0), (4609, 10, 0, 0, 0),
                                                          (7, 2, 0, 1, 2), (20000, 1024, 0, 1, 0),
                                                          (131072 + 4, 8, 0, 1, 1), (1001, 6, 0, 1, 0)])
def test_tell_stored_against_oracle(evo, P, pop, rule, shaping, optimizer):
    """tell with the perturbations read back from the stored population.  The population handed to
    the library is the ORACLE's (uploaded), so that both sides read the same fp32 values."""
    mu0 = gen.initial_mu(13, P)
    kw = {"lr_sigma": 0.005} if rule == 1 else {}
    g, o = _states(evo, P, pop, mu0, sigma_rule=rule, shaping=shaping, optimizer=optimizer, **kw)
    scratch = torch.empty(pop, P, dtype=torch.float32, device="cuda")
    ill = np.zeros(P, dtype=bool)
    for it in range(2):
        seed = 3000 + it
        g.ask(seed, pop, scratch)              # records the pending ask
        theta = opgpe.ask(o, seed, pop)
        params = dev(theta)
        f = gen.random_fitness(90 + it, pop, ties=3 if it == 1 else 0)
        fd = dev(f)
        gmu = torch.empty(P, dtype=torch.float32, device="cuda")
        gsg = torch.empty(P, dtype=torch.float32, device="cuda")
        evo.evo_pgpe_gradients(g.handle, fd, gmu, gsg, params)
        g.tell_stored(fd, params)
        ref_gmu, ref_gsg = opgpe.tell(o, f, return_grads=True, stored=theta)
        assert_close(host(gmu), ref_gmu, 1e-5, "g_mu from the stored population")
        assert_close(host(gsg), ref_gsg, 1e-5, "g_sigma from the stored population")
        if optimizer == 0:
            ill |= adam_ill_conditioned(ref_gmu, o.cfg.eps)
            if rule == 1:
                ill |= adam_ill_conditioned(ref_gsg, o.cfg.eps)
            assert ill.mean() < 2e-2
        if optimizer == 0:
            _compare_state(g, o, ill)
        else:                                  # m holds the velocity; ClipUp uses v as scratch
            for name in ("mu", "sigma", "m"):
                assert_close(host(getattr(g, name)), getattr(o, name), 1e-5, name)
        assert g.generation == o.t == it + 2
        # teacher-forced: eps = theta - mu is taken against the library's own mu, so a mu that differs
        # from the oracle's within its tolerance (1e-5 |mu|) would enter eps ~ sigma amplified by 1 / sigma
        g.mu.copy_(dev(o.mu)), g.sigma.copy_(dev(o.sigma)), g.m.copy_(dev(o.m)), g.v.copy_(dev(o.v))
        if rule == 1:
            g.aux.copy_(dev(np.concatenate([o.m_sigma, o.v_sigma])))
    with pytest.raises(evo.EvoError) as ei:
        g.tell_stored(fd, params)
    assert ei.value.code == -2


def test_tell_errors_and_determinism(evo):
    P, pop = 5000, 128
    g, _ = _states(evo, P, pop)
    f = dev(gen.random_fitness(1, pop))
    with pytest.raises(evo.EvoError) as ei:
        g.tell(f)
    assert ei.value.code == -2
    params = torch.empty(pop, P, dtype=torch.float32, device="cuda")
    with pytest.raises(evo.EvoError):
        g.ask(1, pop + 2, params)
    with pytest.raises(evo.EvoError):
        g.ask(1, pop - 1, params)
    outs = []
    for _ in range(2):
        h, _ = _states(evo, P, pop, gen.initial_mu(9, P))
        h.ask(3, pop, params)
        h.tell(f)
        outs.append((host(h.mu).copy(), host(h.sigma).copy(), host(h.v).copy()))
    for a, b in zip(*outs):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
