"""pgpe_ask_rollout / evo_ask_forward: ask fused into the bfloat16 forward, one workgroup per antithetic pair,
the population never stored (Section 4's ask feeding Section 2's global policy).

Two gates.  (1) Against the materialised path of the same library -- pgpe_ask in bfloat16, then rollout /
pop_forward -- the fused results must be bit-identical: the draws are rounded as ask rounds them and the
products follow the streaming kernel's order.  (2) Against the oracle -- ask(bf16) followed by mlp_forward in
fp64 -- at the 2e-2 of the bfloat16 paths."""
import numpy as np
import pytest
import torch

from oracle import pgpe as opgpe, policy as opolicy, tasks as otasks
from workloads import CONFIGS, generators as gen

from util import assert_close, assert_scalar_rel, adam_ill_conditioned, dev, host

pytestmark = pytest.mark.gpu

DIMS = (64, 256, 256, 16)
P = sum(DIMS[i] * DIMS[i + 1] + DIMS[i + 1] for i in range(3))


@pytest.fixture(scope="module")
def evo():
    import paper_2202_05008_amd as evo
    return evo


@pytest.mark.parametrize("acts,pop,B,generations", [((2, 2, 0), 6, 64, 3), ((2, 2, 0), 4, 40, 1), ((1, 2, 0), 2, 1, 2),
                                                     ((2, 1, 1), 8, 33, 1)])
def test_fused_equals_materialised_and_oracle(evo, acts, pop, B, generations):
    seed = 20220509
    mu0 = gen.initial_mu(4, P, 0.06)
    g = evo.PGPE(evo.make_pgpe_config(P=P, pop_max=pop), mu0)
    o = opgpe.PGPEState.create(opgpe.PGPEConfig(P=P, pop_max=pop), mu0)
    obs, tgt = gen.teacher_regression(21, pop, B, DIMS)
    od, tg = dev(obs), dev(tgt)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, DIMS, acts, evo.EVO_BF16)
    td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=B, obs=od, obs_member_stride=B * DIMS[0], target=tg)
    params = torch.empty(pop, P, dtype=torch.bfloat16, device="cuda")
    ill = np.zeros(P, dtype=bool)      # elements on which Adam's sign-like early steps are ill-conditioned, so far
    for t in range(generations):
        # the hook first: it leaves no pending ask behind
        out_fused = torch.full((pop, B, DIMS[-1]), np.nan, dtype=torch.float32, device="cuda")
        evo.evo_ask_forward(g.handle, seed, pop, pd, od, B * DIMS[0], out_fused, B)
        with pytest.raises(evo.EvoError):
            g.tell(torch.zeros(pop, device="cuda"))
        # materialised: ask, forward, fitness
        g.ask(seed, pop, params, evo.EVO_BF16)
        out_mat = torch.full_like(out_fused, np.nan)
        evo.pop_forward(pd, params, od, B * DIMS[0], out_mat, pop, B)
        fit_mat = torch.full((pop,), np.nan, dtype=torch.float32, device="cuda")
        evo.rollout(td, pd, params, pop, 1, fit_mat)
        # fused: records the same pending ask again
        fit_fused = torch.full((pop,), np.nan, dtype=torch.float32, device="cuda")
        g.ask_rollout(seed, pop, td, pd, fit_fused)
        assert torch.equal(out_fused, out_mat), "generation %d: fused outputs differ from ask + pop_forward" % (t + 1)
        assert torch.equal(fit_fused, fit_mat), "generation %d: fused fitness differs from ask + rollout" % (t + 1)
        # the oracle: its own bfloat16 population, fp64 forward
        ref_params = opgpe.ask(o, seed, pop, opgpe.DT_BF16)
        ref_out = opolicy.mlp_forward(ref_params, obs, DIMS, acts)
        got = host(out_fused)
        for m in range(pop):
            assert np.abs(got[m] - ref_out[m]).max() <= 2e-2 * np.abs(ref_out[m]).max(), "member %d" % m
        ref_fit = otasks.regress_fitness(ref_out, tgt)
        assert_scalar_rel(host(fit_fused), ref_fit, 2e-2, "fused fitness")
        # both sides tell the oracle's fitness: the fused call left a pending ask that tell consumes
        f32 = ref_fit.astype(np.float32)
        g.tell(dev(f32))
        g_mu, _ = opgpe.tell(o, f32, return_grads=True)
        ill |= adam_ill_conditioned(g_mu, o.cfg.eps)
        ok = ~ill
        assert ok.mean() > 0.97
        assert_close(host(g.mu)[ok], o.mu[ok], 1e-5, "mu after tell %d" % (t + 1))
        assert_close(host(g.sigma), o.sigma, 1e-5, "sigma after tell %d" % (t + 1))
    assert g.generation == o.t == generations + 1


def test_fused_refuses_what_it_does_not_cover(evo):
    pop, B = 4, 8
    g = evo.PGPE(evo.make_pgpe_config(P=P, pop_max=pop))
    obs = torch.zeros(pop, B, 64, device="cuda")
    tgt = torch.zeros(pop, B, 16, device="cuda")
    fit = torch.zeros(pop, device="cuda")
    td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=B, obs=obs, obs_member_stride=B * 64, target=tgt)
    f32 = evo.make_policy_desc(evo.EVO_POLICY_MLP, DIMS, (2, 2, 0), evo.EVO_F32)
    other = evo.make_policy_desc(evo.EVO_POLICY_MLP, (64, 128, 128, 16), (2, 2, 0), evo.EVO_BF16)
    bf = evo.make_policy_desc(evo.EVO_POLICY_MLP, DIMS, (2, 2, 0), evo.EVO_BF16)
    for pd, task, code in ((f32, td, -3), (other, td, -1),
                           (bf, evo.make_task_desc(evo.EVO_TASK_CLASSIFY, B=B, obs=obs, target=tgt), -3),
                           (bf, evo.make_task_desc(evo.EVO_TASK_REGRESS, B=100, obs=obs, obs_member_stride=100 * 64,
                                                   target=tgt), -3)):
        with pytest.raises(evo.EvoError) as e:
            g.ask_rollout(1, pop, task, pd, fit)
        assert e.value.code == code
    with pytest.raises(evo.EvoError):
        g.ask_rollout(1, 3, td, bf, fit)          # odd population
    with pytest.raises(evo.EvoError):
        g.tell(fit)                               # none of the refused calls left a pending ask


def test_fused_full_size_equals_materialised(evo):
    """cfg4 at full size: the fused generation gives the fitness of ask + rollout, bit for bit."""
    c = CONFIGS["cfg4"]
    seed = 11
    g = evo.PGPE(evo.make_pgpe_config(P=c.P, pop_max=c.pop), gen.initial_mu(c.data_seed, c.P))
    obs, tgt = gen.teacher_regression(c.data_seed, c.pop, c.B, c.dims)
    od, tg = dev(obs), dev(tgt)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts, evo.EVO_BF16)
    td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=c.B, obs=od, obs_member_stride=c.B * c.dims[0], target=tg)
    params = torch.empty(c.pop, c.P, dtype=torch.bfloat16, device="cuda")
    fit_mat = torch.empty(c.pop, dtype=torch.float32, device="cuda")
    fit_fused = torch.full((c.pop,), np.nan, dtype=torch.float32, device="cuda")
    g.ask(seed, c.pop, params, evo.EVO_BF16)
    evo.rollout(td, pd, params, c.pop, 1, fit_mat)
    g.ask_rollout(seed, c.pop, td, pd, fit_fused)
    assert torch.equal(fit_fused, fit_mat)
    assert np.isfinite(host(fit_fused)).all()
