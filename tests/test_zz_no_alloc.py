"""rollout_static_scratch: the roll-out for callers that cannot allocate (its workspace is a fixed array in
the library's device image) gives, through the C ABI, what rollout gives with a caller-owned workspace --
bit for bit, since the kernels are the same -- on calls in a row of which the later ones are smaller; it
refuses a task whose workspace exceeds the array before launching anything."""
import numpy as np
import pytest
import torch

from workloads import generators as gen

from util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def evo():
    import paper_2202_05008_amd as evo
    return evo


def _both(evo, kind, pd, params, pop, **task):
    td = evo.make_task_desc(kind, **task)
    need = evo.rollout_workspace_bytes(td, pd, pop)
    assert 0 < need <= evo.rollout_static_scratch_bytes()
    work = torch.empty(need, dtype=torch.uint8, device="cuda")
    td_own = evo.make_task_desc(kind, work=work, **task)
    want = torch.full((pop,), np.nan, dtype=torch.float32, device="cuda")
    got = torch.full((pop,), np.nan, dtype=torch.float32, device="cuda")
    evo.rollout(td_own, pd, params, pop, 1, want)
    evo.rollout_static_scratch(td, pd, params, pop, 1, got)        # work_dev is NULL here
    torch.cuda.synchronize()
    assert np.isfinite(host(want)).all()
    assert torch.equal(got, want)
    return host(got)


def test_static_scratch_matches_rollout_on_calls_in_a_row(evo):
    from oracle import policy as opolicy, tasks as otasks
    # a ConvNet classification (partial loss sums per member and chunk), then a smaller one
    pd = evo.make_policy_desc(evo.EVO_POLICY_CONVNET, (28, 8, 16, 10))
    P = evo.policy_param_count(pd)
    for pop, B, seed in ((12, 150, 1), (4, 13, 2)):
        params = gen.random_params(50 + seed, pop, P, 0.1)
        img, y = gen.mnist_shaped_batch(60 + seed, 1, B)
        fit = _both(evo, evo.EVO_TASK_CLASSIFY, pd, dev(params), pop, B=B, obs=dev(img), target=dev(y))
        ref = otasks.classify_fitness(opolicy.convnet_forward(params, img), y)
        assert np.abs(fit - ref).max() <= 1e-5 * np.abs(ref).max()
    # the sphere (partial sums per member and slice of the parameters): large, then small
    for pop, P in ((64, 1 << 16), (6, 4099)):
        params = gen.random_params(70, pop, P, 1.0)
        xs = gen.sphere_target(71, P)
        fit = _both(evo, evo.EVO_TASK_SPHERE, None, dev(params), pop, P=P, target=dev(xs))
        ref = otasks.sphere_fitness(params, xs)
        assert np.abs(fit - ref).max() <= 1e-5 * np.abs(ref).max()
    # an fp32 MLP classification, and back to the first shape: stale contents of the shared array do not matter
    pdm = evo.make_policy_desc(evo.EVO_POLICY_MLP, (16, 32, 4), (1, 0))
    x, y = gen.class_blobs(80, 300, 16, 4)
    _both(evo, evo.EVO_TASK_CLASSIFY, pdm, dev(gen.random_params(81, 10, 676, 0.3)), 10, B=300, obs=dev(x),
          target=dev(y))
    params = gen.random_params(51, 12, evo.policy_param_count(pd), 0.1)
    img, y = gen.mnist_shaped_batch(61, 1, 150)
    _both(evo, evo.EVO_TASK_CLASSIFY, pd, dev(params), 12, B=150, obs=dev(img), target=dev(y))


def test_static_scratch_refuses_what_does_not_fit(evo):
    P, pop = 1 << 20, 16384
    td = evo.make_task_desc(evo.EVO_TASK_SPHERE, P=P, target=torch.zeros(16, device="cuda"))
    assert evo.rollout_workspace_bytes(td, None, pop) > evo.rollout_static_scratch_bytes()
    fake = torch.zeros(16, device="cuda")
    with pytest.raises(evo.EvoError) as e:
        evo.rollout_static_scratch(td, None, fake, pop, 1, torch.zeros(pop, device="cuda"))
    assert e.value.code == -3 and "built-in scratch" in str(e.value)
