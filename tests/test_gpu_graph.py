"""GPU tests of the device-resident generation index: the same numbers as with the index on the
host, and one generation (ask -> rollout -> tell) recorded in a HIP graph whose every replay is the
next generation, bit for bit what direct calls produce."""
import numpy as np
import pytest

from workloads import CONFIGS, generators as gen
from tests.util import dev, host

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

SEED = 20220509


@pytest.fixture(scope="module")
def evo():
    import paper_2202_05008_amd as e
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return e


class _Run:
    """PGPE state + buffers + a task of one small workload; generation() issues ask, rollout, tell."""

    def __init__(self, evo, kind, device_t, optimizer=None):
        self.evo = evo
        c = CONFIGS[{"classify": "cfg1", "cartpole": "cfg3", "forage": "forage", "forage_solo": "forage"}[kind]]
        self.c, self.kind = c, kind
        self.pop = c.pop if kind == "classify" else 64
        self.steps = {"classify": 1, "cartpole": 20, "forage": 12, "forage_solo": 12}[kind]
        kw = {} if optimizer is None else {"optimizer": optimizer}
        self.pg = evo.PGPE(evo.make_pgpe_config(P=c.P, pop_max=self.pop, **kw), gen.initial_mu(c.data_seed, c.P))
        self.gen_dev = self.pg.device_generation() if device_t else None
        self.pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
        self.params = torch.empty(self.pop, c.P, dtype=torch.float32, device="cuda")
        self.fitness = torch.empty(self.pop, dtype=torch.float32, device="cuda")
        if kind == "classify":
            x, y = gen.class_blobs(c.data_seed, c.B, c.dims[0], c.dims[-1])
            self.x, self.y = dev(x), dev(y)
            td = evo.make_task_desc(evo.EVO_TASK_CLASSIFY, B=c.B, obs=self.x, target=self.y)
            n = evo.rollout_workspace_bytes(td, self.pd, self.pop)
            self.work = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
            self.td = evo.make_task_desc(evo.EVO_TASK_CLASSIFY, B=c.B, obs=self.x, target=self.y, work=self.work)

        if kind in ("forage", "forage_solo"):
            task_kind = evo.EVO_TASK_FORAGE if kind == "forage" else evo.EVO_TASK_FORAGE_SOLO
            cp = tuple(c.world[:4]) + (0.125,) + tuple(c.world[5:])        # a wide touch radius: rewards within 12 steps
            self.make = lambda t, work: evo.make_task_desc(task_kind, n_rollouts=3, reset_seed=SEED + 1,
                                                           generation=t, cp=cp, work=work, generation_dev=self.gen_dev)
            n = evo.rollout_workspace_bytes(self.make(1, None), self.pd, self.pop)
            self.work = torch.empty(n, dtype=torch.uint8, device="cuda")

    def task(self, t):
        if self.kind == "classify":
            return self.td
        if self.kind in ("forage", "forage_solo"):
            return self.make(t, self.work)
        return self.evo.make_task_desc(self.evo.EVO_TASK_CARTPOLE, n_rollouts=self.c.n_rollouts, reset_seed=SEED + 1,
                                       generation=t, cp=self.c.cartpole, init_scale=self.c.init_scale,
                                       generation_dev=self.gen_dev)

    def generation(self, t):
        self.pg.ask(SEED, self.pop, self.params)
        self.evo.rollout(self.task(t), self.pd, self.params, self.pop, self.steps, self.fitness)
        self.pg.tell(self.fitness)

    def snapshot(self):
        return [host(a).copy() for a in (self.pg.mu, self.pg.sigma, self.fitness, self.params)]


def _same_bits(a, b, what):
    for name, p, q in zip(("mu", "sigma", "fitness", "params"), a, b):
        assert np.array_equal(p.view(np.uint32), q.view(np.uint32)), "%s: %s differs" % (what, name)


@pytest.mark.parametrize("kind", ["classify", "cartpole", "forage", "forage_solo"])
def test_device_generation_matches_host_generation(evo, kind):
    a, b = _Run(evo, kind, False), _Run(evo, kind, True)
    for t in range(1, 7):
        a.generation(t), b.generation(0)          # in device mode the task's host-side t is not used
        if kind in ("forage", "forage_solo"):     # whole-number rewards: the worlds of generation t, or not
            assert np.array_equal(host(a.fitness), host(b.fitness)) and np.abs(host(a.fitness)).sum() > 0
            continue
        sa, sb = a.snapshot(), b.snapshot()
        # the noise, the roll-outs and the ranks are the same bits; only Adam's bias corrections are formed
        # on the device (same formula, the device's pow): allow one rounding of those two factors
        assert np.array_equal(sa[3].view(np.uint32), sb[3].view(np.uint32)) or t > 1
        np.testing.assert_allclose(sb[0], sa[0], rtol=0, atol=2e-7 * float(np.abs(sa[0]).max()) * t)
        np.testing.assert_allclose(sb[1], sa[1], rtol=1e-6)
        np.testing.assert_allclose(sb[2], sa[2], rtol=1e-4, atol=1e-5)
    assert a.pg.generation == b.pg.generation == 7
    with pytest.raises(evo.EvoError):
        evo.pgpe_set_generation(b.pg.handle, 3)


@pytest.mark.parametrize("kind,optimizer", [("classify", None), ("cartpole", None), ("classify", "clipup"),
                                            ("forage", None), ("forage_solo", None)])
def test_graph_replays_are_successive_generations(evo, kind, optimizer):
    opt = None if optimizer is None else evo.EVO_OPT_CLIPUP
    warm = _Run(evo, kind, True, opt)
    warm.generation(0)                            # every kernel has run once before anything is recorded
    torch.cuda.synchronize()
    eager, rec = _Run(evo, kind, True, opt), _Run(evo, kind, True, opt)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rec.generation(0)                         # recorded, not run: the device index still says 1
    assert rec.pg.generation == 1
    scratch = torch.zeros(1 << 20, device="cuda")
    for t in range(1, 7):
        graph.replay()
        scratch.add_(1.0)                         # the program's own eager work between replays
        assert float(scratch.sum()) == float(t) * (1 << 20)
        eager.generation(0)
        torch.cuda.synchronize()
        _same_bits(rec.snapshot(), eager.snapshot(), "replay %d" % t)
    assert rec.pg.generation == eager.pg.generation == 7
    # the state is an ordinary one afterwards: direct calls continue the run
    rec.generation(0), eager.generation(0)
    _same_bits(rec.snapshot(), eager.snapshot(), "direct call after the replays")
    blob = rec.pg.export_state()
    assert blob == eager.pg.export_state()
