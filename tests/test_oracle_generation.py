"""oracle/generation.py on the CPU: `evaluate` is glue (it routes a task to the policy and the loss / the
roll-out), so it is pinned against the pieces it strings together computed by other means (torch's functional
network and losses, the closed forms, the roll-out's own brute-force pins), and `run_generation` against the
sequence ask -> evaluate -> tell spelled out, on every kind of task the five configurations use."""
import numpy as np
import torch

from oracle import generation as ogen, pgpe as opgpe, policy as opolicy, tasks as otasks
from workloads import generators as gen


def _torch_mlp(theta, x, dims, acts):
    h = torch.from_numpy(np.asarray(x, dtype=np.float64))
    o = 0
    for i, a in enumerate(acts):
        n_in, n_out = dims[i], dims[i + 1]
        W = torch.from_numpy(theta[o:o + n_in * n_out].astype(np.float64).reshape(n_in, n_out))
        o += n_in * n_out
        b = torch.from_numpy(theta[o:o + n_out].astype(np.float64))
        o += n_out
        h = h @ W + b
        h = torch.tanh(h) if a == 1 else torch.relu(h) if a == 2 else h
    return h


def test_evaluate_classify_and_regress_against_torch():
    dims, acts, pop, B = (16, 32, 4), (1, 0), 6, 40
    P = sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(len(dims) - 1))
    params = gen.random_params(1, pop, P, 0.4)
    x, y = gen.class_blobs(2, B, dims[0], dims[-1])
    fit = ogen.evaluate({"kind": "classify", "dims": dims, "acts": acts, "obs": x, "labels": y}, params, 0, 1)
    for m in range(pop):
        ce = torch.nn.functional.cross_entropy(_torch_mlp(params[m], x, dims, acts), torch.from_numpy(y).long())
        assert abs(fit[m] + float(ce)) < 1e-12
    # per-member observations and targets: the mean squared error of every member on its own batch
    obs, tgt = gen.teacher_regression(3, pop, B, dims)
    fit = ogen.evaluate({"kind": "regress", "dims": dims, "acts": acts, "obs": obs, "targets": tgt}, params, 0, 1)
    for m in range(pop):
        mse = torch.nn.functional.mse_loss(_torch_mlp(params[m], obs[m], dims, acts),
                                           torch.from_numpy(tgt[m].astype(np.float64)))
        assert abs(fit[m] + float(mse)) < 1e-12
    # zero parameters: uniform logits, fitness = -ln(classes) whatever the data
    zero = np.zeros((2, P), dtype=np.float32)
    fit = ogen.evaluate({"kind": "classify", "dims": dims, "acts": acts, "obs": x, "labels": y}, zero, 0, 1)
    assert np.allclose(fit, -np.log(4.0), atol=1e-15)


def test_evaluate_convnet_sphere_and_cartpole_route_to_their_definitions():
    pop, B = 3, 5
    params = gen.random_params(4, pop, 9098, 0.2)
    img, y = gen.mnist_shaped_batch(5, 1, B)
    fit = ogen.evaluate({"kind": "classify", "convnet": True, "dims": (8, 16, 10), "obs": img, "labels": y}, params, 0, 1)
    logits = opolicy.convnet_forward(params, img, 8, 16, 10)
    want = [-float(torch.nn.functional.cross_entropy(torch.from_numpy(logits[m]), torch.from_numpy(y).long()))
            for m in range(pop)]
    assert np.allclose(fit, want, atol=1e-12)
    # sphere: the closed form, and the seed / generation arguments do not enter
    xs = gen.sphere_target(6, 50)
    th = gen.random_params(7, 4, 50, 1.0)
    fit = ogen.evaluate({"kind": "sphere", "x_star": xs}, th, 123, 9)
    assert np.allclose(fit, [-np.sum((th[m].astype(np.float64) - xs) ** 2) for m in range(4)], rtol=1e-15)
    # cart-pole: the seed and the generation select the reset states (other seed or generation: other fitness),
    # the roll-out count and horizon are passed on, and a policy of zeros is the free system
    dims, acts = (5, 16, 1), (1, 1)
    P = 5 * 16 + 16 + 16 + 1
    task = {"kind": "cartpole", "dims": dims, "acts": acts, "n_rollouts": 3, "steps": 25}
    th = gen.random_params(8, 2, P, 0.5)
    th[1] = 0.0
    f = ogen.evaluate(task, th, 11, 2)
    assert np.array_equal(f, otasks.cartpole_rollout(th, dims, acts, 11, 2, 3, 25))
    assert not np.allclose(f, ogen.evaluate(task, th, 12, 2)) and not np.allclose(f, ogen.evaluate(task, th, 11, 3))
    s = otasks.cartpole_reset(11, 2, 3)
    ret = np.zeros(3)
    alive = np.ones(3, dtype=bool)
    for _ in range(25):                      # the free system, stepped by hand
        s_new, r = otasks.cartpole_step(s, np.zeros(3))
        ret += np.where(alive, r, 0.0)
        s = np.where(alive[:, None], s_new, s)
        alive &= np.abs(s_new[:, 0]) <= otasks.CP_DEFAULT[7]
    assert abs(f[1] - ret.mean()) < 1e-12


def test_run_generation_is_ask_evaluate_tell():
    P, pop, seed = 30, 8, 5
    xs = gen.sphere_target(9, P)
    task = {"kind": "sphere", "x_star": xs}
    a = opgpe.PGPEState.create(opgpe.PGPEConfig(P=P, pop_max=pop), gen.initial_mu(10, P))
    b = opgpe.PGPEState.create(opgpe.PGPEConfig(P=P, pop_max=pop), gen.initial_mu(10, P))
    for _ in range(3):
        params, fit = ogen.run_generation(a, task, seed, pop)
        want_params = opgpe.ask(b, seed, pop)
        want_fit = otasks.sphere_fitness(want_params, xs).astype(np.float32)
        opgpe.tell(b, want_fit)
        assert np.array_equal(params, want_params) and np.array_equal(fit, want_fit)
        assert np.array_equal(a.mu, b.mu) and np.array_equal(a.sigma, b.sigma) and a.t == b.t
    assert a.t == 4
