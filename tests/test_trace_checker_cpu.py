"""The per-step checker of the cart-pole trace (tests/test_gpu_cartpole_trace.py) on the CPU: it accepts
a trace produced by stepping the oracle with binary32 states, and it catches planted mistakes (a wrong
sign in the dynamics, a clip in place of the last tanh, a reward taken at the old state, an episode that keeps running beyond the track)."""
import numpy as np
import pytest

from oracle import policy as opolicy, tasks as otasks
from workloads import CONFIGS, generators as gen

from test_gpu_cartpole_trace import check_trace, mlp_param_count

CP = CONFIGS["cfg3"].cartpole[:6] + (0.02, 0.45)


def make_trace(params, dims, acts, R, steps, seed, t, cp, step_fn=otasks.cartpole_step, reward_at_old=False,
               never_dies=False, act_fn=None):
    n = params.shape[0]
    trace = np.zeros((n, R, steps, 12), dtype=np.float32)
    s = np.broadcast_to(otasks.cartpole_reset(seed, t, R), (n, R, 4)).astype(np.float32)
    alive = np.ones((n, R), dtype=bool)
    run = np.zeros((n, R), dtype=np.float32)
    for k in range(steps):
        lin = opolicy.mlp_forward(params, otasks.cartpole_obs(s.astype(np.float64)), dims,
                                  tuple(acts[:-1]) + (0,))[..., 0].astype(np.float32)
        a = (act_fn or opolicy._act)(lin.astype(np.float64), acts[-1])
        nxt, _ = step_fn(s.astype(np.float64), a, cp)
        nxt = nxt.astype(np.float32)
        r = otasks.cartpole_reward(s if reward_at_old else nxt).astype(np.float32)
        trace[:, :, k, 0:4] = s
        trace[:, :, k, 4] = lin
        trace[:, :, k, 5] = a
        trace[:, :, k, 6] = r
        trace[:, :, k, 7] = alive
        run = np.where(alive, (run.astype(np.float64) + r).astype(np.float32), run)
        trace[:, :, k, 8] = run
        s = np.where(alive[..., None], nxt, s)
        if not never_dies:
            alive = alive & (np.abs(nxt[..., 0]) <= np.float32(cp[7]))
    return trace, s.copy(), run.copy(), run.astype(np.float64).mean(axis=1).astype(np.float32)


@pytest.fixture(scope="module")
def case():
    dims, acts = (5, 16, 16, 1), (1, 1, 1)
    params = gen.random_params(26, 4, mlp_param_count(dims), 1.5)
    return params, dims, acts


def test_checker_accepts_the_oracle_stepped_in_binary32(case):
    params, dims, acts = case
    tr, fin, ret, fit = make_trace(params, dims, acts, 16, 60, 31, 2, CP)
    info = check_trace(params, dims, acts, tr, fin, ret, fit, 31, 2, CP, 0.2, "self")
    assert 0.05 < info["dead"] < 0.95
    assert info["states"] < 1e-6 and info["actions"] < 1e-6


def test_checker_catches_planted_mistakes(case):
    params, dims, acts = case

    def wrong_sign(s, a, cp):        # friction pushing instead of braking
        return otasks.cartpole_step(s, a, cp[:4] + (-cp[4],) + cp[5:])

    def hard_tanh(x, code):          # a clip in place of the last tanh
        return np.clip(x, -1.0, 1.0)

    small = params * 0.05            # actions of a few percent, where the two differ by 1e-5 and more
    tr, fin, ret, fit = make_trace(small, dims, acts, 16, 60, 31, 2, CP, act_fn=hard_tanh)
    with pytest.raises(AssertionError):
        check_trace(small, dims, acts, tr, fin, ret, fit, 31, 2, CP, 0.2, "hard tanh")
    for kw in (dict(step_fn=wrong_sign), dict(reward_at_old=True), dict(never_dies=True)):
        tr, fin, ret, fit = make_trace(params, dims, acts, 16, 60, 31, 2, CP, **kw)
        with pytest.raises(AssertionError):
            check_trace(params, dims, acts, tr, fin, ret, fit, 31, 2, CP, 0.2, str(kw))
