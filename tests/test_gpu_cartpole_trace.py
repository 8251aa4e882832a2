"""Every step of the fused cart-pole roll-out against the fp64 oracle, teacher-forced along the
device's own trajectory (Section 3, "Control Tasks": the roll-out loop; Section 4: reset / step).

Over 1000 chaotic steps an fp32 trajectory leaves the fp64 one, so whole-episode results cannot be
compared element by element.  Each single step can: evo_rollout_trace records, for every (member,
roll-out, step), the state the policy saw, the policy's linear output and the action, the step's
reward, the alive flag and the running return, as the fused kernel used them.  The oracle is then
asked, for every record on its own, what the policy does in that state and where the step leads;
errors cannot pile up, and no summation order of the matrix cores has to be mirrored.

Gates (all 1e-5 by the vector rule |got - ref| <= 1e-5 max(|ref|, rms(ref))):
  reset states; the policy's linear output in the device's state (rms per member: it is the vector the
  contractions produce, and where weights of order one saturate the last tanh its error is what an fp32
  evaluation can hold at 1e-5 -- the squashed action then differs by up to tanh' times that); the last
  activation applied to the device's own linear output (a tanh is formed as a difference from 1 and so
  carries a few roundings of 1: 4 * 2^-23 absolute is allowed besides the relative bound; it enters the
  dynamics as a force, and the state gates below bound its effect); the state after the step under the ORACLE's
  action, and under the device's; the reward at the device's new state; the alive flag (decided on the
  device's own x' in binary32, and on the oracle's x' outside the tolerance of the limit); frozen state
  and return after the end; the running return; the fitness."""
import numpy as np
import pytest
import torch

from oracle import policy as opolicy, tasks as otasks
from workloads import CONFIGS, generators as gen

from util import dev, host

pytestmark = pytest.mark.gpu

CP = CONFIGS["cfg3"].cartpole
TOL = 1e-5


@pytest.fixture(scope="module")
def evo():
    import paper_2202_05008_amd as evo
    return evo


def mlp_param_count(dims):
    return sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(len(dims) - 1))


def run_trace(evo, dims, acts, p_d, pop, R, steps, seed, t, cp=CP, init_scale=0.2):
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    td = evo.make_task_desc(evo.EVO_TASK_CARTPOLE, n_rollouts=R, reset_seed=seed, generation=t, cp=cp,
                            init_scale=init_scale)
    trace = torch.full((pop, R, steps, 12), np.nan, dtype=torch.float32, device="cuda")
    fin = torch.full((pop, R, 4), np.nan, dtype=torch.float32, device="cuda")
    ret = torch.empty(pop, R, dtype=torch.float32, device="cuda")
    fit = torch.empty(pop, dtype=torch.float32, device="cuda")
    evo.evo_rollout_trace(td, pd, p_d, pop, steps, trace, fin)
    evo.evo_rollout_details(td, pd, p_d, pop, steps, ret, None)
    evo.rollout(td, pd, p_d, pop, steps, fit)
    return trace, fin, ret, fit


def worst(got, ref):
    """max |got - ref| / max(|ref|, rms(ref)) (the vector tolerance rule), rms per last-axis component."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    flat = ref.reshape(-1, ref.shape[-1]) if ref.ndim > 1 else ref.reshape(-1, 1)
    rms = np.sqrt((flat * flat).mean(axis=0))
    scale = np.maximum(np.abs(ref), rms if ref.ndim > 1 else rms[0])
    scale = np.where(scale == 0.0, 1.0, scale)
    return float((np.abs(got - ref) / scale).max())


def check_trace(params, dims, acts, trace, fin, ret, fit, seed, t, cp, init_scale, what):
    """params[n,P] fp32 host values of the traced members; trace[n,R,steps,12], fin[n,R,4], ret[n,R], fit[n]."""
    n, R, steps, _ = trace.shape
    assert np.isfinite(trace).all() and np.isfinite(fin).all(), what
    s = trace[..., 0:4]                                        # state before step t
    s_next = np.concatenate([s[:, :, 1:], fin[:, :, None, :]], axis=2)   # state after step t
    lin, action, reward, alive, run = trace[..., 4], trace[..., 5], trace[..., 6], trace[..., 7], trace[..., 8]
    assert (trace[..., 9:] == 0.0).all(), what
    alive_b = alive == 1.0
    assert np.isin(alive, (0.0, 1.0)).all() and alive_b[:, :, 0].all(), what

    # the reset: the same states for every member
    s0 = otasks.cartpole_reset(seed, t, R, init_scale)
    assert worst(s[:, :, 0], np.broadcast_to(s0, (n, R, 4))) <= TOL, what + ": reset states"

    # the policy in the state the device was in: its linear output (per member), then the last activation
    obs = otasks.cartpole_obs(s.astype(np.float64)).reshape(n, R * steps, 5)
    lin_ref = opolicy.mlp_forward(params, obs, dims, tuple(acts[:-1]) + (opolicy.ACT_NONE,))[..., 0].reshape(n, R, steps)
    a_ref = opolicy._act(lin_ref, acts[-1])
    w_l = max(worst(lin[m][alive_b[m]][:, None], lin_ref[m][alive_b[m]][:, None]) for m in range(n))
    act_dev = opolicy._act(lin.astype(np.float64), acts[-1])
    err_act = np.abs(action - act_dev)[alive_b]
    if acts[-1] == opolicy.ACT_TANH:
        err_act = np.maximum(err_act - 4.0 * 2.0 ** -23, 0.0)
    rms_act = np.sqrt((act_dev[alive_b] ** 2).mean())
    w_act = float((err_act / np.maximum(np.maximum(np.abs(act_dev[alive_b]), rms_act), 1e-30)).max())
    w_a = worst(action[alive_b][:, None], a_ref[alive_b][:, None])        # reported, implied by the two above
    # the step from that state under the oracle's action, and under the device's
    nxt_ref, _ = otasks.cartpole_step(s.astype(np.float64), a_ref, cp)
    nxt_dev, _ = otasks.cartpole_step(s.astype(np.float64), action.astype(np.float64), cp)
    r_ref = otasks.cartpole_reward(s_next)                     # the reward is a function of the new state
    w_s = worst(s_next[alive_b], nxt_ref[alive_b])
    w_sd = worst(s_next[alive_b], nxt_dev[alive_b])
    w_r = worst(reward[alive_b][:, None], r_ref[alive_b][:, None])
    print("%s: linear output %.2e, activation %.2e (largest absolute error %.2e), action %.2e, state %.2e "
          "(device action %.2e), reward %.2e"
          % (what, w_l, w_act, float(np.abs(action - act_dev)[alive_b].max()), w_a, w_s, w_sd, w_r))
    assert w_l <= TOL, "%s: the policy's linear output off by %.3g" % (what, w_l)
    assert w_act <= TOL, "%s: last activation off by %.3g" % (what, w_act)
    assert w_s <= TOL, "%s: next states off by %.3g" % (what, w_s)
    assert w_sd <= TOL, "%s: next states under the device's action off by %.3g" % (what, w_sd)
    assert w_r <= TOL, "%s: rewards off by %.3g" % (what, w_r)

    # alive: never set again; cleared by the step that ends beyond the track, decided on the device's own x'
    # in binary32 (the oracle's x' decides too, except within the tolerance of the limit)
    xlim32 = np.float32(cp[7])
    over_dev = np.abs(s_next[..., 0]) > xlim32
    alive_after = np.concatenate([alive_b[:, :, 1:], np.zeros((n, R, 1), dtype=bool)], axis=2)
    inner = np.s_[:, :, :-1]
    assert (alive_after[inner] == (alive_b[inner] & ~over_dev[inner])).all(), what + ": alive flags"
    over_ref = np.abs(nxt_ref[..., 0]) > cp[7]
    clear = np.abs(np.abs(nxt_ref[..., 0]) - cp[7]) > TOL * cp[7]
    assert (over_dev == over_ref)[alive_b & clear].all(), what + ": termination decisions"
    assert (alive_b & ~clear).mean() < 1e-3

    # a dead episode is frozen: state and return stay bit for bit
    dead = ~alive_b
    assert (s_next[dead] == s[dead]).all(), what + ": frozen states"
    prev_run = np.concatenate([np.zeros((n, R, 1), dtype=np.float32), run[:, :, :-1]], axis=2)
    assert (run[dead] == prev_run[dead]).all(), what + ": frozen returns"

    # returns: the running sum of the rewards while alive; fitness: their mean over the roll-outs
    run_ref = np.cumsum(np.where(alive_b, r_ref, 0.0), axis=2)
    assert worst(run.reshape(-1, 1), run_ref.reshape(-1, 1)) <= TOL, what + ": running returns"
    assert (run[:, :, -1] == ret).all(), what + ": the trace and the roll-out details disagree"
    assert worst(fit[:, None], run_ref[:, :, -1].mean(axis=1)[:, None]) <= TOL, what + ": fitness"
    return dict(linear=w_l, activation=w_act, actions=w_a, states=w_s, rewards=w_r, dead=float(dead.mean()))


CASES = [
    # dims, acts, pop, R, steps, weight scale, cart-pole constants
    ((5, 64, 64, 1), (1, 1, 1), 4, 16, 1000, 1e-3, CP),
    ((5, 64, 64, 1), (1, 1, 1), 4, 16, 1000, 0.3, CP),
    ((5, 64, 64, 1), (1, 1, 1), 4, 16, 1000, 1.0, CP),
    ((5, 64, 64, 1), (1, 1, 1), 3, 16, 1000, 3.0, CP),
    ((5, 16, 16, 1), (1, 1, 1), 4, 16, 60, 1.5, CP[:6] + (0.02, 0.45)),     # episodes that end early
    ((5, 32, 32, 1), (1, 2, 1), 3, 5, 400, 0.5, CP),                        # a ReLU layer, five roll-outs
    ((5, 32, 32, 1), (2, 0, 1), 3, 20, 200, 0.3, CP),                       # two passes of sixteen roll-outs
    ((5, 16, 1), (1, 0), 3, 16, 300, 0.5, CP),                              # one hidden layer, unbounded action
    ((5, 64, 1), (1, 1), 2, 7, 1000, 1.0, CP),
    # operands far beyond fp16's own range (the scales of the two-term products are set at run time)
    ((5, 64, 64, 1), (1, 1, 1), 3, 16, 300, "huge", CP),
    ((5, 64, 64, 1), (2, 2, 1), 3, 16, 300, "huge", CP),
    ((5, 32, 32, 1), (0, 2, 1), 3, 16, 300, "huge", CP),
]


def _params(dims, acts, pop, scale):
    """Random parameters; "huge": members whose layer-2 operands lie far outside fp16's range, built so that the
    network stays well conditioned (an fp32 evaluation of sums of thousands that cancel, or of a tanh fed by
    pre-activations of +-1000 that cross zero, is itself off by more than 1e-5 of its output)."""
    P = mlp_param_count(dims)
    if scale != "huge":
        return gen.random_params(26, pop, P, scale)
    H = dims[1]
    params = gen.random_params(26, pop, P, 0.5)
    l2 = slice(5 * H + H, 5 * H + H + H * H)
    params[0, 5 * H + H + 70] = -1.0e5               # one weight of the second layer
    params[2, l2] *= 1.0e-6                          # all of layer 2 tiny next to its ordinary biases
    if acts[0] != 1:
        # unbounded layer-1 activations in the thousands; positive weights behind them, so that the sums of
        # layers 2 and 3 do not cancel; a small output layer brings the action's argument back to order one
        params[1, :5 * H] *= 2000.0
        params[1, 5 * H + H:] = np.abs(params[1, 5 * H + H:])
        params[1, l2.stop + H:l2.stop + 2 * H] *= 1.0e-6
    return params


@pytest.mark.parametrize("dims,acts,pop,R,steps,scale,cp", CASES)
def test_every_step_against_the_oracle(evo, dims, acts, pop, R, steps, scale, cp):
    params = _params(dims, acts, pop, scale)
    if len(dims) == 4 and dims[1] == 16:
        params[3] = 0.0                   # the zero policy: the free system
    seed, t = 31, 2
    trace, fin, ret, fit = run_trace(evo, dims, acts, dev(params), pop, R, steps, seed, t, cp)
    info = check_trace(params, dims, acts, host(trace), host(fin), host(ret), host(fit), seed, t, cp, 0.2,
                       "dims %s acts %s scale %s" % (dims, acts, scale))
    print(info)
    if cp[7] < 1.0:
        assert 0.05 < info["dead"] < 0.95, "the case is meant to have episodes that end early and ones that do not"


def test_the_configured_size_every_step_of_sampled_members(evo):
    """The benchmark's launch (1024 members, 16 roll-outs, 1000 steps): every step of a sample of members."""
    c = CONFIGS["cfg3"]
    seed, t = 11, 2
    params = gen.random_params(3, c.pop, c.P, 0.3)
    trace, fin, ret, fit = run_trace(evo, c.dims, c.acts, dev(params), c.pop, c.n_rollouts, c.steps, seed, t,
                                     c.cartpole, c.init_scale)
    members = np.array([0, 1, 4, 77, 300, 511, 512, 900, 1022, 1023])
    idx = torch.from_numpy(members).cuda()
    info = check_trace(params[members], c.dims, c.acts, host(trace[idx]), host(fin[idx]), host(ret[idx]),
                       host(fit[idx]), seed, t, c.cartpole, c.init_scale, "cfg3")
    print(info)
    # the whole population: the returns of the trace are the returns of the plain roll-out
    assert torch.equal(trace[:, :, -1, 8], ret)
