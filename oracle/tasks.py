"""CPU ORACLE (test infrastructure, not part of the product path) -- tasks and fitness.

Tasks are stateless functions of a carried state (Section 4, "Experimenting with More
Tasks": reset(keys) / step); supervised problems are single-step tasks (Section 3,
"Supervised Learning Tasks") and control tasks run a roll-out loop (Section 3, "Control
Tasks").  All members start a roll-out from identical observations (Section 4,
"Exploring Novel Policy Architectures").  The paper prints no loss, reward or dynamics;
the definitions below are this build's reading.

  classify :  fitness = -mean_b CE(softmax(logits_b), y_b)
  regress  :  fitness = -mean_{b,a} (out - target)^2
  sphere   :  fitness = -sum_i (theta_i - x*_i)^2
  cart-pole swing-up: uniform rod (mass m, length l) hinged on a cart (mass M), theta from
      upright, viscous friction b on the cart, force F = f_scale * a:
          D       = 4 (M+m) - 3 m cos^2(theta)
          x_dd    = [4 (F - b x_d) + 2 m l theta_d^2 sin(theta) - 3 m g sin(theta) cos(theta)] / D
          theta_dd= [6 (M+m) g sin(theta) - 6 (F - b x_d) cos(theta) - 3 m l theta_d^2 sin(theta) cos(theta)] / (l D)
      explicit Euler with every derivative taken at the old state; observation
      (x, x_d, cos theta, sin theta, theta_d); reward of a step = cos(theta') exp(-x'^2) at the
      NEW state, counted while the episode is alive; the episode dies after a step that
      ends with |x'| > x_limit (that step's reward still counts).  Reset state of roll-out r
      at generation t: (x, x_d, theta - pi, theta_d) = init_scale * (the four normals of the
      Philox counter (0, r, t, TAG_RESET)), identical for every member.
      Member fitness = mean over the roll-outs of the episode return.

fp64 arithmetic.  Pins: tests/test_oracle_tasks.py (Lagrangian energy / momentum
conservation, small-angle period, closed-form losses).
"""
import numpy as np

from . import philox
from .policy import mlp_unpack, _act

CP_DEFAULT = (9.82, 0.5, 0.5, 0.6, 0.1, 10.0, 0.01, 2.4)   # g, M, m, l, b, f_scale, dt, x_limit


def classify_fitness(logits, labels):
    """logits[pop,B,C] fp64, labels[B] -> fitness[pop] = -mean cross-entropy."""
    z = np.asarray(logits, dtype=np.float64)
    zmax = z.max(axis=-1, keepdims=True)
    lse = zmax[..., 0] + np.log(np.exp(z - zmax).sum(axis=-1))
    picked = np.take_along_axis(z, np.asarray(labels, dtype=np.int64)[None, :, None], axis=-1)[..., 0]
    return -(lse - picked).mean(axis=-1)


def regress_fitness(out, target):
    d = np.asarray(out, dtype=np.float64) - np.asarray(target, dtype=np.float64)
    return -(d * d).mean(axis=(-2, -1))


def sphere_fitness(params, x_star):
    d = np.asarray(params, dtype=np.float64) - np.asarray(x_star, dtype=np.float64)[None, :]
    return -(d * d).sum(axis=-1)


def cartpole_derivs(s, action, cp=CP_DEFAULT):
    """(x_dd, theta_dd) at states s[...,4] = (x, x_d, theta, theta_d) under action in [-1,1]."""
    g, M, m, l, b, fs = cp[:6]
    xd, th, thd = s[..., 1], s[..., 2], s[..., 3]
    sn, cs = np.sin(th), np.cos(th)
    Fe = fs * action - b * xd
    D = 4.0 * (M + m) - 3.0 * m * cs * cs
    xdd = (4.0 * Fe + 2.0 * m * l * thd * thd * sn - 3.0 * m * g * sn * cs) / D
    thdd = (6.0 * (M + m) * g * sn - 6.0 * Fe * cs - 3.0 * m * l * thd * thd * sn * cs) / (l * D)
    return xdd, thdd


def cartpole_reward(s):
    """Reward of arriving at states s[...,4]: cos(theta) exp(-x^2)."""
    s = np.asarray(s, dtype=np.float64)
    return np.cos(s[..., 2]) * np.exp(-s[..., 0] ** 2)


def cartpole_step(s, action, cp=CP_DEFAULT):
    """One explicit-Euler step; returns (next state, reward at the new state)."""
    s = np.asarray(s, dtype=np.float64)
    action = np.asarray(action, dtype=np.float64)
    dt = cp[6]
    xdd, thdd = cartpole_derivs(s, action, cp)
    nxt = np.stack([s[..., 0] + dt * s[..., 1], s[..., 1] + dt * xdd,
                    s[..., 2] + dt * s[..., 3], s[..., 3] + dt * thdd], axis=-1)
    return nxt, cartpole_reward(nxt)


def cartpole_obs(s):
    return np.stack([s[..., 0], s[..., 1], np.cos(s[..., 2]), np.sin(s[..., 2]), s[..., 3]], axis=-1)


def cartpole_reset(seed, generation, n_rollouts, init_scale=0.2):
    """s0[R,4]: identical for every member (common random numbers)."""
    z = philox.block_normals(seed, 0, np.arange(n_rollouts), generation, philox.TAG_RESET)
    s0 = init_scale * z
    s0[:, 2] += np.pi
    return s0


def cartpole_energy(s, cp=CP_DEFAULT):
    g, M, m, l = cp[:4]
    xd, th, thd = s[..., 1], s[..., 2], s[..., 3]
    T = 0.5 * (M + m) * xd ** 2 + 0.5 * m * l * xd * thd * np.cos(th) + m * l * l * thd ** 2 / 6.0
    return T + 0.5 * m * g * l * np.cos(th)


def cartpole_momentum(s, cp=CP_DEFAULT):
    _, M, m, l = cp[:4]
    return (M + m) * s[..., 1] + 0.5 * m * l * s[..., 3] * np.cos(s[..., 2])


def cartpole_rollout(params, dims, acts, seed, generation, n_rollouts, steps, cp=CP_DEFAULT,
                     init_scale=0.2, return_details=False):
    """fitness[pop] of MLP policies on the swing-up task (fp64)."""
    params = np.asarray(params, dtype=np.float64)
    pop = params.shape[0]
    layers = [mlp_unpack(params[m], dims) for m in range(pop)]
    Ws = [np.stack([layers[m][i][0] for m in range(pop)]) for i in range(len(dims) - 1)]
    bs = [np.stack([layers[m][i][1] for m in range(pop)]) for i in range(len(dims) - 1)]
    s = np.broadcast_to(cartpole_reset(seed, generation, n_rollouts, init_scale), (pop, n_rollouts, 4)).copy()
    ret = np.zeros((pop, n_rollouts))
    alive = np.ones((pop, n_rollouts), dtype=bool)
    for _ in range(steps):
        h = cartpole_obs(s)
        for W, b, a in zip(Ws, bs, acts):
            h = _act(np.matmul(h, W) + b[:, None, :], a)
        s_new, r = cartpole_step(s, h[..., 0], cp)
        ret += np.where(alive, r, 0.0)
        s = np.where(alive[..., None], s_new, s)
        alive &= np.abs(s_new[..., 0]) <= cp[7]
    fit = ret.mean(axis=1)
    if return_details:
        return fit, ret, s, alive
    return fit
