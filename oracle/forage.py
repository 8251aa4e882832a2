"""CPU ORACLE (test infrastructure, not part of the product path) -- the shared-world task.

Section 3's WaterWorld paragraph describes a training scheme, not rules: the whole population is
spawned in one task roll-out and every agent's performance is measured in that multi-agent world;
an agent collects food and avoids poison.  The paper gives no dynamics, sensors or constants, so
the world below is this build's own definition (a reading, not the original environment's rules):

* World r (r < n_worlds) of generation t: the unit square with every member of the population in
  it as one agent (agent a = member a), F food items and Q poison items (items 0..F-1 are food).
* Reset: agent a starts at (u(x0), u(x1)) of the Philox block with counter
  (a, r, t, TAG_WORLD_AGENT), at rest.  Item i that has been eaten c times lies at (u(x0), u(x1))
  of the block with counter (256 c + i, r, t, TAG_WORLD_ITEM); items do not move.  u is the
  24-bit uniform of the noise generator, so every start position is exact in fp32.
* Observation (8 numbers): own velocity, offset to the nearest food, to the nearest poison and to
  the nearest other agent (offset = other - own, per axis).  Nearest = smallest
  d2 = fl(fl(dx dx) + fl(dy dy)), lowest index among equals.
* Action: the policy's two outputs clipped to [-1, 1].
* Step: v' = clip(fl(fl(drag v) + fl(thrust a)), -vmax, vmax); p' = fl(p + fl(dt v')) per axis; an
  axis that leaves [0, 1] is put on the wall with zero velocity.  Then every item (where it lay at
  the start of the step) with d2(p', item) <= r2 is touched: +1 for food, -1 for poison, for every
  agent that touches it; a touched item is eaten once and lies at its next position from the next
  step on.  Agents interact through the items they take from each other and through what they see.
* Fitness of member a: its summed reward, averaged over the worlds.
* Single-agent form (the same paragraph's first sentence: one agent collecting food and avoiding
  poison): every member lives alone in its own copy of each world -- a world with one agent, agent
  index 0, so all members start at the same place among the same items (identical initial
  observations, Section 4) and part ways through what they eat.  With nobody else around, the offset
  to the nearest other agent is (0, 0).  `rollout_solitary` is that definition spelt out: the
  shared-world roll-out of each member on its own.

Precision: the task fixes the world's arithmetic as IEEE binary32 with every operation rounded on
its own (no fused multiply-add), because it decides integers (who is nearest, who touches); the
policy between observation and action is the fp64 MLP of oracle/policy.py, its output rounded to
binary32 before the clip.  Pins: tests/test_oracle_forage.py (k-d tree and double-loop nearest
neighbours, closed forms of the motion, exact touch geometry, a brute-force count for agents at
rest, the corner reached under a constant action).
"""
import numpy as np

from . import philox
from .policy import mlp_forward

TAG_WORLD_AGENT = 2
TAG_WORLD_ITEM = 3
OBS_DIM = 8
F32 = np.float32

# dt, thrust (velocity gained per step at full action), drag, vmax, touch radius
WORLD_DEFAULT = dict(dt=0.0625, thrust=0.015625, drag=0.875, vmax=0.25, radius=0.03125, n_food=24, n_poison=24)


def _unit(x):
    return philox.u32_to_unit(x).astype(F32)      # (2k+1) 2^-24: exact in binary32


def agent_reset(seed, generation, world, pop):
    """Start positions [pop,2] (binary32) of world `world`."""
    x = philox.philox_block(seed, np.arange(pop), world, generation, TAG_WORLD_AGENT)
    return np.stack([_unit(x[0]), _unit(x[1])], axis=-1)


def item_positions(seed, generation, world, counts):
    """Positions [n_items,2] (binary32) of the items of one world, given how often each was eaten."""
    counts = np.asarray(counts, dtype=np.int64)
    j = 256 * counts + np.arange(counts.shape[0])
    x = philox.philox_block(seed, j, world, generation, TAG_WORLD_ITEM)
    return np.stack([_unit(x[0]), _unit(x[1])], axis=-1)


def dist2(p, q):
    """d2[n,m] between p[n,2] and q[m,2] in binary32, products and the sum rounded one by one."""
    p, q = np.asarray(p, dtype=F32), np.asarray(q, dtype=F32)
    dx = q[None, :, 0] - p[:, None, 0]
    dy = q[None, :, 1] - p[:, None, 1]
    return (dx * dx).astype(F32) + (dy * dy).astype(F32), dx, dy


def nearest_offsets(p, q, exclude_self=False):
    """For every p[n]: (index of the nearest q, offset q - p), lowest index among equal distances."""
    d2, dx, dy = dist2(p, q)
    if exclude_self:
        d2 = d2.copy()
        np.fill_diagonal(d2, np.inf)
    idx = np.argmin(d2, axis=1)                   # first minimum = lowest index
    rows = np.arange(d2.shape[0])
    return idx, np.stack([dx[rows, idx], dy[rows, idx]], axis=-1)


def observe(pos, vel, items, n_food):
    """obs[pop,8] (binary32): velocity, nearest food, nearest poison, nearest other agent."""
    _, food = nearest_offsets(pos, items[:n_food])
    _, poison = nearest_offsets(pos, items[n_food:])
    _, other = nearest_offsets(pos, pos, exclude_self=True)
    return np.concatenate([np.asarray(vel, dtype=F32), food, poison, other], axis=1).astype(F32)


def step(pos, vel, action, items, n_food, w=WORLD_DEFAULT):
    """One step of one world: (pos', vel', reward[pop] int, hit[n_items] bool)."""
    pos, vel = np.asarray(pos, dtype=F32), np.asarray(vel, dtype=F32)
    a = np.clip(np.asarray(action, dtype=F32), F32(-1), F32(1))
    dt, thrust, drag, vmax = F32(w["dt"]), F32(w["thrust"]), F32(w["drag"]), F32(w["vmax"])
    v = (drag * vel).astype(F32) + (thrust * a).astype(F32)
    v = np.clip(v, -vmax, vmax).astype(F32)
    p = pos + (dt * v).astype(F32)
    low, high = p < 0, p > 1
    p = np.where(low, F32(0), np.where(high, F32(1), p)).astype(F32)
    v = np.where(low | high, F32(0), v).astype(F32)
    r2 = F32(w["radius"]) * F32(w["radius"])
    d2, _, _ = dist2(p, items)
    touch = d2 <= r2                                      # [pop, n_items]
    sign = np.where(np.arange(items.shape[0]) < n_food, 1, -1)
    reward = (touch * sign[None, :]).sum(axis=1)
    return p, v, reward.astype(np.int64), touch.any(axis=0)


def rollout(params, dims, acts, seed, generation, n_worlds, steps, w=WORLD_DEFAULT, return_details=False):
    """fitness[pop] (fp64) of a population of MLP policies living together in each of n_worlds worlds."""
    params = np.asarray(params, dtype=np.float64)
    pop = params.shape[0]
    n_food, n_items = int(w["n_food"]), int(w["n_food"]) + int(w["n_poison"])
    total = np.zeros((n_worlds, pop), dtype=np.int64)
    details = []
    for r in range(n_worlds):
        pos = agent_reset(seed, generation, r, pop)
        vel = np.zeros((pop, 2), dtype=F32)
        counts = np.zeros(n_items, dtype=np.int64)
        for _ in range(steps):
            items = item_positions(seed, generation, r, counts)
            obs = observe(pos, vel, items, n_food)
            act = mlp_forward(params, obs[:, None, :].astype(np.float64), dims, acts)[:, 0, :].astype(F32)
            pos, vel, reward, hit = step(pos, vel, act, items, n_food, w)
            total[r] += reward
            counts += hit
        details.append((pos, vel, counts))
    fit = total.mean(axis=0)
    if return_details:
        return fit, total, details
    return fit


def rollout_solitary(params, dims, acts, seed, generation, n_worlds, steps, w=WORLD_DEFAULT, return_details=False):
    """fitness[pop] (fp64) when every member lives alone in its own copy of each world."""
    params = np.asarray(params, dtype=np.float64)
    fit = np.empty(params.shape[0])
    totals, details = [], []
    for m in range(params.shape[0]):
        f, total, det = rollout(params[m:m + 1], dims, acts, seed, generation, n_worlds, steps, w, return_details=True)
        fit[m] = f[0]
        totals.append(total[:, 0])
        details.append(det)
    if return_details:
        return fit, np.stack(totals, axis=1), details      # total[world, member]; details[member][world]
    return fit
