"""CPU ORACLE (test infrastructure, not part of the product path) -- one whole generation.

Strings the pieces together in the order the paper's training loop has them (Section 2,
Figure 2 and the trainer / simulation-manager paragraph; Section 4's ask / tell):
ask -> evaluate every member with the global policy on the vectorised task -> tell.
`task` is a plain dict: kind in {"classify","regress","cartpole","sphere","seq2seq","forage","forage_solo"}, the policy
description and the task's input arrays.  parity unpinned as a whole: the paper prints no
value of any generation; every stage it calls is pinned on its own, and the routing done here is
pinned in tests/test_oracle_generation.py (torch's functional network and losses, closed forms, the
free cart-pole stepped by hand, ask -> evaluate -> tell spelled out).
"""
import numpy as np

from . import forage, pgpe, policy, seq2seq, tasks


def evaluate(task, params, seed, generation):
    """fitness[pop] (fp64) of a population on a task."""
    kind = task["kind"]
    if kind == "sphere":
        return tasks.sphere_fitness(params, task["x_star"])
    if kind == "cartpole":
        return tasks.cartpole_rollout(params, task["dims"], task["acts"], seed, generation,
                                      task["n_rollouts"], task["steps"], task.get("cp", tasks.CP_DEFAULT),
                                      task.get("init_scale", 0.2))
    if kind == "forage_solo":
        return forage.rollout_solitary(params, task["dims"], task["acts"], seed, generation, task["n_worlds"],
                                       task["steps"], task.get("world", forage.WORLD_DEFAULT))
    if kind == "forage":
        return forage.rollout(params, task["dims"], task["acts"], seed, generation, task["n_worlds"], task["steps"],
                              task.get("world", forage.WORLD_DEFAULT))
    if kind == "seq2seq":
        return seq2seq.fitness(seq2seq.forward(params, task["query"], task["answer"], task["H"]), task["answer"])
    if task.get("convnet"):
        c1, c2, n_cls = task["dims"]
        out = policy.convnet_forward(params, task["obs"], c1, c2, n_cls)
    else:
        out = policy.mlp_forward(params, task["obs"], task["dims"], task["acts"])
    if kind == "classify":
        return tasks.classify_fitness(out, task["labels"])
    if kind == "regress":
        return tasks.regress_fitness(out, task["targets"])
    raise ValueError("unknown task kind %r" % (kind,))


def run_generation(state, task, seed, pop, dtype=pgpe.DT_F32):
    """ask -> evaluate -> tell; returns (params fp32, fitness fp32)."""
    t = state.t
    params = pgpe.ask(state, seed, pop, dtype)
    fit = evaluate(task, params, seed, t).astype(np.float32)
    pgpe.tell(state, fit)
    return params, fit
