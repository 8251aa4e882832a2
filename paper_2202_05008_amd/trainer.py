"""Minimal training shell around the C ABI: the loop, testing of the centre, JSON-lines logging
and checkpoints with exact resume (the trainer of Section 2: loop, log, test of the centre,
periodic saving).

Host-side orchestration only: every number it logs is produced by the library's kernels
(ask, rollout, tell, pgpe_center); torch supplies device memory, the stream and the
max / mean of the fitness vector that goes into the log.
"""
import json
import os
import struct
import time

import torch

from . import api

_CKPT_MAGIC = b"EVOTRAIN1"


class Trainer:
    """One PGPE run on one GPU.

    pgpe        api.PGPE (owns mu, sigma and the moments on the device)
    policy      policy_desc, or None for the sphere task
    train_task  callable t -> task_desc of generation t (t = 1, 2, ...): the training data / reset
                seeds of that generation
    test_task   optional callable t -> task_desc used to evaluate the centre mu without perturbation
    pop, steps  population size and roll-out steps per evaluation
    seed        seed of the noise stream; generation t of a run is a function of (seed, t) alone
    log_path    JSON-lines log (appended), or None
    ckpt_path   checkpoint file written every `save_every` generations (0 = never), atomically
    profile     also log the device time of each stage (ask, rollout, tell) from events on the stream
    test_pop    copies of the centre that are evaluated together (a shared world needs company: the
                test fitness is then the mean over the copies); 1 for every other task
    """

    def __init__(self, pgpe, policy, train_task, pop, steps=1, seed=0, test_task=None, test_every=0, log_path=None,
                 ckpt_path=None, save_every=0, test_pop=1, profile=False, one_launch=False):
        self.pgpe, self.policy, self.train_task, self.test_task = pgpe, policy, train_task, test_task
        self.pop, self.steps, self.seed = int(pop), int(steps), int(seed)
        self.test_every, self.save_every = int(test_every), int(save_every)
        self.log_path, self.ckpt_path = log_path, ckpt_path
        self.dtype = policy.dtype if policy is not None else api.EVO_F32
        tdtype = torch.bfloat16 if self.dtype == api.EVO_BF16 else torch.float32
        dev = pgpe.mu.device
        self.params = torch.empty(self.pop, pgpe.cfg.P, dtype=tdtype, device=dev)
        self.fitness = torch.empty(self.pop, dtype=torch.float32, device=dev)
        self.profile = bool(profile)
        self.one_launch = bool(one_launch)      # small supervised problems: the whole generation as one launch (same bits)
        self.test_pop = int(test_pop)
        self._center = torch.empty(self.test_pop, pgpe.cfg.P, dtype=tdtype, device=dev)
        self._center_fit = torch.empty(self.test_pop, dtype=torch.float32, device=dev)
        self.history = []

    # ---- one generation ---------------------------------------------------------------------
    def step(self):
        """ask -> rollout -> tell for the next generation; returns its log record."""
        t = self.pgpe.generation
        t0 = time.perf_counter()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if self.profile else None
        mark = (lambda i: ev[i].record()) if self.profile else (lambda i: None)
        mark(0)
        if self.one_launch:
            self.pgpe.generation_step(self.seed, self.pop, self.train_task(t), self.policy, self.fitness)
            mark(1), mark(2)
        else:
            self.pgpe.ask(self.seed, self.pop, self.params, self.dtype)
            mark(1)
            api.rollout(self.train_task(t), self.policy, self.params, self.pop, self.steps, self.fitness)
            mark(2)
            self.pgpe.tell(self.fitness)
        mark(3)
        fmax, fmean = float(self.fitness.max()), float(self.fitness.mean())   # waits for the generation
        rec = {"generation": t, "fitness_max": fmax, "fitness_mean": fmean,
               "ms": (time.perf_counter() - t0) * 1e3}
        if self.profile:
            ev[3].synchronize()
            rec["stage_ms"] = {n: ev[i].elapsed_time(ev[i + 1]) for i, n in enumerate(("ask", "rollout", "tell"))}
        if self.test_task is not None and self.test_every and t % self.test_every == 0:
            rec["test_fitness"] = self.test()
        self.history.append(rec)
        if self.log_path:
            with open(self.log_path, "a") as f:
                f.write(json.dumps(rec) + "\n")
        if self.ckpt_path and self.save_every and t % self.save_every == 0:
            self.save(self.ckpt_path)
        return rec

    def run(self, generations):
        for _ in range(generations):
            self.step()
        return self.history

    # ---- testing: the centre, unperturbed -----------------------------------------------------
    def test(self, task=None):
        """Fitness of the centre mu (no perturbation) on the test task of the current generation."""
        t = self.pgpe.generation
        td = task if task is not None else self.test_task(t)
        self.pgpe.center(self.test_pop, self._center, self.dtype)
        api.rollout(td, self.policy, self._center, self.test_pop, self.steps, self._center_fit)
        return float(self._center_fit.mean())

    # ---- checkpoints ----------------------------------------------------------------------------
    def save(self, path):
        """Algorithm state (pgpe_state_export) plus the run's seed and population size."""
        blob = self.pgpe.export_state()
        tmp = path + ".tmp"
        with open(tmp, "wb") as f:
            f.write(_CKPT_MAGIC)
            f.write(struct.pack("<QII", self.seed, self.pop, self.steps))
            f.write(blob)
        os.replace(tmp, path)

    def load(self, path):
        """Restore a checkpoint written by save(); the run then continues exactly where it stopped."""
        with open(path, "rb") as f:
            raw = f.read()
        n = len(_CKPT_MAGIC)
        if raw[:n] != _CKPT_MAGIC:
            raise ValueError("%s is not a trainer checkpoint" % path)
        seed, pop, steps = struct.unpack("<QII", raw[n:n + 16])
        if pop != self.pop or steps != self.steps:
            raise ValueError("checkpoint was written with pop=%d, steps=%d; this trainer has pop=%d, steps=%d"
                             % (pop, steps, self.pop, self.steps))
        self.seed = seed
        self.pgpe.import_state(raw[n + 16:])
        return self.pgpe.generation
