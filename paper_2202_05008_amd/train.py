"""Command line of the training shell: PGPE on one of the named synthetic workloads.

    python -m paper_2202_05008_amd.train --workload cfg1 --generations 200 --test-every 20 \\
        --log run.jsonl --ckpt run.ckpt --save-every 50
    python -m paper_2202_05008_amd.train --workload cfg1 --generations 100 --ckpt run.ckpt --resume

One JSON line per generation goes to stdout (and to --log): generation, max / mean fitness of the
population, milliseconds (with --profile also the device time of each stage), and every
--test-every generations the fitness of the unperturbed centre on held-out inputs.  A run resumed from a checkpoint continues bit-for-bit (the noise of generation t
is a function of (seed, t) alone).
"""
import argparse
import json
import sys

import torch

from . import api as evo
from .trainer import Trainer


FORAGE_TEST_POP = 64      # copies of the centre that share the held-out worlds when it is tested


def _tasks(name, c, seed, dev):
    """(policy_desc, train_task(t), test_task(t)) of a named workload; inputs from workloads.generators."""
    from workloads import generators as gen
    from workloads import configs as wc

    def with_work(make, pd, pop):
        td = make(None)
        n = evo.rollout_workspace_bytes(td, pd, pop)
        return make(torch.empty(max(n, 16), dtype=torch.uint8, device=dev))

    up = lambda a: torch.from_numpy(a).to(dev)
    if name in ("cfg1", "cfg2"):
        if name == "cfg1":
            pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
            batches = [gen.class_blobs(c.data_seed, c.B, c.dims[0], c.dims[-1])]
            held_out = gen.class_blobs(c.data_seed + 1, c.B, c.dims[0], c.dims[-1])
        else:
            pd = evo.make_policy_desc(evo.EVO_POLICY_CONVNET, (28,) + tuple(c.dims))
            batches = [gen.mnist_shaped_batch(c.data_seed, g + 1, c.B) for g in range(8)]
            held_out = gen.mnist_shaped_batch(c.data_seed, 1000, c.B)

        def classify(batch, pop):
            x, y = up(batch[0]), up(batch[1])
            return with_work(lambda w: evo.make_task_desc(evo.EVO_TASK_CLASSIFY, B=c.B, obs=x, target=y, work=w), pd, pop)

        tds = [classify(b, c.pop) for b in batches]
        test_td = classify(held_out, 1)
        return pd, (lambda t: tds[t % len(tds)]), (lambda t: test_td)
    if name == "cfg3":
        pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
        make = lambda s, t: evo.make_task_desc(evo.EVO_TASK_CARTPOLE, n_rollouts=c.n_rollouts, reset_seed=s,
                                               generation=t, cp=c.cartpole, init_scale=c.init_scale)
        return pd, (lambda t: make(seed, t)), (lambda t: make(seed + 1, 1))
    if name == "cfg4":
        pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts, evo.EVO_BF16)
        obs, tgt = gen.teacher_regression(c.data_seed, c.pop, c.B, c.dims)
        od, tg = up(obs), up(tgt)
        td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=c.B, obs=od, obs_member_stride=c.B * c.dims[0], target=tg)
        test_td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=c.B, obs=od, obs_member_stride=c.B * c.dims[0], target=tg)
        return pd, (lambda t: td), (lambda t: test_td)      # the centre is tested on the first member's observations
    if name == "cfg5":
        xs = up(gen.sphere_target(c.data_seed, c.P))
        td = with_work(lambda w: evo.make_task_desc(evo.EVO_TASK_SPHERE, P=c.P, target=xs, work=w), None, c.pop)
        test_td = with_work(lambda w: evo.make_task_desc(evo.EVO_TASK_SPHERE, P=c.P, target=xs, work=w), None, 1)
        return None, (lambda t: td), (lambda t: test_td)
    if name == "seq2seq":
        pd = evo.make_policy_desc(evo.EVO_POLICY_LSTM_SEQ2SEQ, c.dims)

        def strings(g):
            q, a = gen.addition_batch(c.data_seed, g, c.B, c.digits)
            return evo.make_task_desc(evo.EVO_TASK_SEQ2SEQ, B=c.B, obs=up(q), target=up(a), seq_in=q.shape[1],
                                      seq_out=a.shape[1])

        tds = [strings(g + 1) for g in range(16)]
        test_td = strings(1000)
        return pd, (lambda t: tds[t % len(tds)]), (lambda t: test_td)
    if name in ("forage", "forage_solo"):
        kind = evo.EVO_TASK_FORAGE if name == "forage" else evo.EVO_TASK_FORAGE_SOLO
        pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
        work = {}

        def world(s, t, pop):      # one workspace per population size, a fresh descriptor per generation
            make = lambda w: evo.make_task_desc(kind, n_rollouts=c.n_rollouts, reset_seed=s, generation=t,
                                                cp=tuple(c.world), work=w)
            if pop not in work:
                work[pop] = torch.empty(evo.rollout_workspace_bytes(make(None), pd, pop), dtype=torch.uint8, device=dev)
            return make(work[pop])

        test_pop = FORAGE_TEST_POP if name == "forage" else 1
        return pd, (lambda t: world(seed, t, c.pop)), (lambda t: world(seed + 1, 1, test_pop))
    raise SystemExit("unknown workload %r" % name)


def main(argv=None):
    from workloads import CONFIGS, generators as gen
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", default="cfg1", choices=sorted(CONFIGS))
    ap.add_argument("--generations", type=int, default=100)
    ap.add_argument("--seed", type=int, default=20220509)
    ap.add_argument("--lr-mu", type=float, default=None, help="step size of the centre (default: the workload's)")
    ap.add_argument("--optimizer", default="adam", choices=["adam", "clipup", "momentum"])
    ap.add_argument("--test-every", type=int, default=0)
    ap.add_argument("--log", default=None, help="JSON-lines file to append to")
    ap.add_argument("--ckpt", default=None, help="checkpoint file")
    ap.add_argument("--save-every", type=int, default=0)
    ap.add_argument("--resume", action="store_true", help="continue from --ckpt")
    ap.add_argument("--profile", action="store_true", help="log the device time of ask, rollout and tell per generation")
    ap.add_argument("--one-launch", action="store_true",
                    help="small supervised problems (cfg1): ask, evaluation and tell of a generation as one launch, same results")
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        raise SystemExit("paper_2202_05008_amd.train needs a GPU (there is no CPU fallback)")
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    c = CONFIGS[args.workload]
    opt = {"adam": evo.EVO_OPT_ADAM, "clipup": evo.EVO_OPT_CLIPUP, "momentum": evo.EVO_OPT_MOMENTUM}[args.optimizer]
    cfg = evo.make_pgpe_config(P=c.P, pop_max=c.pop, sigma_init=c.sigma_init,
                               lr_mu=c.lr_mu if args.lr_mu is None else args.lr_mu, lr_sigma=c.lr_sigma,
                               sigma_max_change=c.sigma_max_change, optimizer=opt)
    mu0 = None if args.workload == "cfg5" else gen.initial_mu(c.data_seed, c.P)
    pg = evo.PGPE(cfg, mu0)
    pd, train_task, test_task = _tasks(args.workload, c, args.seed, dev)
    tr = Trainer(pg, pd, train_task, c.pop, steps=c.steps, seed=args.seed, test_task=test_task,
                 test_every=args.test_every, log_path=args.log, ckpt_path=args.ckpt, save_every=args.save_every,
                 test_pop=FORAGE_TEST_POP if args.workload == "forage" else 1, profile=args.profile, one_launch=args.one_launch)
    if args.resume:
        if not args.ckpt:
            raise SystemExit("--resume needs --ckpt")
        print(json.dumps({"resumed_at_generation": tr.load(args.ckpt)}), flush=True)
    for _ in range(args.generations):
        print(json.dumps(tr.step()), flush=True)
    if args.ckpt:
        tr.save(args.ckpt)
    print(json.dumps({"final_test_fitness": tr.test(), "generation": pg.generation}), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
