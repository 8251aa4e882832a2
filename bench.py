#!/usr/bin/env python3
"""Benchmark of one whole PGPE generation (ask -> evaluate -> tell) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2]

A step is one generation of the named synthetic workload with every input already resident
in device memory.  Prints ONE JSON line: whole-job throughput in member-evals/s, ms per
generation, the roofline of the dominant kernel (timed with events on the launch stream), the
CPU oracle timed on a bounded sample of the same workload (one thread, and all cores), and what
this GPU measures for the quantities the roofline peaks are quoted for.  Without --workload the
headline is cfg2 and the line also carries `per_config`: the same measurement for each of the five
configurations.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
# The ConvNet, cart-pole and LSTM kernels deliver fp32-accurate results, but their contractions are issued as
# fp16 matrix instructions on two-term scaled operand splits (three instructions per product): `frac` prices
# the launch as issued, against the fp16 matrix peak; `fp32_equivalent` prices the algorithmic fp32 flops
# against the fp32 matrix peak (it can exceed 1, which says that peak is no bound for these kernels).  By the
# counters in profiles/ all three are bound by vector-instruction issue, not by the matrix pipe.
PEAK_MFMA_F32_TF = 157.3       # dense fp32 matrix
PEAK_MFMA_BF16_TF = 2500.0     # dense bf16 / fp16 matrix
PEAK_ALU_F32_TF = 157.3        # fp32 vector (256 CU x 4 SIMD x 32 lanes x 2.4 GHz x 2 flop)

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this file, scaled by what the same counters read for a 1 GiB copy in the same process (on this
# box FETCH_SIZE x 2.0, WRITE_SIZE x 1.0).  Sources: the summaries under profiles/.  Counters cannot be
# read from inside the run, so `traffic` is what the profile of this same command measured, not this run.
MEASURED_TRAFFIC_BYTES = {
    "cfg1": 2924945,       # profiles/mlp_f32_kernel_cfg1.md
    "cfg2": 37831063,      # profiles/convnet_kernel_cfg2.md (algorithmic 12.5 MB: the batch, as 4 KB of fp16 planes per
                           # image, is re-fetched per L2)
    "cfg3": 19116032,      # profiles/cartpole_kernel_cfg3.md
    "cfg4": 807197617,     # profiles/mlp_bf16_stream_kernel_cfg4.md
    "cfg5": 4305387571,    # profiles/ask_sphere_tell_kernels_cfg5.md (ask)
    "seq2seq": 890661888,  # profiles/lstm_seq2seq_kernel_seq2seq.md (algorithmic 598 MB: the rest is register spill traffic)
    "forage": 6920192,     # profiles/world_step_kernel_forage.md (per step launch: weights 5.8 MB + positions)
    "forage_solo": 5979136,  # profiles/world_solo_kernel_forage_solo.md (the weights, read once; the rest stays on chip)
}


# Timed generations per workload when --steps is not given (about a second of GPU time or less) and
# the population of the oracle's bounded sample (about 10-30 s of CPU time on one core).
# What the rocprofv3 counters in profiles/ say bounds the dominant kernel.
BOUND_DETAIL = {
    "cfg1": "launch latency: five launches of a few microseconds each (profiles/mlp_f32_kernel_cfg1.md)",
    "cfg2": "both convolutions on the matrix cores: MFMA busy 47 %, VALU issue 63 % on the same SIMDs (16 % of the cycles overlap), LDS busy 64 %, "
            "31 % of wave time waiting at three waves per SIMD (profiles/convnet_kernel_cfg2.md)",
    "cfg3": "vector-instruction issue along a 1000-step dependency chain: VALU busy 66 %, MFMA busy 21 %, 36 % of wave "
            "time waiting (profiles/cartpole_kernel_cfg3.md)",
    "cfg4": "HBM weight stream: 64 flop per weight byte (profiles/mlp_bf16_stream_kernel_cfg4.md)",
    "cfg5": "HBM write of the population in ask (profiles/ask_sphere_tell_kernels_cfg5.md)",
    "seq2seq": "instruction issue: VALU busy 44 % + MFMA busy 37 %, 29 % of wave time waiting (profiles/lstm_seq2seq_kernel_seq2seq.md)",
    "forage": "latency of one step launch: vector ALU 20 % busy (profiles/world_step_kernel_forage.md)",
    "forage_solo": "vector-instruction issue along the step chain: vector ALU 82 % busy (profiles/world_solo_kernel_forage_solo.md)",
}

DEFAULT_STEPS = {"cfg1": 200, "cfg2": 50, "cfg3": 20, "cfg4": 50, "cfg5": 20, "seq2seq": 20, "forage": 20, "forage_solo": 50}
ORACLE_SAMPLE_POP = {"cfg1": 64, "cfg2": 96, "cfg3": 512, "cfg4": 1024, "cfg5": 96, "seq2seq": 32, "forage": 128, "forage_solo": 24}
ORACLE_SAMPLE_GENERATIONS = {"cfg1": 600}


def _build_workload(name, seed, batch=None, f32=False):
    import dataclasses
    import numpy as np
    import torch
    import paper_2202_05008_amd as evo
    from workloads import CONFIGS, generators as gen
    from workloads import configs as wc

    c = CONFIGS[name]
    if batch is not None:      # cfg4 only: observations per member, for the sweep of arithmetic intensity
        c = dataclasses.replace(c, B=batch)
    if f32:                    # cfg4 only: the same shape with fp32 parameters (the fp32 matrix-core MLP kernel)
        c = dataclasses.replace(c, dtype=wc.DT_F32)
    dev = torch.device("cuda:0")
    mu0 = None if name == "cfg5" else gen.initial_mu(c.data_seed, c.P)
    pg = evo.PGPE(evo.make_pgpe_config(P=c.P, pop_max=c.pop, sigma_init=c.sigma_init, lr_mu=c.lr_mu,
                                       lr_sigma=c.lr_sigma, sigma_max_change=c.sigma_max_change), mu0)
    tdtype = torch.bfloat16 if c.dtype == wc.DT_BF16 else torch.float32
    params = torch.empty(c.pop, c.P, dtype=tdtype, device=dev)
    fitness = torch.empty(c.pop, dtype=torch.float32, device=dev)
    wl = {"cfg": c, "pgpe": pg, "params": params, "fitness": fitness, "evo": evo}

    def with_work_cached(make):      # one workspace, a fresh descriptor per generation
        if "work" not in wl:
            n = evo.rollout_workspace_bytes(make(None), wl.get("pd"), c.pop)
            wl["work"] = torch.empty(max(n, 16), dtype=torch.uint8, device=dev)
        return make(wl["work"])

    def with_work(make):
        td = make(None)
        n = evo.rollout_workspace_bytes(td, wl.get("pd"), c.pop)
        work = torch.empty(max(n, 16), dtype=torch.uint8, device=dev)
        wl.setdefault("keep", []).append(work)
        return make(work)

    if name in ("cfg1", "cfg2"):
        if name == "cfg1":
            wl["pd"] = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
            x, y = gen.class_blobs(c.data_seed, c.B, c.dims[0], c.dims[-1])
            batches = [(torch.from_numpy(x).to(dev), torch.from_numpy(y).to(dev))]
            flops = 2.0 * sum(c.dims[i] * c.dims[i + 1] for i in range(len(c.dims) - 1)) * c.pop * c.B
            wl["roofline"] = ("alu", flops, PEAK_ALU_F32_TF, "TFLOP/s")
            wl["desc"] = "cfg1: plumbing classifier, fp32 MLP 16-32-4, pop 64, 512 samples"
        else:
            wl["pd"] = evo.make_policy_desc(evo.EVO_POLICY_CONVNET, (28,) + tuple(c.dims))
            batches = []
            for g in range(4):      # four distinct batches, cycled: a new batch every generation
                x, y = gen.mnist_shaped_batch(c.data_seed, g + 1, c.B)
                batches.append((torch.from_numpy(x).to(dev), torch.from_numpy(y).to(dev)))
            c1, c2, ncls = c.dims
            per_img = 2.0 * (9 * c1 * 28 * 28 + 9 * c1 * c2 * 14 * 14 + 7 * 7 * c2 * ncls)
            # as issued: v_mfma_f32_16x16x32_f16 (16,384 flop each) per image: conv1 7 passes x 2 tiles x 4, conv2 7 bands x
            # 3 tap columns x 2 output rows x 3 products of split terms
            wl["roofline"] = ("mfma", 16384.0 * (7 * 2 * 4 + 7 * 3 * 2 * 3) * c.pop * c.B, PEAK_MFMA_BF16_TF, "TFLOP/s")
            wl["fp32_flops"] = per_img * c.pop * c.B
            wl["desc"] = "cfg2: MNIST-shaped synthetic images, per-member fp32 ConvNet P=9098, pop 256, batch 1024"
        tds = [with_work(lambda w, b=b: evo.make_task_desc(evo.EVO_TASK_CLASSIFY, B=c.B, obs=b[0], target=b[1], work=w))
               for b in batches]
        wl["keep"].append(batches)
        wl["task"] = lambda t: tds[t % len(tds)]
        wl["n_tasks"] = len(tds)
        wl["dtype"] = "f32"
    elif name == "cfg3":
        wl["pd"] = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
        wl["task"] = lambda t: evo.make_task_desc(evo.EVO_TASK_CARTPOLE, n_rollouts=c.n_rollouts, reset_seed=seed,
                                                  generation=t + 1, cp=c.cartpole, init_scale=c.init_scale,
                                                  generation_dev=wl.get("gen_dev"))
        flops = 2.0 * sum(c.dims[i] * c.dims[i + 1] for i in range(len(c.dims) - 1)) * c.evals_per_generation
        # layer 2 as issued: three fp16 matrix instructions per product (layer 1 runs on the fp32 instruction)
        wl["roofline"] = ("valu-issue", 3.0 * 2.0 * c.dims[1] * c.dims[2] * c.evals_per_generation, PEAK_MFMA_BF16_TF,
                          "TFLOP/s")
        wl["fp32_flops"] = flops
        wl["desc"] = "cfg3: cart-pole swing-up, fp32 MLP 5-64-64-1, pop 1024 x 16 roll-outs x 1000 steps"
        wl["dtype"] = "f32"
    elif name == "cfg4":
        wl["pd"] = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts, evo.EVO_F32 if f32 else evo.EVO_BF16)
        obs, tgt = gen.teacher_regression(c.data_seed, c.pop, c.B, c.dims)
        od, tg = torch.from_numpy(obs).to(dev), torch.from_numpy(tgt).to(dev)
        wl["keep"] = [od, tg]
        td = with_work(lambda w: evo.make_task_desc(evo.EVO_TASK_REGRESS, B=c.B, obs=od, obs_member_stride=c.B * c.dims[0],
                                                    target=tg, work=w))
        wl["task"] = lambda t: td
        nbytes = c.pop * (c.P * (4.0 if f32 else 2.0) + c.B * c.dims[0] * 4.0 + c.B * c.dims[-1] * 4.0 + 4.0)
        flops = 2.0 * sum(c.dims[i] * c.dims[i + 1] for i in range(len(c.dims) - 1)) * c.pop * c.B
        # past the ridge (peak flop rate / peak byte rate = 312 flop per byte) the forward is priced as a contraction
        if flops / nbytes > PEAK_MFMA_BF16_TF * 1e12 / (PEAK_HBM_GBS * 1e9):
            wl["roofline"] = ("mfma", flops, PEAK_MFMA_BF16_TF, "TFLOP/s")
            wl["hbm_bytes_work"] = nbytes
        else:
            wl["roofline"] = ("hbm", nbytes, PEAK_HBM_GBS, "GB/s")
            wl["mfma_tflops_work"] = flops
        wl["desc"] = "cfg4: wide %s MLP 64-256-256-16, pop 4096, %d observations per member" % ("fp32" if f32 else "bf16", c.B)
        wl["dtype"] = "f32" if f32 else "bf16"
        if f32:      # two-term fp16 splits: three matrix instructions per product
            wl["mfma_f16_issued_work"] = 3.0 * flops
    elif name == "cfg5":
        wl["pd"] = None
        xs = torch.from_numpy(gen.sphere_target(c.data_seed, c.P)).to(dev)
        wl["keep"] = [xs]
        wl["x_star"] = xs
        td = with_work(lambda w: evo.make_task_desc(evo.EVO_TASK_SPHERE, P=c.P, target=xs, work=w))
        wl["task"] = lambda t: td
        wl["roofline"] = ("hbm", c.pop * c.P * 4.0 + 2 * c.P * 4.0, PEAK_HBM_GBS, "GB/s")
        wl["roofline_stage"] = "ask"
        wl["desc"] = "cfg5: ask/tell stress on a sphere, P=2^20, pop 1024"
        wl["dtype"] = "f32"
    elif name == "seq2seq":
        V, H, n_out = c.dims
        wl["pd"] = evo.make_policy_desc(evo.EVO_POLICY_LSTM_SEQ2SEQ, c.dims)
        tds = []
        for g in range(4):      # four distinct batches, cycled: a new batch every generation
            q, a = gen.addition_batch(c.data_seed, g + 1, c.B, c.digits)
            qd, ad = torch.from_numpy(q).to(dev), torch.from_numpy(a).to(dev)
            wl.setdefault("keep", []).append((qd, ad))
            tds.append(evo.make_task_desc(evo.EVO_TASK_SEQ2SEQ, B=c.B, obs=qd, target=ad, seq_in=q.shape[1],
                                          seq_out=a.shape[1]))
        wl["task"] = lambda t: tds[t % len(tds)]
        wl["n_tasks"] = len(tds)
        Lq, La = 2 * c.digits + 2, c.digits + 1
        flops = 2.0 * ((Lq + La) * H * 4 * H + La * H * n_out) * c.pop * c.B
        wl["roofline"] = ("valu-issue", 3.0 * flops, PEAK_MFMA_BF16_TF, "TFLOP/s")   # three fp16 instructions per product
        wl["fp32_flops"] = flops
        wl["desc"] = ("seq2seq: LSTM encoder-decoder H=128 (P=145674) on three-digit addition strings, pop 1024, "
                      "128 strings per member")
        wl["dtype"] = "f32"
    elif name in ("forage", "forage_solo"):
        solo = name == "forage_solo"
        wl["pd"] = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
        w = wc.world_dict(c.world)
        cp = tuple(c.world)
        wl["task"] = lambda t: with_work_cached(lambda work: evo.make_task_desc(
            evo.EVO_TASK_FORAGE_SOLO if solo else evo.EVO_TASK_FORAGE, n_rollouts=c.n_rollouts, reset_seed=seed, generation=t + 1, cp=cp, work=work,
            generation_dev=wl.get("gen_dev")))
        # one launch = one step of every world: per agent the scan over the others (2 sub, 2 mul, add, compare per
        # candidate) and over the items (twice: sensing and touching), and the policy's multiply-adds
        n_items = w["n_food"] + w["n_poison"]
        per_agent = (0.0 if solo else 6.0 * c.pop) + 2 * 6.0 * n_items + 2.0 * sum(c.dims[i] * c.dims[i + 1] for i in range(3))
        if solo:      # the whole episode is one launch
            wl["roofline"] = ("alu", per_agent * c.pop * c.n_rollouts * c.steps, PEAK_ALU_F32_TF, "TFLOP/s")
            wl["desc"] = ("forage_solo: every member alone in its own copy of each of %d worlds, %d members, fp32 MLP "
                          "8-32-32-2, %d steps (one launch per episode)" % (c.n_rollouts, c.pop, c.steps))
        else:
            wl["roofline"] = ("alu", per_agent * c.pop * c.n_rollouts, PEAK_ALU_F32_TF, "TFLOP/s")
            wl["launches"] = c.steps      # the stage is `steps` launches of the step kernel (+ reset and finish)
            wl["desc"] = ("forage: the population as %d agents of each of %d shared worlds, fp32 MLP 8-32-32-2, %d "
                          "steps (one launch per step)" % (c.pop, c.n_rollouts, c.steps))
        wl["dtype"] = "f32"
    else:
        raise SystemExit("unknown workload %r" % name)
    wl.setdefault("roofline_stage", "rollout")
    return wl


_POOL_TASK = None      # the task dict of the oracle's all-cores leg; worker processes inherit it through fork


def _oracle_slice(job):
    """Worker of the all-cores leg: the oracle's fitness of a slice of the population."""
    from oracle import generation as ogen
    params, seed, t = job
    return ogen.evaluate(_POOL_TASK, params, seed, t)


def _cpu_baseline(name, seed):
    """The oracle, as it stands, on a bounded sample of the workload: on one thread, and with the sample's
    population split over all cores of this machine's share (worker processes, each on one BLAS thread; ask and
    tell stay on the parent).  Runs before anything touches the GPU, so that the workers can be forked."""
    global _POOL_TASK
    import multiprocessing
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import pgpe as opgpe, generation as ogen
    from workloads import CONFIGS, generators as gen
    from workloads import configs as wc

    c = CONFIGS[name]
    sample_pop = ORACLE_SAMPLE_POP[name]
    gens = ORACLE_SAMPLE_GENERATIONS.get(name, 1)
    dtype = opgpe.DT_BF16 if c.dtype == wc.DT_BF16 else opgpe.DT_F32
    if name == "cfg1":
        x, y = gen.class_blobs(c.data_seed, c.B, c.dims[0], c.dims[-1])
        task = {"kind": "classify", "dims": c.dims, "acts": c.acts, "obs": x, "labels": y}
        evals = sample_pop * c.B
    elif name == "cfg2":
        x, y = gen.mnist_shaped_batch(c.data_seed, 1, c.B)
        task = {"kind": "classify", "convnet": True, "dims": c.dims, "obs": x, "labels": y}
        evals = sample_pop * c.B
    elif name == "cfg3":
        task = {"kind": "cartpole", "dims": c.dims, "acts": c.acts, "n_rollouts": c.n_rollouts, "steps": c.steps,
                "cp": c.cartpole, "init_scale": c.init_scale}
        evals = sample_pop * c.n_rollouts * c.steps
    elif name == "cfg4":
        obs, tgt = gen.teacher_regression(c.data_seed, sample_pop, c.B, c.dims)
        task = {"kind": "regress", "dims": c.dims, "acts": c.acts, "obs": obs, "targets": tgt}
        evals = sample_pop * c.B
    elif name == "seq2seq":
        q, a = gen.addition_batch(c.data_seed, 1, c.B, c.digits)
        task = {"kind": "seq2seq", "H": c.dims[1], "query": q, "answer": a}
        evals = sample_pop * c.B
    elif name in ("forage", "forage_solo"):      # forage: a smaller population is a smaller crowd in each world
        task = {"kind": name, "dims": c.dims, "acts": c.acts, "n_worlds": c.n_rollouts, "steps": c.steps,
                "world": wc.world_dict(c.world)}
        evals = sample_pop * c.n_rollouts * c.steps
    else:
        task = {"kind": "sphere", "x_star": gen.sphere_target(c.data_seed, c.P)}
        evals = sample_pop
    mu0 = None if name == "cfg5" else gen.initial_mu(c.data_seed, c.P)
    st = opgpe.PGPEState.create(opgpe.PGPEConfig(P=c.P, pop_max=sample_pop), mu0)
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        for _ in range(gens):
            ogen.run_generation(st, task, seed, sample_pop, dtype)
        dt = time.perf_counter() - t0
    out = {"value": evals * gens / dt, "unit": "member-evals/s", "cores": 1, "kind": "oracle",
           "sample": "%d generation(s) of %s with pop=%d (all other sizes as configured), %.1f s"
                     % (gens, name, sample_pop, dt)}
    # ---- all cores: members are independent in every task but the shared worlds; per-member data goes with its slice
    nproc = os.cpu_count() or 1
    cores = max(1, min(nproc, 16, sample_pop))      # a one-GPU machine's share of the host is 16 cores
    if name == "forage" or cores == 1:
        out["all_cores"] = None
        return out
    bounds = np.linspace(0, sample_pop, cores + 1).astype(int)
    st = opgpe.PGPEState.create(opgpe.PGPEConfig(P=c.P, pop_max=sample_pop), mu0)
    per_member = [k for k in ("obs", "targets") if name == "cfg4" and k in task]
    with threadpool_limits(limits=1):
        if per_member:       # cfg4: every member has its own observations and targets; a worker gets its slice only
            full = {k: task[k] for k in per_member}
        _POOL_TASK = task
        ctx = multiprocessing.get_context("fork")
        with ctx.Pool(cores) as pool:
            pool.map(_noop, range(cores))      # workers are up before the clock starts
            t0 = time.perf_counter()
            for _ in range(gens):
                t = st.t
                params = opgpe.ask(st, seed, sample_pop, dtype)
                if per_member:
                    fit = np.concatenate(pool.map(_oracle_slice_own, [(params[lo:hi], seed, t, lo, hi)
                                                                      for lo, hi in zip(bounds[:-1], bounds[1:])]))
                else:
                    fit = np.concatenate(pool.map(_oracle_slice, [(params[lo:hi], seed, t)
                                                                  for lo, hi in zip(bounds[:-1], bounds[1:])]))
                opgpe.tell(st, fit.astype(np.float32))
            dt_all = time.perf_counter() - t0
    out["all_cores"] = {"value": evals * gens / dt_all, "cores": cores, "nproc": nproc,
                        "how": "the sample's population split over %d forked worker processes, one BLAS thread each; "
                               "ask and tell on the parent; %.1f s" % (cores, dt_all)}
    return out


def _noop(_):
    return None


def _oracle_slice_own(job):
    """As _oracle_slice for a task whose members have their own observations and targets."""
    from oracle import generation as ogen
    params, seed, t, lo, hi = job
    task = dict(_POOL_TASK)
    task["obs"], task["targets"] = _POOL_TASK["obs"][lo:hi], _POOL_TASK["targets"][lo:hi]
    return ogen.evaluate(task, params, seed, t)


def _measure_peaks(evo, torch):
    """What this GPU delivers for the quantities the roofline peaks are quoted for: a plain 1 GiB device copy
    and register-only loops of one instruction kind (evo_probe_rate), each timed with events, second run kept."""
    def timed(fn):
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            work = fn()
            e1.record()
            e1.synchronize()
            ms = e0.elapsed_time(e1)
            best = (work, ms) if best is None or ms < best[1] else best
        return best

    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    work, ms = timed(lambda: (dst.copy_(src), 2.0 * src.numel() * 4)[1])
    peaks = {"hbm_copy_1GiB_GBs": work / (ms * 1e-3) / 1e9, "hbm_published_GBs": PEAK_HBM_GBS}
    del src, dst
    out = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    for key, kind, iters, published in (("fma_f32_vector_TFs", 0, 100000, PEAK_ALU_F32_TF),
                                        ("mfma_f16_16x16x32_TFs", 1, 10000, PEAK_MFMA_BF16_TF),
                                        ("mfma_bf16_32x32x16_TFs", 2, 5000, PEAK_MFMA_BF16_TF),
                                        ("mfma_f32_16x16x4_TFs", 3, 5000, PEAK_MFMA_F32_TF)):
        work, ms = timed(lambda: evo.evo_probe_rate(kind, iters, out))
        peaks[key] = work / (ms * 1e-3) / 1e12
        peaks[key.replace("_TFs", "_published_TFs")] = published
    return peaks


def _run_workload(name, args, steps, warmup, torch):
    """Time `steps` whole generations of one workload; returns the fields of its JSON line."""
    wl = _build_workload(name, args.seed, args.batch, args.variant == "f32")
    c, pg, evo = wl["cfg"], wl["pgpe"], wl["evo"]
    stage_names = ("ask", "rollout", "tell")
    events = []

    def generation(t, timed):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if timed else None
        td = wl["task"](t)
        if timed:
            ev[0].record()
        if args.variant == "fused" and name == "cfg1":      # the whole generation in one launch: timed as the ask stage
            pg.generation_step(args.seed, c.pop, td, wl["pd"], wl["fitness"])
            if timed:
                for e in ev[1:]:
                    e.record()
                events.append(ev)
            return
        if args.variant == "fused":      # one call stands for ask + rollout: the rollout stage reads 0
            if name == "cfg4":
                pg.ask_rollout(args.seed, c.pop, td, wl["pd"], wl["fitness"])
            else:
                pg.ask_sphere(args.seed, c.pop, wl["x_star"], wl["fitness"])
        else:
            pg.ask(args.seed, c.pop, wl["params"], c.dtype)
        if timed:
            ev[1].record()
        if args.variant != "fused":
            evo.rollout(td, wl["pd"], wl["params"], c.pop, c.steps, wl["fitness"])
        if timed:
            ev[2].record()
        if args.variant == "stored":
            pg.tell_stored(wl["fitness"], wl["params"])
        else:
            pg.tell(wl["fitness"])
        if timed:
            ev[3].record()
            events.append(ev)

    if args.graph:
        wl["gen_dev"] = pg.device_generation()
    for t in range(warmup):
        generation(t, False)
    torch.cuda.synchronize()
    if args.graph:      # one recorded generation per distinct batch; each replay is the next generation
        for t in range(min(steps, 20)):
            generation(warmup + t, True)
        graphs = []
        for k in range(wl.get("n_tasks", 1)):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                generation(k, False)
            graphs.append(g)
        _ = pg.generation      # recording moved the host copy of the index, not the device's: bring it back
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(steps):
            graphs[t % len(graphs)].replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        t0 = time.perf_counter()
        for t in range(steps):
            generation(warmup + t, True)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0

    stage_ms = {n: sum(e[i].elapsed_time(e[i + 1]) for e in events) / len(events) for i, n in enumerate(stage_names)}
    assert torch.isfinite(wl["fitness"]).all(), "non-finite fitness after the timed region"
    ms_per_step = elapsed * 1e3 / steps
    value = c.evals_per_generation * steps / elapsed
    bound, work, peak, unit = wl["roofline"]
    dom_stage = "ask" if args.variant == "fused" else wl["roofline_stage"]      # the fused call is timed as the ask stage
    dom_ms = stage_ms[dom_stage] / wl.get("launches", 1)      # average duration of one launch
    achieved = work / (dom_ms * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9)
    out = {
        "metric": "member-evals/sec (pop x samples, or env-steps/s, or pop for the sphere) for one whole ES generation",
        "value": value, "unit": "member-evals/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl["dtype"], "data": "synthetic",
        "config": {"workload": wl["desc"], "pop": c.pop, "P": c.P, "generation": "ask -> rollout -> tell"},
        "stage_ms": stage_ms,
        "roofline": {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(name),
                     "traffic_source": "rocprofv3 --pmc summary under profiles/ of this command (not read in this run)",
                     "kernel": wl["roofline_stage"], "kernel_ms": dom_ms, "bound_detail": BOUND_DETAIL.get(name)},
    }
    if "launches" in wl:
        out["roofline"]["launches_per_generation"] = wl["launches"]
    if "fp32_flops" in wl:      # the same launch priced as the fp32 work it stands for
        tf = wl["fp32_flops"] / (dom_ms * 1e-3) / 1e12
        out["roofline"]["priced_as"] = "fp16 matrix instructions as issued (two-term splits of fp32 operands)"
        out["roofline"]["fp32_equivalent"] = {"achieved": tf, "peak": PEAK_MFMA_F32_TF, "unit": "TFLOP/s",
                                              "frac": tf / PEAK_MFMA_F32_TF}
    if "mfma_f16_issued_work" in wl:
        out["roofline"]["mfma_f16_issued_tflops"] = wl["mfma_f16_issued_work"] / (dom_ms * 1e-3) / 1e12
        out["roofline"]["bound_detail"] = ("fp32 MLP on the matrix cores (mlp_f32_mfma_kernel): one workgroup per CU, a chain of "
                                           "weight-fetch, split and product phases per neuron tile")
        out["roofline"]["traffic"] = None
    if "mfma_tflops_work" in wl:      # the forward's matrix-core rate next to its HBM rate
        out["roofline"]["mfma_bf16_tflops"] = wl["mfma_tflops_work"] / (dom_ms * 1e-3) / 1e12
        out["roofline"]["mfma_bf16_frac"] = out["roofline"]["mfma_bf16_tflops"] / PEAK_MFMA_BF16_TF
    if "hbm_bytes_work" in wl:      # ... and its HBM rate next to its matrix-core rate
        out["roofline"]["hbm_GBs"] = wl["hbm_bytes_work"] / (dom_ms * 1e-3) / 1e9
        out["roofline"]["hbm_frac"] = out["roofline"]["hbm_GBs"] / PEAK_HBM_GBS
        out["roofline"]["bound_detail"] = ("bf16 matrix instructions of the register-resident forward: MFMA busy 42 %, "
                                           "co-limited by LDS operand reads (profiles/mlp_bf16_resident_kernel_cfg4_b2048.md)")
    if args.graph:
        out["config"]["launch"] = "HIP graph replay of one recorded generation; stage_ms from direct calls before it"
    if args.batch is not None:
        out["config"]["batch_override"] = args.batch
        out["roofline"]["traffic"] = None
    if args.variant != "materialised":
        out["config"]["generation"] = {"fused": "pgpe_generation: ask, evaluation, ranks and tell in one launch" if name == "cfg1" else
                                                ("ask_rollout" if name == "cfg4" else "ask_sphere") +
                                                " (ask + fitness in one kernel, no population) -> tell",
                                       "stored": "ask -> rollout -> tell_stored",
                                       "f32": "ask -> rollout -> tell with fp32 parameters"}[args.variant]
        out["roofline"]["traffic"] = None
        if args.variant == "fused" and name == "cfg1":
            out["roofline"]["kernel"] = "generation_small_kernel"
            out["roofline"]["kernel_ms"] = dom_ms
            out["roofline"]["bound_detail"] = "launch latency: one launch whose update workgroups wait for the evaluation"
        elif args.variant == "fused":      # no population is written: the stage is bound by the noise generation
            normals = c.pop / 2 * c.P
            out["roofline"] = {"bound": "alu", "achieved": normals / (dom_ms * 1e-3) / 1e9, "peak": None,
                               "unit": "Gnormal/s", "frac": None, "traffic": None,
                               "kernel": "ask_rollout" if name == "cfg4" else "ask_sphere", "kernel_ms": dom_ms,
                               "bound_detail": "vector instructions of the noise generation (Philox4x32-10 + Box-Muller "
                               "per antithetic pair): no published peak applies; VALU busy " +
                               ("70 % (profiles/mlp_bf16_stream_kernel_cfg4.md)" if name == "cfg4" else
                                "as in profiles/ask_sphere_tell_kernels_cfg5.md")}
    pg.close()
    del wl
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None,
                    choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "seq2seq", "forage", "forage_solo"],
                    help="one workload only; default: cfg2 as the headline plus per_config for cfg1..cfg5")
    ap.add_argument("--seed", type=int, default=20220509)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measured-peak probes")
    ap.add_argument("--batch", type=int, default=None,
                    help="cfg4 only: observations per member (default 64); sweeps the arithmetic intensity of the forward")
    ap.add_argument("--variant", default="materialised", choices=["materialised", "fused", "stored", "f32"],
                    help="cfg5: 'fused' = ask fused with the sphere fitness (no population in memory), 'stored' = tell "
                         "reads the perturbations back from the stored population; cfg4: 'fused' = ask fused into the forward; cfg1: 'fused' = the whole generation in one launch; cfg4: 'f32' = the same shape with fp32 parameters")
    ap.add_argument("--graph", action="store_true",
                    help="replay each generation from a recorded HIP graph (generation index kept on the device); "
                         "the per-stage times then come from an untimed pass of direct calls before the replays")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    headline = args.workload or "cfg2"
    all_configs = args.workload is None and args.batch is None and args.variant == "materialised" and not args.graph
    if args.batch is not None and headline != "cfg4":
        raise SystemExit("--batch applies to --workload cfg4 only")
    if args.variant != "materialised" and not ((headline == "cfg5" and args.variant != "f32") or
                                               (headline in ("cfg1", "cfg4") and args.variant == "fused") or
                                               (headline == "cfg4" and args.variant == "f32")):
        raise SystemExit("--variant applies to --workload cfg5 (fused, stored), cfg1 (fused) and cfg4 (fused, f32) only")
    # the oracle first: its all-cores leg forks worker processes, which must happen before the GPU is initialised
    cpu = None
    if not args.no_cpu_baseline and args.batch is None and args.variant == "materialised":
        cpu = _cpu_baseline(headline, args.seed)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    import paper_2202_05008_amd as evo
    if args.calibrate_copy:      # a copy kernel of known size: reads 1 GiB, writes 1 GiB
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[headline]
    out = _run_workload(headline, args, steps, args.warmup, torch)
    if all_configs:
        per = {}
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
            r = out if name == headline else _run_workload(name, args, DEFAULT_STEPS[name], args.warmup, torch)
            per[name] = {"workload": r["config"]["workload"], "ms_per_generation": r["ms_per_step"], "steps": r["steps"],
                         "value": r["value"], "unit": r["unit"], "dtype": r["dtype"], "stage_ms": r["stage_ms"],
                         "roofline": r["roofline"]}
            if name == "cfg1":      # the same generation as one launch
                fa = argparse.Namespace(**{**vars(args), "variant": "fused"})
                r = _run_workload(name, fa, DEFAULT_STEPS[name], args.warmup, torch)
                per[name]["one_launch"] = {"ms_per_generation": r["ms_per_step"], "value": r["value"],
                                           "generation": r["config"]["generation"]}
            if name == "cfg4":      # the same generation with ask fused into the forward (no population in memory)
                fa = argparse.Namespace(**{**vars(args), "variant": "fused"})
                r = _run_workload(name, fa, DEFAULT_STEPS[name], args.warmup, torch)
                per[name]["ask_fused_into_forward"] = {"ms_per_generation": r["ms_per_step"], "value": r["value"],
                                                       "stage_ms": r["stage_ms"], "roofline": r["roofline"]}
        out["per_config"] = per
    if not args.no_peaks:
        out["measured_peaks"] = _measure_peaks(evo, torch)
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
