"""Thin Python binding of the C ABI (include/evo.h): argument marshalling only.

Every function has the name of the C entry point it calls.  torch tensors supply device
memory and the current HIP stream; all arithmetic runs in the library's kernels."""
import ctypes as C

import torch

from . import _lib
from ._lib import pgpe_config, policy_desc, task_desc

EVO_F32, EVO_BF16 = 0, 1
EVO_ACT_NONE, EVO_ACT_TANH, EVO_ACT_RELU = 0, 1, 2
EVO_POLICY_MLP, EVO_POLICY_CONVNET, EVO_POLICY_LSTM_SEQ2SEQ = 0, 1, 2
EVO_TASK_CLASSIFY, EVO_TASK_REGRESS, EVO_TASK_CARTPOLE, EVO_TASK_SPHERE, EVO_TASK_SEQ2SEQ, EVO_TASK_FORAGE, EVO_TASK_FORAGE_SOLO = range(7)
EVO_TAG_NOISE, EVO_TAG_RESET, EVO_TAG_WORLD_AGENT, EVO_TAG_WORLD_ITEM = 0, 1, 2, 3
EVO_OPT_ADAM, EVO_OPT_CLIPUP, EVO_OPT_MOMENTUM = 0, 1, 2


class EvoError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("evo error %d: %s" % (code, message))
        self.code = code


def _check(rc):
    if rc != 0:
        raise EvoError(rc, _lib.load().evo_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype=None, allow_none=False):
    if t is None:
        if allow_none:
            return C.c_void_p(0)
        raise ValueError("tensor argument is None")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    return C.c_void_p(t.data_ptr())


def evo_version():
    return _lib.load().evo_version().decode()


def make_pgpe_config(P, pop_max, **fields):
    """pgpe_config_defaults, then the fields given by name; an unnamed max_speed follows lr_mu (the library's rule)."""
    lib = _lib.load()
    cfg = pgpe_config()
    _check(lib.pgpe_config_defaults(C.byref(cfg), P, pop_max))
    max_speed = fields.pop("max_speed", None)
    for name, value in fields.items():
        if name not in dict(pgpe_config._fields_):
            raise TypeError("pgpe_config has no field %r" % name)
        setattr(cfg, name, value)
    cfg.max_speed = lib.pgpe_clipup_default_max_speed(cfg.lr_mu) if max_speed is None else max_speed
    return cfg


def make_policy_desc(kind, dims, act=(), dtype=EVO_F32):
    pd = policy_desc()
    pd.kind = kind
    pd.n_layers = len(dims) - 1 if kind == EVO_POLICY_MLP else 0
    for i, d in enumerate(dims):
        pd.dims[i] = d
    for i, a in enumerate(act):
        pd.act[i] = a
    pd.dtype = dtype
    return pd


def make_task_desc(kind, n_rollouts=1, B=0, P=0, reset_seed=0, generation=1, obs=None, obs_member_stride=0,
                   target=None, cp=None, init_scale=0.2, work=None, seq_in=0, seq_out=0, generation_dev=None):
    td = task_desc()
    td.kind, td.n_rollouts, td.B, td.P = kind, n_rollouts, B, P
    td.seq_in, td.seq_out = seq_in, seq_out
    td.reset_seed, td.generation = reset_seed, generation
    td.obs_dev = obs.data_ptr() if obs is not None else None
    td.obs_member_stride = obs_member_stride
    td.target_dev = target.data_ptr() if target is not None else None
    if cp is not None:
        for i, v in enumerate(cp):
            td.cp[i] = v
    td.init_scale = init_scale
    td.work_dev = work.data_ptr() if work is not None else None
    td.generation_dev = generation_dev
    td._keepalive = (obs, target, work)
    return td


def pgpe_workspace_bytes(cfg):
    return int(_lib.load().pgpe_workspace_bytes(C.byref(cfg)))


def pgpe_create(cfg, mu, sigma, m, v, aux, work):
    """Returns the opaque handle (keep the tensors alive as long as it is used)."""
    h = C.c_void_p()
    _check(_lib.load().pgpe_create(C.byref(h), C.byref(cfg), _ptr(mu, torch.float32), _ptr(sigma, torch.float32),
                                   _ptr(m, torch.float32), _ptr(v, torch.float32),
                                   _ptr(aux, torch.float32, allow_none=True), _ptr(work)))
    return h


def pgpe_destroy(h):
    _check(_lib.load().pgpe_destroy(h))


def pgpe_reset(h):
    _check(_lib.load().pgpe_reset(h, _stream()))


def pgpe_get_generation(h):
    t = C.c_uint32()
    _check(_lib.load().pgpe_get_generation(h, C.byref(t)))
    return t.value


def pgpe_set_generation(h, t):
    _check(_lib.load().pgpe_set_generation(h, t))


def pgpe_center(h, rows, params, dtype=EVO_F32):
    want = torch.float32 if dtype == EVO_F32 else torch.bfloat16
    _check(_lib.load().pgpe_center(h, rows, _ptr(params, want), dtype, _stream()))


def pgpe_state_bytes(h):
    return int(_lib.load().pgpe_state_bytes(h))


def pgpe_state_export(h):
    """The state as a bytes object (header + arrays); waits for the current stream."""
    n = pgpe_state_bytes(h)
    buf = C.create_string_buffer(n)
    _check(_lib.load().pgpe_state_export(h, buf, n, _stream()))
    return buf.raw


def pgpe_state_import(h, blob):
    buf = C.create_string_buffer(bytes(blob), len(blob))
    _check(_lib.load().pgpe_state_import(h, buf, len(blob), _stream()))


def pgpe_device_generation(h):
    """Keep the generation index on the device too (for HIP-graph replays); returns its device address."""
    p = C.c_void_p()
    _check(_lib.load().pgpe_device_generation(h, C.byref(p), _stream()))
    return p.value


def pgpe_sync_generation(h):
    _check(_lib.load().pgpe_sync_generation(h, _stream()))


def pgpe_ask(h, seed, pop, params, dtype=EVO_F32):
    want = torch.float32 if dtype == EVO_F32 else torch.bfloat16
    _check(_lib.load().pgpe_ask(h, seed, pop, _ptr(params, want), dtype, _stream()))


def pgpe_tell(h, fitness):
    _check(_lib.load().pgpe_tell(h, _ptr(fitness, torch.float32), _stream()))


def pgpe_ask_sphere_workspace_bytes(cfg):
    return int(_lib.load().pgpe_ask_sphere_workspace_bytes(C.byref(cfg)))


def pgpe_ask_sphere(h, seed, pop, x_star, fitness, work):
    _check(_lib.load().pgpe_ask_sphere(h, seed, pop, _ptr(x_star, torch.float32), _ptr(fitness, torch.float32),
                                       _ptr(work), _stream()))


def pgpe_ask_rollout(h, seed, pop, td, pd, fitness):
    _check(_lib.load().pgpe_ask_rollout(h, seed, pop, C.byref(td), C.byref(pd), _ptr(fitness, torch.float32), _stream()))


def pgpe_generation(h, seed, pop, td, pd, fitness):
    _check(_lib.load().pgpe_generation(h, seed, pop, C.byref(td), C.byref(pd), _ptr(fitness, torch.float32), _stream()))


def evo_ask_forward(h, seed, pop, pd, obs, obs_member_stride, out, B):
    _check(_lib.load().evo_ask_forward(h, seed, pop, C.byref(pd), _ptr(obs, torch.float32), obs_member_stride,
                                       _ptr(out, torch.float32), B, _stream()))


def pgpe_tell_stored(h, fitness, params):
    _check(_lib.load().pgpe_tell_stored(h, _ptr(fitness, torch.float32), _ptr(params, torch.float32), _stream()))


def policy_param_count(pd):
    n = _lib.load().policy_param_count(C.byref(pd))
    if n < 0:
        _check(int(n))
    return int(n)


def pop_forward(pd, params, obs, obs_member_stride, out, pop, B):
    _check(_lib.load().pop_forward(C.byref(pd), _ptr(params), _ptr(obs, torch.float32), obs_member_stride,
                                   _ptr(out, torch.float32), pop, B, _stream()))


def rollout_workspace_bytes(td, pd, pop):
    return int(_lib.load().rollout_workspace_bytes(C.byref(td), C.byref(pd) if pd is not None else None, pop))


def rollout(td, pd, params, pop, steps, fitness):
    _check(_lib.load().rollout(C.byref(td), C.byref(pd) if pd is not None else None, _ptr(params), pop, steps,
                               _ptr(fitness, torch.float32), _stream()))


def rollout_static_scratch_bytes():
    return int(_lib.load().rollout_static_scratch_bytes())


def rollout_static_scratch(td, pd, params, pop, steps, fitness):
    """rollout with the workspace inside the library (no allocation anywhere); td.work_dev is ignored."""
    _check(_lib.load().rollout_static_scratch(C.byref(td), C.byref(pd) if pd is not None else None, _ptr(params),
                                              pop, steps, _ptr(fitness, torch.float32), _stream()))


def evo_philox_u32(seed, gen, pair, block0, nblocks, tag, out):
    _check(_lib.load().evo_philox_u32(seed, gen, pair, block0, nblocks, tag, _ptr(out, torch.int32), _stream()))


def evo_philox_normal(seed, gen, pair, block0, nblocks, tag, out):
    _check(_lib.load().evo_philox_normal(seed, gen, pair, block0, nblocks, tag, _ptr(out, torch.float32), _stream()))


def evo_centered_rank(fitness, pop, rank, shaped):
    _check(_lib.load().evo_centered_rank(_ptr(fitness, torch.float32), pop, _ptr(rank, torch.int32),
                                         _ptr(shaped, torch.float32), _stream()))


def evo_pgpe_gradients(h, fitness, gmu, gsigma, params=None):
    _check(_lib.load().evo_pgpe_gradients(h, _ptr(fitness, torch.float32), _ptr(gmu, torch.float32),
                                          _ptr(gsigma, torch.float32),
                                          _ptr(params, torch.float32, allow_none=True), _stream()))


def evo_seq2seq_logits(td, pd, params, pop, logits):
    _check(_lib.load().evo_seq2seq_logits(C.byref(td), C.byref(pd), _ptr(params, torch.float32), pop,
                                          _ptr(logits, torch.float32), _stream()))


def evo_task_step(td, state, action, nxt, reward, n):
    _check(_lib.load().evo_task_step(C.byref(td), _ptr(state, torch.float32), _ptr(action, torch.float32),
                                     _ptr(nxt, torch.float32), _ptr(reward, torch.float32), n, _stream()))


def evo_forage_step(td, pop, pos, vel, counts, action, obs, next_pos, next_vel, reward, hit):
    f32, i32 = torch.float32, torch.int32
    _check(_lib.load().evo_forage_step(C.byref(td), pop, _ptr(pos, f32), _ptr(vel, f32), _ptr(counts, i32),
                                       _ptr(action, f32), _ptr(obs, f32), _ptr(next_pos, f32), _ptr(next_vel, f32),
                                       _ptr(reward, i32), _ptr(hit, i32), _stream()))


def evo_forage_state(td, pd, params, pop, steps, pos=None, vel=None, reward=None, counts=None):
    f32, i32 = torch.float32, torch.int32
    _check(_lib.load().evo_forage_state(C.byref(td), C.byref(pd), _ptr(params), pop, steps,
                                        _ptr(pos, f32, allow_none=True), _ptr(vel, f32, allow_none=True),
                                        _ptr(reward, i32, allow_none=True), _ptr(counts, i32, allow_none=True),
                                        _stream()))


def evo_rollout_details(td, pd, params, pop, steps, ret, final):
    _check(_lib.load().evo_rollout_details(C.byref(td), C.byref(pd), _ptr(params), pop, steps,
                                           _ptr(ret, torch.float32, allow_none=True),
                                           _ptr(final, torch.float32, allow_none=True), _stream()))


def evo_rollout_trace(td, pd, params, pop, steps, trace, final=None):
    _check(_lib.load().evo_rollout_trace(C.byref(td), C.byref(pd), _ptr(params), pop, steps,
                                         _ptr(trace, torch.float32),
                                         _ptr(final, torch.float32, allow_none=True), _stream()))


def evo_probe_rate(kind, iters, out):
    """Enqueue one rate probe; returns the floating-point operations it performs (the caller times it)."""
    flop = C.c_double()
    _check(_lib.load().evo_probe_rate(kind, iters, C.byref(flop), _ptr(out, torch.float32), _stream()))
    return flop.value


class PGPE:
    """Convenience owner of the device arrays behind one pgpe_state handle."""

    def __init__(self, cfg, mu0=None, device="cuda:0"):
        self.cfg = cfg
        P = cfg.P
        dev = torch.device(device)
        self.mu = torch.zeros(P, dtype=torch.float32, device=dev)
        if mu0 is not None:
            self.mu.copy_(torch.as_tensor(mu0, dtype=torch.float32))
        self.sigma = torch.empty(P, dtype=torch.float32, device=dev)
        self.m = torch.empty(P, dtype=torch.float32, device=dev)
        self.v = torch.empty(P, dtype=torch.float32, device=dev)
        self.aux = torch.empty(2 * P, dtype=torch.float32, device=dev) if cfg.sigma_rule == 1 else None
        self.work = torch.empty(pgpe_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
        self.handle = pgpe_create(cfg, self.mu, self.sigma, self.m, self.v, self.aux, self.work)
        pgpe_reset(self.handle)

    def ask(self, seed, pop, params, dtype=EVO_F32):
        pgpe_ask(self.handle, seed, pop, params, dtype)

    def tell(self, fitness):
        pgpe_tell(self.handle, fitness)

    def ask_sphere(self, seed, pop, x_star, fitness):
        if getattr(self, "_sphere_work", None) is None:
            self._sphere_work = torch.empty(pgpe_ask_sphere_workspace_bytes(self.cfg), dtype=torch.uint8,
                                            device=self.mu.device)
        pgpe_ask_sphere(self.handle, seed, pop, x_star, fitness, self._sphere_work)

    def ask_rollout(self, seed, pop, td, pd, fitness):
        pgpe_ask_rollout(self.handle, seed, pop, td, pd, fitness)

    def generation_step(self, seed, pop, td, pd, fitness):
        """ask, evaluation and tell in one launch (small supervised problems; EvoError otherwise)."""
        pgpe_generation(self.handle, seed, pop, td, pd, fitness)

    def tell_stored(self, fitness, params):
        pgpe_tell_stored(self.handle, fitness, params)

    def center(self, rows, params, dtype=EVO_F32):
        pgpe_center(self.handle, rows, params, dtype)

    def export_state(self):
        return pgpe_state_export(self.handle)

    def import_state(self, blob):
        pgpe_state_import(self.handle, blob)

    def device_generation(self):
        """Switch to a device-resident generation index (graph replays then advance it); returns its address."""
        self._gen_dev = pgpe_device_generation(self.handle)
        return self._gen_dev

    @property
    def generation(self):
        if getattr(self, "_gen_dev", None):
            pgpe_sync_generation(self.handle)      # replays advance only the device copy
        return pgpe_get_generation(self.handle)

    def close(self):
        if self.handle is not None:
            pgpe_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
