"""CPU ORACLE (test infrastructure, not part of the product path) -- PGPE ask / tell.

The paper names PGPE as its released algorithm (Section 5) behind the ask/tell
interface (Section 4, "Devising New Algorithms") and says gradient estimates are fed to
deep-learning optimizers (Section 2, "Modern ML Optimizers"); it prints no formula.  This
file writes out the symmetric-sampling PGPE estimator of the works cited there, with
perturbations eps = sigma * z, centered-rank fitness shaping and an Adam ascent step:

  ask :  theta[2k]   = mu + sigma * z_k,   theta[2k+1] = mu - sigma * z_k        (k < N = pop/2)
  rank:  r_m = position of (fitness_m, m) in ascending order; c_m = (2 r_m - (pop-1)) / (2 (pop-1))
  tell:  b = mean(c);  w_k = (c[2k] - c[2k+1]) / 2;  u_k = (c[2k] + c[2k+1]) / 2 - b
         g_mu    = sigma / N * sum_k w_k z_k
         g_sigma = sigma / N * sum_k u_k (z_k^2 - 1)
         Adam ascent on mu (bias-corrected, eps outside the square root, t starts at 1); or, by
         cfg.optimizer, ClipUp (the optimizer cited with PGPE in Section 5: velocity of bounded
         norm fed by the normalised gradient) or plain momentum ascent
         sigma: rule 0: sigma += clip(lr_sigma * g_sigma, -c_max sigma, +c_max sigma)
                rule 1: Adam ascent with its own moments, then sigma = max(sigma, 1e-8)

All arithmetic is fp64 on fp32-representable inputs; state arrays are rounded to fp32
after every tell because that is the precision they are stored in.
Pins: tests/test_oracle_pgpe.py (brute force on tiny populations, closed-form expected
gradients, pair-swap / shift identities, the stored-population form against the
regenerating one, Adam closed forms, ClipUp / momentum closed forms
and a library optimizer, sphere convergence).
"""
from dataclasses import dataclass, field
import numpy as np

from . import philox

DT_F32, DT_BF16 = 0, 1


@dataclass
class PGPEConfig:
    P: int
    pop_max: int = 4096
    sigma_init: float = 0.1
    lr_mu: float = 0.01
    lr_sigma: float = 0.1
    sigma_max_change: float = 0.2
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    sigma_rule: int = 0     # 0 clipped ascent, 1 Adam
    shaping: int = 1        # 1 centered ranks, 0 raw fitness
    optimizer: int = 0      # update of mu: 0 Adam, 1 ClipUp, 2 momentum ascent (velocity kept in m)
    momentum: float = 0.9   # ClipUp / momentum ascent
    max_speed: float = 0.02  # ClipUp: bound on the norm of the velocity (customarily 2 lr_mu)

    def __post_init__(self):
        # the hyper-parameters cross the library boundary as fp32: the oracle computes in fp64 on
        # those fp32 values (e.g. 1 - beta2 is taken from float32(0.999), not from 0.999)
        for name in ("sigma_init", "lr_mu", "lr_sigma", "sigma_max_change", "beta1", "beta2", "eps", "momentum",
                     "max_speed"):
            setattr(self, name, float(np.float32(getattr(self, name))))


@dataclass
class PGPEState:
    cfg: PGPEConfig
    mu: np.ndarray
    sigma: np.ndarray
    m: np.ndarray = None
    v: np.ndarray = None
    m_sigma: np.ndarray = None
    v_sigma: np.ndarray = None
    t: int = 1              # generation index of the NEXT ask
    last: tuple = field(default=None)   # (seed, pop, t) of the pending ask

    @classmethod
    def create(cls, cfg, mu0=None):
        P = cfg.P
        mu = np.zeros(P, np.float32) if mu0 is None else np.asarray(mu0, np.float32).copy()
        z = lambda: np.zeros(P, np.float32)
        return cls(cfg, mu, np.full(P, cfg.sigma_init, np.float32), z(), z(), z(), z())


def round_to_bf16(x32):
    """Round-to-nearest-even of fp32 values to bfloat16, returned as fp32 values.
    NaN stays NaN (quiet); overflow rounds to infinity as RNE prescribes."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    bits = x32.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = ((bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    out = (rounded & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.float32)
    nan = np.isnan(x32)
    if nan.any():
        out = out.copy()
        out[nan] = np.float32(np.nan)
    return out


def ask_rows(state, seed, pop, members=None, cols=None, dtype=DT_F32):
    """theta[m, i] for the requested members / columns (default all) of the population that
    `ask(seed, pop)` would generate at the state's current generation; fp32 values."""
    if pop <= 0 or pop % 2:
        raise ValueError("pop must be a positive even number")
    members = np.arange(pop) if members is None else np.asarray(members, dtype=np.int64)
    P = state.cfg.P
    mu = state.mu.astype(np.float64)
    sg = state.sigma.astype(np.float64)
    if cols is not None:
        cols = np.asarray(cols, dtype=np.int64)
        mu, sg = mu[cols], sg[cols]
    z = philox.pair_noise(seed, state.t, members >> 1, P, cols)
    sign = np.where(members & 1, -1.0, 1.0)[:, None]
    theta = (mu[None, :] + sign * (sg[None, :] * z)).astype(np.float32)
    if dtype == DT_BF16:
        theta = round_to_bf16(theta)
    return theta


def ask(state, seed, pop, dtype=DT_F32):
    """Generate the whole population and remember (seed, pop) for the matching tell."""
    theta = ask_rows(state, seed, pop, dtype=dtype)
    state.last = (int(seed), int(pop), state.t)
    return theta


def orderable_key(f32):
    """Monotone map fp32 -> u32: -0 counts as +0, every NaN becomes the lowest key."""
    f = np.ascontiguousarray(f32, dtype=np.float32).copy()
    f[f == 0.0] = 0.0                                  # -0 -> +0
    bits = f.view(np.uint32)
    neg = (bits >> np.uint32(31)).astype(bool)
    key = np.where(neg, ~bits, bits | np.uint32(0x80000000)).astype(np.uint32)
    key[np.isnan(f)] = 0
    return key


def centered_rank(fitness):
    """(rank u32[pop], c fp32[pop]).  Ascending stable rank with index tie-break; the worst
    member gets rank 0 -> c = -0.5, the best rank pop-1 -> c = +0.5.  c is one correctly
    rounded fp32 division of two exactly representable integers."""
    f = np.asarray(fitness, dtype=np.float32)
    pop = f.shape[0]
    key = (orderable_key(f).astype(np.uint64) << np.uint64(32)) | np.arange(pop, dtype=np.uint64)
    order = np.argsort(key)                 # keys are unique: one correct permutation
    rank = np.empty(pop, dtype=np.uint32)
    rank[order] = np.arange(pop, dtype=np.uint32)
    if pop == 1:
        return rank, np.zeros(1, np.float32)
    num = (2 * rank.astype(np.int64) - (pop - 1)).astype(np.float32)
    den = np.float32(2 * (pop - 1))
    return rank, (num / den).astype(np.float32)


def pair_weights(c):
    """w_k, u_k (fp64) from per-member utilities c (shaped or raw)."""
    c = np.asarray(c, dtype=np.float64)
    b = c.mean()
    return (c[0::2] - c[1::2]) / 2.0, (c[0::2] + c[1::2]) / 2.0 - b


def gradients(z, sigma, c):
    """g_mu, g_sigma (fp64) from materialised noise z[N,P], sigma[P] and utilities c[pop]."""
    w, u = pair_weights(c)
    N = z.shape[0]
    sg = np.asarray(sigma, dtype=np.float64)
    g_mu = sg * (w @ z) / N
    g_sigma = sg * (u @ (z * z - 1.0)) / N
    return g_mu, g_sigma


def gradients_from_population(theta_plus, mu, sigma, c):
    """The same estimate taken from the STORED population instead of regenerated noise: with
    eps_k = theta[2k] - mu (the perturbation of the + member of pair k, as it was rounded when
    the population was written),
        g_mu = 1/N sum_k w_k eps_k,      g_sigma = 1/N sum_k u_k (eps_k^2 - sigma^2) / sigma,
    which is `gradients` with eps = sigma z.  A parameter with sigma = 0 has eps = 0 and gets
    g_sigma = 0.  theta_plus[N,P] holds the even rows of the population; fp64 throughout."""
    w, u = pair_weights(c)
    mu = np.asarray(mu, dtype=np.float64)
    sg = np.asarray(sigma, dtype=np.float64)
    eps = np.asarray(theta_plus, dtype=np.float64) - mu[None, :]
    N = eps.shape[0]
    g_mu = (w @ eps) / N
    safe = np.where(sg > 0.0, sg, 1.0)
    g_sigma = np.where(sg > 0.0, (u @ (eps * eps - (sg * sg)[None, :])) / safe / N, 0.0)
    return g_mu, g_sigma


def adam_ascent(x, m, v, g, lr, beta1, beta2, eps, t):
    """One bias-corrected Adam step that INCREASES the objective; returns (x, m, v) in fp64."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return x + lr * m_hat / (np.sqrt(v_hat) + eps), m, v


def clipup_ascent(x, vel, g, step, momentum, max_speed):
    """One ClipUp step that INCREASES the objective (Toklu, Liskowski, Srivastava 2020): the
    velocity takes momentum * velocity + step * g / |g| (only the direction of the gradient
    enters), is scaled back to norm max_speed if longer, and is added to x.  Returns (x, vel)."""
    g = np.asarray(g, dtype=np.float64)
    norm = np.sqrt(np.sum(g * g))
    vel = momentum * vel + (step * g / norm if norm > 0.0 else 0.0)
    speed = np.sqrt(np.sum(vel * vel))
    if speed > max_speed:
        vel = vel * (max_speed / speed)
    return x + vel, vel


def momentum_ascent(x, vel, g, lr, momentum):
    """Heavy-ball ascent: velocity = momentum * velocity + lr * g; x += velocity.  Returns (x, vel)."""
    vel = momentum * vel + lr * np.asarray(g, dtype=np.float64)
    return x + vel, vel


def utilities(state, fitness):
    f = np.asarray(fitness, dtype=np.float32)
    return centered_rank(f)[1] if state.cfg.shaping == 1 else f


def tell(state, fitness, chunk=1 << 15, return_grads=False, stored=None):
    """Consume the fitness of the pending ask and update (mu, sigma, moments, t).
    The noise is regenerated from the counter-based stream in column chunks; or, when `stored`
    is the population [pop,P] that ask wrote (fp32), the perturbations are read back from its
    even rows (`gradients_from_population`)."""
    if state.last is None:
        raise RuntimeError("tell without a pending ask")
    seed, pop, t = state.last
    f = np.asarray(fitness, dtype=np.float32)
    if f.shape != (pop,):
        raise ValueError("fitness must have shape [pop]")
    cfg = state.cfg
    c = utilities(state, f)
    w, u = pair_weights(c)
    N, P = pop // 2, cfg.P
    g_mu = np.empty(P)
    g_sg = np.empty(P)
    sg = state.sigma.astype(np.float64)
    pairs = np.arange(N)
    for lo in range(0, P, chunk):
        hi = min(P, lo + chunk)
        if stored is not None:
            g_mu[lo:hi], g_sg[lo:hi] = gradients_from_population(np.asarray(stored)[0::2, lo:hi], state.mu[lo:hi],
                                                                 sg[lo:hi], c)
            continue
        lo4 = lo & ~3
        z = philox.block_normals(seed, np.arange(lo4 >> 2, (hi + 3) >> 2)[None, :], pairs[:, None], t,
                                 philox.TAG_NOISE).reshape(N, -1)[:, lo - lo4: hi - lo4]
        g_mu[lo:hi] = sg[lo:hi] * (w @ z) / N
        g_sg[lo:hi] = sg[lo:hi] * (u @ (z * z - 1.0)) / N
    mu0, m0, v = state.mu.astype(np.float64), state.m.astype(np.float64), state.v.astype(np.float64)
    if cfg.optimizer == 0:
        mu, m, v = adam_ascent(mu0, m0, v, g_mu, cfg.lr_mu, cfg.beta1, cfg.beta2, cfg.eps, t)
    elif cfg.optimizer == 1:
        mu, m = clipup_ascent(mu0, m0, g_mu, cfg.lr_mu, cfg.momentum, cfg.max_speed)
    elif cfg.optimizer == 2:
        mu, m = momentum_ascent(mu0, m0, g_mu, cfg.lr_mu, cfg.momentum)
    else:
        raise ValueError("optimizer must be 0 (Adam), 1 (ClipUp) or 2 (momentum)")
    if cfg.sigma_rule == 0:
        lim = cfg.sigma_max_change * sg
        new_sg = sg + np.clip(cfg.lr_sigma * g_sg, -lim, lim)
    else:
        new_sg, ms, vs = adam_ascent(sg, state.m_sigma.astype(np.float64), state.v_sigma.astype(np.float64),
                                     g_sg, cfg.lr_sigma, cfg.beta1, cfg.beta2, cfg.eps, t)
        new_sg = np.maximum(new_sg, 1e-8)
        state.m_sigma, state.v_sigma = ms.astype(np.float32), vs.astype(np.float32)
    state.mu, state.m, state.v = mu.astype(np.float32), m.astype(np.float32), v.astype(np.float32)
    state.sigma = new_sg.astype(np.float32)
    state.t = t + 1
    state.last = None
    if return_grads:
        return g_mu, g_sg
    return None
