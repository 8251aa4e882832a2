"""Seeded synthetic input data (numpy's own PCG64 streams; no method arithmetic here).

Every function returns plain numpy arrays that BOTH the CPU oracle and the HIP path are
fed with.  The recipes mirror the shapes and value distributions of the paper's example
tasks (Section 3): Gaussian class blobs for the plumbing classifier, MNIST-shaped images
(the MNIST example of Section 3 / Table 1; the real data set is not used), per-member
observations with a fixed random teacher, a shifted sphere, and the addition strings of the
sequence-to-sequence example ("012+345=" -> "0357").
"""
import numpy as np


def _rng(seed, *stream):
    return np.random.default_rng([int(seed) & 0xFFFFFFFF, int(seed) >> 32, *[int(s) for s in stream]])


def initial_mu(seed, P, scale=0.1):
    """Initial centre of the search distribution, N(0, scale^2), fp32."""
    return (_rng(seed, 5).standard_normal(P) * scale).astype(np.float32)


def class_blobs(seed, n=512, D=16, n_classes=4, mean_std=2.0):
    """x ~ N(class_mean[y], I), class_mean ~ N(0, mean_std^2 I), y = i mod n_classes."""
    r = _rng(seed, 2, 0)
    means = r.standard_normal((n_classes, D)) * mean_std
    y = (np.arange(n) % n_classes).astype(np.int32)
    x = means[y] + r.standard_normal((n, D))
    return x.astype(np.float32), y


def image_prototypes(seed, n_classes=10, hw=28):
    return _rng(seed, 2, 1).uniform(0.0, 1.0, size=(n_classes, 1, hw, hw))


def mnist_shaped_batch(seed, generation, n=1024, n_classes=10, hw=28, noise=0.1):
    """Images [n,1,hw,hw] in [0,1]: per-class prototype + N(0, noise^2), clipped; balanced labels.
    The prototypes depend on `seed` only; the noise is re-drawn for every generation."""
    proto = image_prototypes(seed, n_classes, hw)
    y = (np.arange(n) % n_classes).astype(np.int32)
    eps = _rng(seed, 2, 2, generation).standard_normal((n, 1, hw, hw)) * noise
    img = np.clip(proto[y] + eps, 0.0, 1.0)
    return img.astype(np.float32), y


def teacher_regression(seed, pop, B, dims):
    """Per-member observations obs[pop,B,dims[0]] ~ N(0,1) and the outputs of one fixed random
    ReLU teacher network of widths `dims` (weights ~ N(0, 1/fan_in), zero biases)."""
    r = _rng(seed, 3)
    Ws = [r.standard_normal((dims[i], dims[i + 1])) / np.sqrt(dims[i]) for i in range(len(dims) - 1)]
    obs = _rng(seed, 4).standard_normal((pop, B, dims[0])).astype(np.float32)
    h = obs.astype(np.float64)
    for i, W in enumerate(Ws):
        h = h @ W
        if i + 1 < len(Ws):
            h = np.maximum(h, 0.0)
    return obs, h.astype(np.float32)


def sphere_target(seed, P):
    return _rng(seed, 2, 3).standard_normal(P).astype(np.float32)


def random_params(seed, pop, P, scale=0.3):
    return (_rng(seed, 6).standard_normal((pop, P)) * scale).astype(np.float32)


def random_fitness(seed, pop, ties=0, specials=False):
    """Fitness vector for rank/tell tests.  `ties` > 0 quantises to that many distinct values;
    `specials` plants +-0, +-inf and NaN entries."""
    r = _rng(seed, 7)
    f = r.standard_normal(pop).astype(np.float32) * 3.0
    if ties:
        f = np.round(f * ties / 6.0).astype(np.float32)
    if specials and pop >= 8:
        idx = r.permutation(pop)[:6]
        f[idx[0]] = 0.0
        f[idx[1]] = -0.0
        f[idx[2]] = np.inf
        f[idx[3]] = -np.inf
        f[idx[4]] = np.nan
        f[idx[5]] = np.nan
    return f


def random_states(seed, n, scale=1.0):
    """Cart-pole states (x, x_dot, theta, theta_dot) and actions in (-1,1) for single-step tests."""
    r = _rng(seed, 8)
    s = r.standard_normal((n, 4)) * np.array([1.0, 2.0, 3.0, 4.0]) * scale
    a = np.tanh(r.standard_normal(n))
    return s.astype(np.float32), a.astype(np.float32)


def addition_batch(seed, generation, n=128, digits=3):
    """Token strings for the addition of two random integers below 10^digits, zero-padded to equal
    lengths as in the paper's sequence-to-sequence example: query[n, 2 digits + 2] =
    "aaa+bbb=" with '+' = 10 and '=' = 11, answer[n, digits + 1] = the decimal digits of the sum,
    most significant first.  int32."""
    r = _rng(seed, 9, generation)
    a = r.integers(0, 10 ** digits, n)
    b = r.integers(0, 10 ** digits, n)

    def dec(x, width):
        return np.stack([(x // 10 ** (width - 1 - i)) % 10 for i in range(width)], axis=1)

    query = np.concatenate([dec(a, digits), np.full((n, 1), 10), dec(b, digits), np.full((n, 1), 11)], axis=1)
    return query.astype(np.int32), dec(a + b, digits + 1).astype(np.int32)
