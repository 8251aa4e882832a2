"""Pins for oracle/policy.py: the explicit nested-loop definitions, library routines
(torch.nn.functional in fp64, scipy.signal) and zero-weight closed forms."""
import numpy as np
import torch
import torch.nn.functional as F
from scipy import signal

from oracle import policy, tasks
from workloads import mlp_param_count, convnet_param_count


def test_param_counts_of_the_named_workloads():
    assert mlp_param_count((16, 32, 4)) == 676
    assert mlp_param_count((5, 64, 64, 1)) == 4609
    assert mlp_param_count((64, 256, 256, 16)) == 86544
    assert convnet_param_count(8, 16, 10, 28) == 9098


def test_mlp_against_loops_and_torch_linear():
    dims, acts = (3, 4, 2), (policy.ACT_TANH, policy.ACT_RELU)
    rng = np.random.default_rng(0)
    P = mlp_param_count(dims)
    params = rng.standard_normal((2, P))
    obs = rng.standard_normal((5, 3))
    got = policy.mlp_forward(params, obs, dims, acts)
    for m in range(2):
        th = params[m]
        for b in range(5):
            h = list(obs[b])
            off = 0
            for li in range(2):
                n_in, n_out = dims[li], dims[li + 1]
                new = []
                for o in range(n_out):
                    acc = th[off + n_in * n_out + o]
                    for i in range(n_in):
                        acc += h[i] * th[off + i * n_out + o]          # W[in][out], out contiguous
                    new.append(np.tanh(acc) if acts[li] == policy.ACT_TANH else max(acc, 0.0))
                off += n_in * n_out + n_out
                h = new
            np.testing.assert_allclose(got[m, b], h, rtol=1e-12)
    # library routine: torch linear takes weight[out,in] = W^T
    (W0, b0), (W1, b1) = policy.mlp_unpack(params[1], dims)
    t = torch.tanh(F.linear(torch.tensor(obs), torch.tensor(W0.T.copy()), torch.tensor(b0)))
    t = torch.relu(F.linear(t, torch.tensor(W1.T.copy()), torch.tensor(b1)))
    np.testing.assert_allclose(got[1], t.numpy(), rtol=1e-12, atol=1e-14)
    # per-member observations
    obs3 = rng.standard_normal((2, 5, 3))
    got3 = policy.mlp_forward(params, obs3, dims, acts)
    np.testing.assert_allclose(got3[1], policy.mlp_forward(params[1:2], obs3[1], dims, acts)[0])


def test_conv3x3_against_nested_loops_and_scipy():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 6, 6, 3))
    W = rng.standard_normal((3, 3, 3, 4))
    b = rng.standard_normal(4)
    got = policy.conv3x3_same(x, W, b)
    want = np.zeros_like(got)
    for n in range(2):
        for h in range(6):
            for w in range(6):
                for o in range(4):
                    acc = b[o]
                    for dy in range(3):
                        for dx in range(3):
                            hh, ww = h + dy - 1, w + dx - 1
                            if 0 <= hh < 6 and 0 <= ww < 6:
                                for c in range(3):
                                    acc += x[n, hh, ww, c] * W[dy, dx, c, o]
                    want[n, h, w, o] = acc
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    sc = sum(signal.correlate2d(x[0, :, :, c], W[:, :, c, 1], mode="same") for c in range(3)) + b[1]
    np.testing.assert_allclose(got[0, :, :, 1], sc, rtol=1e-12, atol=1e-13)


def test_convnet_against_torch_functional():
    c1, c2, n_cls, hw, B = 8, 16, 10, 28, 3
    rng = np.random.default_rng(2)
    P = convnet_param_count(c1, c2, n_cls, hw)
    params = rng.standard_normal((2, P)) * 0.2
    img = rng.uniform(0, 1, size=(B, 1, hw, hw))
    got = policy.convnet_forward(params, img, c1, c2, n_cls)
    for m in range(2):
        W1, b1, W2, b2, Wd, bd = policy.convnet_unpack(params[m], c1, c2, n_cls, hw)
        t = torch.tensor(img)
        t = F.max_pool2d(torch.relu(F.conv2d(t, torch.tensor(W1.transpose(3, 2, 0, 1).copy()), torch.tensor(b1), padding=1)), 2)
        t = F.max_pool2d(torch.relu(F.conv2d(t, torch.tensor(W2.transpose(3, 2, 0, 1).copy()), torch.tensor(b2), padding=1)), 2)
        t = t.permute(0, 2, 3, 1).reshape(B, -1)                       # (h, w, c) with c fastest
        t = t @ torch.tensor(Wd) + torch.tensor(bd)
        np.testing.assert_allclose(got[m], t.numpy(), rtol=1e-11, atol=1e-12)


def test_flatten_order_and_pooling():
    c1, c2, n_cls, hw = 2, 3, 4, 8
    P = convnet_param_count(c1, c2, n_cls, hw)
    x = np.arange(2 * 4 * 4 * 1, dtype=np.float64).reshape(2, 4, 4, 1)
    p = policy.maxpool2(x)
    assert p.shape == (2, 2, 2, 1) and p[0, 0, 0, 0] == 5 and p[0, 1, 1, 0] == 15 and p[1, 0, 1, 0] == 16 + 7
    # a network whose conv layers copy the centre pixel: dense weight at (h, w, c) picks that feature
    th = np.zeros(P)
    W1, b1, W2, b2, Wd, bd = policy.convnet_unpack(th, c1, c2, n_cls, hw)
    W1[1, 1, 0, 0] = 1.0
    W2[1, 1, 0, 2] = 1.0
    hsel, wsel, csel = 1, 0, 2
    Wd[(hsel * 2 + wsel) * c2 + csel, 3] = 1.0
    img = np.random.default_rng(3).uniform(0, 1, size=(1, 1, hw, hw))
    out = policy.convnet_forward(th[None], img, c1, c2, n_cls)
    want = img[0, 0, 4 * hsel:4 * hsel + 4, 4 * wsel:4 * wsel + 4].max()
    np.testing.assert_allclose(out[0, 0], [0, 0, 0, want], atol=1e-15)


def test_zero_weights_give_bias_and_log_classes():
    rng = np.random.default_rng(4)
    P = convnet_param_count()
    img = rng.uniform(0, 1, size=(20, 1, 28, 28))
    y = np.arange(20) % 10
    out = policy.convnet_forward(np.zeros((1, P)), img)
    assert (out == 0).all()
    np.testing.assert_allclose(tasks.classify_fitness(out, y), -np.log(10.0), rtol=1e-14)
    P = mlp_param_count((16, 32, 4))
    th = np.zeros((1, P))
    th[0, -4:] = [0.5, -1.0, 2.0, 0.0]
    out = policy.mlp_forward(th, rng.standard_normal((7, 16)), (16, 32, 4), (1, 0))
    assert (out == np.array([0.5, -1.0, 2.0, 0.0])).all()
    np.testing.assert_allclose(tasks.classify_fitness(np.zeros((1, 7, 4)), np.arange(7) % 4), -np.log(4.0))
