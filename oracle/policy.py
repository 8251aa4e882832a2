"""CPU ORACLE (test infrastructure, not part of the product path) -- the "global policy".

One network definition is evaluated for every population member with that member's own
flat parameter vector; observations and parameters are both data (Section 2, "Global
Policy"; Section 4, "Exploring Novel Policy Architectures": calling get_actions amounts to
passing a batch through the model).  The paper gives no architecture details; the flat
layouts below are this build's reading.

MLP, per layer l in order:   W_l[in][out] (out contiguous), then b_l[out];
                             h_{l+1} = act_l(h_l W_l + b_l),  act in {none, tanh, relu}.
ConvNet (the "ConvNet with ~10K parameters" of Section 3's MNIST example, shapes from the
workload description): conv3x3 (zero-padded SAME, stride 1) -> ReLU -> maxpool 2x2/2,
twice, then a dense layer.  Flat layout:
   W1[3][3][1][c1], b1[c1], W2[3][3][c1][c2], b2[c2], Wd[(H/4)(W/4)c2][n_cls], bd[n_cls];
   the dense input is flattened in (h, w, c) order with c fastest.  Images are [B,1,H,W].

fp64 arithmetic throughout.  Pins: tests/test_oracle_policy.py (explicit nested-loop
definition, scipy.signal.correlate2d, zero-weight closed forms).
"""
import numpy as np

ACT_NONE, ACT_TANH, ACT_RELU = 0, 1, 2


def _act(h, code):
    if code == ACT_TANH:
        return np.tanh(h)
    if code == ACT_RELU:
        return np.maximum(h, 0.0)
    if code == ACT_NONE:
        return h
    raise ValueError("unknown activation code %r" % (code,))


def mlp_unpack(theta, dims):
    """[(W[in,out], b[out]), ...] views of one flat parameter vector."""
    out, o = [], 0
    for i in range(len(dims) - 1):
        n_in, n_out = dims[i], dims[i + 1]
        W = theta[o:o + n_in * n_out].reshape(n_in, n_out)
        o += n_in * n_out
        b = theta[o:o + n_out]
        o += n_out
        out.append((W, b))
    if o != theta.shape[0]:
        raise ValueError("parameter vector has %d entries, layout needs %d" % (theta.shape[0], o))
    return out


def mlp_forward(params, obs, dims, acts):
    """params[pop,P]; obs[B,D] (shared by all members) or obs[pop,B,D]; returns fp64 out[pop,B,A]."""
    params = np.asarray(params, dtype=np.float64)
    obs = np.asarray(obs, dtype=np.float64)
    pop = params.shape[0]
    out = np.empty((pop, obs.shape[-2], dims[-1]))
    for m in range(pop):
        h = obs if obs.ndim == 2 else obs[m]
        for (W, b), a in zip(mlp_unpack(params[m], dims), acts):
            h = _act(h @ W + b, a)
        out[m] = h
    return out


def convnet_unpack(theta, c1, c2, n_cls, hw):
    feat = (hw // 4) * (hw // 4) * c2
    sizes = [9 * c1, c1, 9 * c1 * c2, c2, feat * n_cls, n_cls]
    if sum(sizes) != theta.shape[0]:
        raise ValueError("parameter vector has %d entries, layout needs %d" % (theta.shape[0], sum(sizes)))
    parts, o = [], 0
    for s in sizes:
        parts.append(theta[o:o + s])
        o += s
    W1 = parts[0].reshape(3, 3, 1, c1)
    W2 = parts[2].reshape(3, 3, c1, c2)
    Wd = parts[4].reshape(feat, n_cls)
    return W1, parts[1], W2, parts[3], Wd, parts[5]


def conv3x3_same(x, W, b):
    """x[B,H,W,Cin] -> [B,H,W,Cout]: out[h,w,o] = b[o] + sum_{dy,dx,c} x[h+dy-1, w+dx-1, c] W[dy,dx,c,o],
    with zeros outside the image."""
    B, H, Wd_, _ = x.shape
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    out = np.zeros((B, H, Wd_, W.shape[3])) + b
    for dy in range(3):
        for dx in range(3):
            out += xp[:, dy:dy + H, dx:dx + Wd_, :] @ W[dy, dx]
    return out


def maxpool2(x):
    B, H, W, C = x.shape
    return x.reshape(B, H // 2, 2, W // 2, 2, C).max(axis=(2, 4))


def convnet_forward(params, images, c1=8, c2=16, n_cls=10):
    """params[pop,P]; images[B,1,H,W] shared by all members; returns fp64 logits[pop,B,n_cls]."""
    params = np.asarray(params, dtype=np.float64)
    img = np.asarray(images, dtype=np.float64)
    B, _, H, _ = img.shape
    x0 = img.transpose(0, 2, 3, 1)                       # NHWC, C = 1
    out = np.empty((params.shape[0], B, n_cls))
    for m in range(params.shape[0]):
        W1, b1, W2, b2, Wd, bd = convnet_unpack(params[m], c1, c2, n_cls, H)
        h = maxpool2(np.maximum(conv3x3_same(x0, W1, b1), 0.0))
        h = maxpool2(np.maximum(conv3x3_same(h, W2, b2), 0.0))
        out[m] = h.reshape(B, -1) @ Wd + bd
    return out
