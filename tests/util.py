"""Shared helpers of the parity tests: tolerances and host<->device marshalling."""
import numpy as np


def rel_err_ok(got, ref, tol=1e-5):
    """|got - ref| <= tol * max(|ref|, rms(ref)) element-wise (vectors); returns (ok, worst ratio)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    scale = np.maximum(np.abs(ref), rms)
    scale = np.where(scale == 0.0, 1.0, scale)
    ratio = np.abs(got - ref) / scale
    worst = float(ratio.max()) if ratio.size else 0.0
    return worst <= tol, worst


def assert_close(got, ref, tol=1e-5, what=""):
    assert np.asarray(got).shape == np.asarray(ref).shape, "%s: shape %s vs %s" % (what, np.shape(got), np.shape(ref))
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), "%s: non-finite values" % what
    ok, worst = rel_err_ok(got, ref, tol)
    assert ok, "%s: worst error %.3g x scale exceeds %.1g" % (what, worst, tol)


def assert_scalar_rel(got, ref, tol=1e-5, what=""):
    """Plain relative error for scalars such as fitness values."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    denom = np.where(ref == 0.0, 1.0, np.abs(ref))
    worst = float((np.abs(got - ref) / denom).max())
    assert worst <= tol, "%s: worst relative error %.3g exceeds %.1g" % (what, worst, tol)


def adam_ill_conditioned(g, eps=1e-8):
    """Elements of an ORACLE gradient g on which Adam's early, sign-like steps are ill-conditioned.

    The gradient itself is gated at 1e-5 rms(g) (absolute).  Through the first Adam step
    mu += lr g / (|g| + eps) that allowance moves mu by lr eps / (|g| + eps)^2 * 1e-5 rms(g), which
    exceeds the 1e-5 lr allowed on mu exactly where eps rms(g) > |g| (|g| + eps).  Those elements
    (and anything below 1e-4 rms(g), the fp32 noise floor of the sums) are compared on the gradient
    only.  Later steps are less sensitive, so the first-step set is used for every step."""
    g = np.abs(np.asarray(g, dtype=np.float64))
    rms = float(np.sqrt(np.mean(g * g))) if g.size else 0.0
    return (g < 1e-4 * rms) | (eps * rms > g * (g + eps))


def dev(x, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def host(t):
    return t.detach().cpu().numpy()


def bf16_bits_to_f32(t):
    """torch bfloat16 device tensor -> numpy fp32 values."""
    import torch
    return t.detach().to(torch.float32).cpu().numpy()
