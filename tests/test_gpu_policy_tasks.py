"""GPU parity: population-batched forward passes, fused single-step tasks, the sphere and
the cart-pole roll-out, each against oracle/ on the same seeded inputs."""
import numpy as np
import pytest

from oracle import policy as opolicy, tasks as otasks, pgpe as opgpe
from workloads import generators as gen, mlp_param_count, convnet_param_count, CONFIGS
from tests.util import assert_close, assert_scalar_rel, dev, host

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def evo():
    import paper_2202_05008_amd as e
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return e


def _work(evo, td, pd, pop):
    n = evo.rollout_workspace_bytes(td, pd, pop)
    return torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")


def _classify(evo, pd, params_d, obs_d, labels_d, pop, B):
    td = evo.make_task_desc(evo.EVO_TASK_CLASSIFY, B=B, obs=obs_d, target=labels_d)
    work = _work(evo, td, pd, pop)
    td = evo.make_task_desc(evo.EVO_TASK_CLASSIFY, B=B, obs=obs_d, target=labels_d, work=work)
    fit = torch.empty(pop, dtype=torch.float32, device="cuda")
    evo.rollout(td, pd, params_d, pop, 1, fit)
    return host(fit)


# ---------------------------------------------------------------- fp32 MLP
@pytest.mark.parametrize("dims,acts,pop,B,shared", [
    ((16, 32, 4), (1, 0), 64, 512, True), ((16, 32, 4), (1, 0), 5, 70, False), ((7, 13, 3), (2, 1), 3, 1, True),
    ((5, 64, 64, 1), (1, 1, 1), 4, 130, False), ((64, 256, 256, 16), (2, 2, 0), 2, 64, False),
    ((3, 5), (0,), 2, 65, True)])
def test_pop_forward_mlp_f32(evo, dims, acts, pop, B, shared):
    P = mlp_param_count(dims)
    params = gen.random_params(11, pop, P, 0.4)
    r = np.random.default_rng(12)
    obs = r.standard_normal((B, dims[0]) if shared else (pop, B, dims[0])).astype(np.float32)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    out = torch.full((pop, B, dims[-1]), np.nan, dtype=torch.float32, device="cuda")
    evo.pop_forward(pd, dev(params), dev(obs), 0 if shared else B * dims[0], out, pop, B)
    ref = opolicy.mlp_forward(params, obs, dims, acts)
    assert_close(host(out), ref, 1e-5, "mlp forward")


# Networks with a fan-in of 64 or more run their layers on the matrix cores (two-term fp16 splits of the fp32
# operands, scales set at run time): fp32 accuracy over ragged widths, batches and value ranges.
@pytest.mark.parametrize("dims,acts,pop,B,shared,scale", [
    ((64, 256, 256, 16), (2, 2, 0), 3, 200, False, 0.1), ((64, 256, 256, 16), (1, 1, 1), 2, 64, True, 0.4),
    ((70, 100, 3), (2, 0), 3, 65, False, 0.3), ((64, 48, 5), (0, 0), 2, 1, True, 0.5),
    ((200, 256, 256, 7), (1, 2, 0), 2, 130, False, 0.2), ((256, 17), (1,), 4, 33, True, 0.3),
    ((64, 256, 256, 16), (2, 2, 0), 2, 70, False, 1e-3), ((64, 256, 256, 16), (2, 0, 0), 2, 70, False, 30.0),
    ((64, 96, 16), (2, 0), 11, 130, False, 0.3)])   # members beyond one group of eight, three tiles each
def test_pop_forward_mlp_f32_matrix_cores(evo, dims, acts, pop, B, shared, scale):
    P = mlp_param_count(dims)
    params = gen.random_params(16, pop, P, scale)
    r = np.random.default_rng(17)
    obs = r.standard_normal((B, dims[0]) if shared else (pop, B, dims[0])).astype(np.float32)
    if not shared and 1 not in acts:
        # one sample far larger than the others, one far smaller: scales are per sample.  (Not in front of a tanh:
        # pre-activations of +-1e4 that cancel to order one are off by more than 1e-5 in any fp32 evaluation.)
        obs[0, 0] *= 1.0e4
        obs[-1, -1] *= 1.0e-4
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    out = torch.full((pop, B, dims[-1]), np.nan, dtype=torch.float32, device="cuda")
    evo.pop_forward(pd, dev(params), dev(obs), 0 if shared else B * dims[0], out, pop, B)
    ref = opolicy.mlp_forward(params, obs, dims, acts)
    got = host(out)
    for m in range(pop):
        for b in range(B):           # every sample on its own scale
            assert_close(got[m, b], ref[m, b], 1e-5, "member %d sample %d" % (m, b))


def test_rollout_losses_mlp_f32_matrix_cores(evo):
    dims, acts, pop, B = (64, 128, 10), (2, 0), 5, 150
    P = mlp_param_count(dims)
    params = gen.random_params(18, pop, P, 0.2)
    x, y = gen.class_blobs(19, B, dims[0], dims[-1])
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    fit = _classify(evo, pd, dev(params), dev(x), dev(y), pop, B)
    ref = otasks.classify_fitness(opolicy.mlp_forward(params, x, dims, acts), y)
    assert_scalar_rel(fit, ref, 1e-5, "classification fitness")
    obs, tgt = gen.teacher_regression(20, pop, B, dims)
    od, tdv = dev(obs), dev(tgt)
    td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=B, obs=od, obs_member_stride=B * dims[0], target=tdv)
    work = _work(evo, td, pd, pop)
    td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=B, obs=od, obs_member_stride=B * dims[0], target=tdv, work=work)
    fit = torch.empty(pop, dtype=torch.float32, device="cuda")
    evo.rollout(td, pd, dev(params), pop, 1, fit)
    ref = otasks.regress_fitness(opolicy.mlp_forward(params, obs, dims, acts), tgt)
    assert_scalar_rel(host(fit), ref, 1e-5, "regression fitness")


def test_rollout_classify_mlp_cfg1(evo):
    c = CONFIGS["cfg1"]
    x, y = gen.class_blobs(c.data_seed, c.B, c.dims[0], c.dims[-1])
    params = gen.random_params(13, c.pop, c.P, 0.3)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, c.dims, c.acts)
    fit = _classify(evo, pd, dev(params), dev(x), dev(y), c.pop, c.B)
    ref = otasks.classify_fitness(opolicy.mlp_forward(params, x, c.dims, c.acts), y)
    assert_scalar_rel(fit, ref, 1e-5, "cfg1 fitness")
    # ragged batch, zero weights: CE = ln(classes) exactly up to rounding
    fit0 = _classify(evo, pd, dev(np.zeros((4, c.P), np.float32)), dev(x[:77]), dev(y[:77]), 4, 77)
    assert_scalar_rel(fit0, np.full(4, -np.log(4.0)), 1e-6, "ln 4")


def test_rollout_regress_mlp_f32(evo):
    dims, acts, pop, B = (6, 20, 3), (2, 0), 7, 90
    P = mlp_param_count(dims)
    params = gen.random_params(14, pop, P, 0.5)
    obs, tgt = gen.teacher_regression(15, pop, B, dims)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    od, tdv = dev(obs), dev(tgt)
    td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=B, obs=od, obs_member_stride=B * dims[0], target=tdv)
    work = _work(evo, td, pd, pop)
    td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=B, obs=od, obs_member_stride=B * dims[0], target=tdv, work=work)
    fit = torch.empty(pop, dtype=torch.float32, device="cuda")
    evo.rollout(td, pd, dev(params), pop, 1, fit)
    ref = otasks.regress_fitness(opolicy.mlp_forward(params, obs, dims, acts), tgt)
    assert_scalar_rel(host(fit), ref, 1e-5, "regress fitness")


# ---------------------------------------------------------------- ConvNet
@pytest.mark.parametrize("H,n_cls,pop,B", [(28, 10, 3, 37), (28, 10, 2, 1), (12, 4, 5, 9), (28, 16, 2, 8),
                                           # image sizes around the tiling of conv1 (8 window columns per matrix tile)
                                           (4, 3, 2, 5), (8, 10, 2, 14), (16, 10, 3, 13), (20, 7, 2, 25), (24, 10, 2, 12)])
def test_convnet_forward_and_fitness(evo, H, n_cls, pop, B):
    P = convnet_param_count(8, 16, n_cls, H)
    params = gen.random_params(16, pop, P, 0.25)
    img, y = gen.mnist_shaped_batch(17, 1, B, n_cls, H)
    pd = evo.make_policy_desc(evo.EVO_POLICY_CONVNET, (H, 8, 16, n_cls))
    assert evo.policy_param_count(pd) == P
    out = torch.full((pop, B, n_cls), np.nan, dtype=torch.float32, device="cuda")
    pdv, imd = dev(params), dev(img)
    evo.pop_forward(pd, pdv, imd, 0, out, pop, B)
    ref = opolicy.convnet_forward(params, img, 8, 16, n_cls)
    assert_close(host(out), ref, 1e-5, "convnet logits")
    fit = _classify(evo, pd, pdv, imd, dev(y), pop, B)
    assert_scalar_rel(fit, otasks.classify_fitness(ref, y), 1e-5, "convnet fitness")


def test_convnet_many_chunks_and_zero_weights(evo):
    H, n_cls, pop, B = 28, 10, 4, 203          # several images per wave, ragged last chunk
    P = convnet_param_count(8, 16, n_cls, H)
    params = gen.random_params(18, pop, P, 0.2)
    params[3] = 0.0
    img, y = gen.mnist_shaped_batch(19, 2, B, n_cls, H)
    pd = evo.make_policy_desc(evo.EVO_POLICY_CONVNET, (H, 8, 16, n_cls))
    fit = _classify(evo, pd, dev(params), dev(img), dev(y), pop, B)
    ref = otasks.classify_fitness(opolicy.convnet_forward(params, img), y)
    assert_scalar_rel(fit, ref, 1e-5, "convnet fitness")
    assert abs(fit[3] + np.log(10.0)) < 1e-5 * np.log(10.0)


@pytest.mark.parametrize("scale", [1e-3, 0.02, 3.0])
def test_convnet_keeps_fp32_accuracy_over_value_ranges(evo, scale):
    """conv2 runs on the fp16 matrix instruction with every operand split into two scaled fp16
    terms: the result must stay fp32-accurate for small and for large weights alike."""
    H, n_cls, pop, B = 28, 10, 3, 21
    P = convnet_param_count(8, 16, n_cls, H)
    params = gen.random_params(31, pop, P, scale)
    img, _ = gen.mnist_shaped_batch(32, 1, B, n_cls, H)
    pd = evo.make_policy_desc(evo.EVO_POLICY_CONVNET, (H, 8, 16, n_cls))
    out = torch.empty(pop, B, n_cls, dtype=torch.float32, device="cuda")
    evo.pop_forward(pd, dev(params), dev(img), 0, out, pop, B)
    assert_close(host(out), opolicy.convnet_forward(params, img, 8, 16, n_cls), 1e-5, "convnet logits, scale %g" % scale)


def test_convnet_any_finite_magnitude(evo):
    """The operands of the fp16 matrix products carry run-time powers of two, so nothing finite is out of
    range: a conv2 weight of 1e5, images whose conv1 activations reach 1e4 and beyond, tiny weights next to
    ordinary biases all give the oracle's logits; a non-finite weight gives that member NaN logits."""
    H, n_cls, pop, B = 28, 10, 5, 6
    P = convnet_param_count(8, 16, n_cls, H)
    params = gen.random_params(33, pop, P, 0.2)
    params[1, 88 + 7] = 1.0e5                      # one weight of W2 (W1 and b1 take 80 + 8 entries)
    params[2, :80] *= 300.0                        # conv1 weights: activations far beyond 4094 on bright images
    params[3, 88:88 + 1152] *= 1.0e-6              # all of W2 tiny, its biases ordinary
    params[4, 88 + 100] = np.nan
    img, y = gen.mnist_shaped_batch(34, 1, B, n_cls, H)
    img[1] *= 400.0                                # a bright image
    img[2] *= 1.0e-4                               # and a dark one
    pd = evo.make_policy_desc(evo.EVO_POLICY_CONVNET, (H, 8, 16, n_cls))
    out = torch.empty(pop, B, n_cls, dtype=torch.float32, device="cuda")
    evo.pop_forward(pd, dev(params), dev(img), 0, out, pop, B)
    got = host(out)
    ref = opolicy.convnet_forward(params[:4], img, 8, 16, n_cls)
    assert np.abs(ref[2, 1]).max() > 1e4
    for m in range(4):
        for b in range(B):           # every (member, image) on its own scale
            assert_close(got[m, b], ref[m, b], 1e-5, "member %d image %d" % (m, b))
    assert np.isnan(got[4]).all()
    fit = _classify(evo, pd, dev(params), dev(img), dev(y), pop, B)
    assert_scalar_rel(fit[:4], otasks.classify_fitness(ref, y), 1e-5, "fitness")
    assert np.isnan(fit[4])


def test_convnet_conv1_operand_ranges(evo):
    """conv1 runs on the fp16 matrix instruction with a scale per output channel and per image: one tap far above
    its channel's other taps, a channel ruled by its bias, channels of very different size, a black image, an image
    with a single bright pixel and one with pixels of both signs all give the oracle's logits."""
    H, n_cls, pop, B = 28, 10, 5, 7
    P = convnet_param_count(8, 16, n_cls, H)
    params = gen.random_params(35, pop, P, 0.2)
    params[1, 4 * 8 + 3] = 2.0e3                   # W1[tap 4][channel 3]: the centre tap 10^4 times its neighbours
    params[2, 72 + 5] = 1.0e6                      # b1[5]: that channel is its bias
    params[3, 0:72:8] *= 1.0e-5                    # channel 0 of conv1 tiny, the others ordinary
    params[3, 1:72:8] *= 1.0e3                     # and channel 1 large
    params[4, :72] = 0.0                           # conv1 weights all zero: activations = relu(bias)
    img, y = gen.mnist_shaped_batch(36, 1, B, n_cls, H)
    img[1] = 0.0
    img[2] = 0.0
    img[2, 0, 13, 17] = 250.0
    img[3] = img[3] - 0.5                          # pixels of both signs
    img[4] *= 1.0e-6
    pd = evo.make_policy_desc(evo.EVO_POLICY_CONVNET, (H, 8, 16, n_cls))
    out = torch.empty(pop, B, n_cls, dtype=torch.float32, device="cuda")
    evo.pop_forward(pd, dev(params), dev(img), 0, out, pop, B)
    got = host(out)
    ref = opolicy.convnet_forward(params, img, 8, 16, n_cls)
    for m in range(pop):
        for b in range(B):           # every (member, image) on its own scale
            assert_close(got[m, b], ref[m, b], 1e-5, "member %d image %d" % (m, b))


# ---------------------------------------------------------------- bf16 MLP on the matrix cores
@pytest.mark.parametrize("dims,acts,pop,B", [((64, 256, 256, 16), (2, 2, 0), 6, 64), ((64, 256, 256, 16), (2, 2, 0), 3, 40),
                                             ((64, 256, 256, 16), (2, 2, 0), 3, 520), ((64, 256, 256, 16), (1, 2, 0), 2, 448),
                                             ((64, 256, 256, 16), (2, 2, 0), 3, 128),       # two tiles of 64 rows
                                             ((64, 256, 256, 16), (2, 2, 0), 2, 200),       # ragged last tile
                                             ((64, 256, 256, 16), (2, 2, 0), 2, 65),        # one row into the second tile
                                             ((64, 256, 256, 16), (2, 1, 1), 2, 1000),      # many tiles, tanh epilogues
                                             ((32, 48, 16), (1, 0), 4, 17), ((16, 16), (0,), 2, 64)])
def test_mlp_bf16(evo, dims, acts, pop, B):
    P = mlp_param_count(dims)
    params = opgpe.round_to_bf16(gen.random_params(20, pop, P, 0.08))     # bf16-representable weights
    obs, tgt = gen.teacher_regression(21, pop, B, dims)
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts, evo.EVO_BF16)
    p_d = dev(params).to(torch.bfloat16)
    assert np.array_equal(p_d.to(torch.float32).cpu().numpy(), params)
    od, tg = dev(obs), dev(tgt)
    out = torch.full((pop, B, dims[-1]), np.nan, dtype=torch.float32, device="cuda")
    evo.pop_forward(pd, p_d, od, B * dims[0], out, pop, B)
    ref = opolicy.mlp_forward(params, obs, dims, acts)      # fp64 with the same bf16 weight values
    got = host(out)
    assert np.isfinite(got).all()
    for m in range(pop):
        assert np.abs(got[m] - ref[m]).max() <= 2e-2 * np.abs(ref[m]).max(), "member %d" % m
    td = evo.make_task_desc(evo.EVO_TASK_REGRESS, B=B, obs=od, obs_member_stride=B * dims[0], target=tg)
    fit = torch.empty(pop, dtype=torch.float32, device="cuda")
    evo.rollout(td, pd, p_d, pop, 1, fit)
    assert_scalar_rel(host(fit), otasks.regress_fitness(ref, tgt), 2e-2, "bf16 fitness")


# ---------------------------------------------------------------- sphere
@pytest.mark.parametrize("P,pop", [(1000, 8), (4099, 3), (1 << 16, 4)])
def test_sphere(evo, P, pop):
    params = gen.random_params(22, pop, P, 1.0)
    xs = gen.sphere_target(23, P)
    xd = dev(xs)
    td = evo.make_task_desc(evo.EVO_TASK_SPHERE, P=P, target=xd)
    work = _work(evo, td, None, pop)
    td = evo.make_task_desc(evo.EVO_TASK_SPHERE, P=P, target=xd, work=work)
    fit = torch.empty(pop, dtype=torch.float32, device="cuda")
    evo.rollout(td, None, dev(params), pop, 1, fit)
    assert_scalar_rel(host(fit), otasks.sphere_fitness(params, xs), 1e-5, "sphere")


# ---------------------------------------------------------------- cart-pole
CP = CONFIGS["cfg3"].cartpole


def test_cartpole_single_step(evo):
    n = 5000
    s, a = gen.random_states(24, n)
    td = evo.make_task_desc(evo.EVO_TASK_CARTPOLE, cp=CP)
    nxt = torch.empty(n, 4, dtype=torch.float32, device="cuda")
    rew = torch.empty(n, dtype=torch.float32, device="cuda")
    evo.evo_task_step(td, dev(s), dev(a), nxt, rew, n)
    ref_n, ref_r = otasks.cartpole_step(s, a, CP)
    assert_close(host(nxt), ref_n, 1e-5, "next state")
    assert_close(host(rew), ref_r, 1e-5, "reward")


def _cartpole(evo, dims, acts, params, R, steps, seed, t, cp=CP, init_scale=0.2):
    pop = params.shape[0]
    pd = evo.make_policy_desc(evo.EVO_POLICY_MLP, dims, acts)
    td = evo.make_task_desc(evo.EVO_TASK_CARTPOLE, n_rollouts=R, reset_seed=seed, generation=t, cp=cp,
                            init_scale=init_scale)
    fit = torch.empty(pop, dtype=torch.float32, device="cuda")
    ret = torch.empty(pop, R, dtype=torch.float32, device="cuda")
    fin = torch.empty(pop, R, 4, dtype=torch.float32, device="cuda")
    p_d = dev(params)
    evo.rollout(td, pd, p_d, pop, steps, fit)
    evo.evo_rollout_details(td, pd, p_d, pop, steps, ret, fin)
    return host(fit), host(ret), host(fin)


@pytest.mark.parametrize("dims,acts,pop,R,steps", [((5, 64, 64, 1), (1, 1, 1), 6, 16, 32), ((5, 64, 64, 1), (1, 1, 1), 3, 20, 8),
                                                   ((5, 32, 32, 1), (1, 2, 1), 4, 5, 24), ((5, 16, 1), (1, 0), 3, 16, 16),
                                                   ((5, 64, 64, 1), (1, 1, 1), 2, 1, 1)])
def test_cartpole_short_horizon(evo, dims, acts, pop, R, steps):
    P = mlp_param_count(dims)
    params = gen.random_params(25, pop, P, 0.5)
    fit, ret, fin = _cartpole(evo, dims, acts, params, R, steps, 777, 3)
    rfit, rret, rfin, _ = otasks.cartpole_rollout(params, dims, acts, 777, 3, R, steps, CP, return_details=True)
    assert_close(fin, rfin, 1e-5, "final states")
    assert_close(ret, rret, 1e-5, "returns")
    assert_scalar_rel(fit, rfit, 1e-5, "fitness")
    if steps == 1:      # after one step the state is the reset state advanced once: same for all members in x, theta
        assert np.allclose(fin[0, :, 0], fin[1, :, 0]) and np.allclose(fin[0, :, 2], fin[1, :, 2])


@pytest.mark.parametrize("init_scale", [0.02, 0.6])
def test_cartpole_narrow_and_wide_reset(evo, init_scale):
    """The spread of the initial states is the task's difficulty knob (Section 3: an easy and a hard
    version of the swing-up): a narrow and a wide reset against the oracle, and the narrow one really
    starts every roll-out next to the hanging-down state."""
    dims, acts, pop, R, steps = (5, 64, 64, 1), (1, 1, 1), 4, 16, 24
    params = gen.random_params(29, pop, mlp_param_count(dims), 0.5)
    fit, ret, fin = _cartpole(evo, dims, acts, params, R, steps, 99, 2, init_scale=init_scale)
    rfit, rret, rfin, _ = otasks.cartpole_rollout(params, dims, acts, 99, 2, R, steps, CP, init_scale=init_scale,
                                                  return_details=True)
    assert_close(fin, rfin, 1e-5, "final states")
    assert_close(ret, rret, 1e-5, "returns")
    assert_scalar_rel(fit, rfit, 1e-5, "fitness")
    _, _, fin0 = _cartpole(evo, dims, acts, params, R, 1, 99, 2, init_scale=init_scale)
    spread = np.abs(fin0[0, :, 2] - np.pi).max()      # one step after the reset
    assert spread < 5.0 * init_scale and (init_scale > 0.1 or spread < 0.15)


def test_cartpole_layer2_range(evo):
    """Layer 2 runs on the fp16 matrix instruction with two-term operands whose scales are set at run time:
    tiny weights keep fp32 accuracy, and so does a member with a layer-2 weight of 1e5 or with ReLU
    activations in the thousands.  (Weights of order one and more over whole episodes: the step-by-step
    gate of test_gpu_cartpole_trace.py.)"""
    dims, R = (5, 64, 64, 1), 16
    P = mlp_param_count(dims)
    params = gen.random_params(41, 3, P, 1e-3)
    fit, ret, fin = _cartpole(evo, dims, (1, 1, 1), params, R, 12, 5, 1)
    rfit, rret, rfin, _ = otasks.cartpole_rollout(params, dims, (1, 1, 1), 5, 1, R, 12, CP, return_details=True)
    assert_close(fin, rfin, 1e-5, "final states, tiny weights")
    assert_scalar_rel(fit, rfit, 1e-5, "fitness, tiny weights")
    for acts in ((1, 1, 1), (2, 1, 1), (0, 2, 1)):     # one step from the reset: nothing for chaos to amplify
        params = gen.random_params(42, 3, P, 0.5)
        params[1, 5 * 64 + 64 + 70] = -1.0e5         # one weight of the second layer
        params[2, :5 * 64] *= 2000.0                 # layer 1: pre-activations in the thousands
        fit, ret, fin = _cartpole(evo, dims, acts, params, R, 1, 5, 1)
        rfit, rret, rfin, _ = otasks.cartpole_rollout(params, dims, acts, 5, 1, R, 1, CP, return_details=True)
        assert_close(fin, rfin, 1e-5, "final states, acts %s" % (acts,))
        assert_scalar_rel(fit, rfit, 1e-5, "fitness, acts %s" % (acts,))


def test_cartpole_termination_and_zero_policy(evo):
    dims, acts = (5, 16, 16, 1), (1, 1, 1)
    P = mlp_param_count(dims)
    params = gen.random_params(26, 4, P, 0.5)
    params[3] = 0.0
    tight = CP[:6] + (0.02, 0.3)       # narrow track: some episodes end early, a short horizon keeps chaos small
    fit, ret, fin = _cartpole(evo, dims, acts, params, 16, 20, 31, 1, tight)
    rfit, rret, rfin, alive = otasks.cartpole_rollout(params, dims, acts, 31, 1, 16, 20, tight, return_details=True)
    assert (~alive).any() and alive.any()
    assert_close(ret, rret, 1e-5, "returns with termination")
    assert_close(fin, rfin, 1e-5, "frozen final states")
    assert_scalar_rel(fit, rfit, 1e-5, "fitness")


def test_cartpole_full_horizon_statistics(evo):
    """1000 chaotic steps in fp32 cannot match an fp64 run trajectory by trajectory; the
    population statistics and the ranking of members must still agree."""
    c = CONFIGS["cfg3"]
    pop = 48
    params = gen.random_params(27, pop, c.P, 0.3)
    fit, ret, _ = _cartpole(evo, c.dims, c.acts, params, c.n_rollouts, c.steps, 5, 1)
    rfit = otasks.cartpole_rollout(params, c.dims, c.acts, 5, 1, c.n_rollouts, c.steps, CP)
    assert np.isfinite(fit).all() and (np.abs(ret) <= c.steps).all()
    assert abs(fit.mean() - rfit.mean()) < 0.05 * rfit.std() + 1.0
    from scipy import stats
    assert stats.spearmanr(fit, rfit).correlation > 0.9
