"""The five synthetic workloads (shapes and hyper-parameters only, no arithmetic).

Each stands in for one of the paper's example categories (Section 3, "EvoJAX Examples"):
supervised single-step tasks (cfg1, cfg2, cfg4), a control task with a roll-out loop (cfg3)
and a pure ask/tell stress (cfg5).  cfg2 takes the shape of the MNIST example of
Section 3 / Table 1 (1x28x28 images in [0,1], 10 balanced classes, ConvNet of ~10K
parameters); the data itself is synthetic.
"""
from dataclasses import dataclass, field
from typing import Tuple

# integer codes shared with the C ABI (include/evo.h) by value
ACT_NONE, ACT_TANH, ACT_RELU = 0, 1, 2
POLICY_MLP, POLICY_CONVNET, POLICY_LSTM_SEQ2SEQ = 0, 1, 2
TASK_CLASSIFY, TASK_REGRESS, TASK_CARTPOLE, TASK_SPHERE, TASK_SEQ2SEQ, TASK_FORAGE = 0, 1, 2, 3, 4, 5
TASK_FORAGE_SOLO = 6
DT_F32, DT_BF16 = 0, 1


def mlp_param_count(dims: Tuple[int, ...]) -> int:
    return sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(len(dims) - 1))


def lstm_seq2seq_param_count(V: int = 12, H: int = 128, n_out: int = 10) -> int:
    return 2 * (V * 4 * H + H * 4 * H + 4 * H) + H * n_out + n_out


def world_dict(world: Tuple[float, ...]) -> dict:
    """The shared world's constants by name (the order of WorkloadConfig.world and of task_desc.cp)."""
    dt, thrust, drag, vmax, radius, n_food, n_poison = world
    return dict(dt=dt, thrust=thrust, drag=drag, vmax=vmax, radius=radius, n_food=int(n_food), n_poison=int(n_poison))


def convnet_param_count(c1: int = 8, c2: int = 16, n_cls: int = 10, hw: int = 28) -> int:
    feat = (hw // 4) * (hw // 4) * c2
    return 9 * 1 * c1 + c1 + 9 * c1 * c2 + c2 + feat * n_cls + n_cls


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    pop: int
    policy_kind: int
    dims: Tuple[int, ...]          # MLP: layer widths; ConvNet: (c1, c2, n_classes); LSTM seq2seq: (V, H, n_out)
    acts: Tuple[int, ...]          # activation after each MLP layer
    dtype: int                     # DT_F32 or DT_BF16 (parameter storage)
    task_kind: int
    B: int = 0                     # samples per member (supervised tasks)
    n_rollouts: int = 1
    steps: int = 1
    generations: int = 1
    shared_obs: bool = True
    sigma_init: float = 0.1
    lr_mu: float = 0.01
    lr_sigma: float = 0.1
    sigma_max_change: float = 0.2
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    data_seed: int = 20220509
    # cart-pole constants: g, m_cart, m_pole, length, friction, force_scale, dt, x_limit
    cartpole: Tuple[float, ...] = field(default=(9.82, 0.5, 0.5, 0.6, 0.1, 10.0, 0.01, 2.4))
    init_scale: float = 0.2
    digits: int = 3                # seq2seq: digits per operand ("012+345=" -> "0357")
    # shared world: dt, thrust, drag, vmax, touch radius, food items, poison items
    world: Tuple[float, ...] = field(default=(0.0625, 0.015625, 0.875, 0.25, 0.03125, 24, 24))

    @property
    def P(self) -> int:
        if self.task_kind == TASK_SPHERE:
            return self.dims[0]
        if self.policy_kind == POLICY_CONVNET:
            return convnet_param_count(self.dims[0], self.dims[1], self.dims[2])
        if self.policy_kind == POLICY_LSTM_SEQ2SEQ:
            return lstm_seq2seq_param_count(*self.dims)
        return mlp_param_count(self.dims)

    @property
    def evals_per_generation(self) -> int:
        """member-evals: pop x samples, or env-steps, or pop x P parameter samples."""
        if self.task_kind in (TASK_CARTPOLE, TASK_FORAGE, TASK_FORAGE_SOLO):
            return self.pop * self.n_rollouts * self.steps
        if self.task_kind == TASK_SPHERE:
            return self.pop
        return self.pop * self.B


CONFIGS = {
    "cfg1": WorkloadConfig("cfg1", pop=64, policy_kind=POLICY_MLP, dims=(16, 32, 4),
                           acts=(ACT_TANH, ACT_NONE), dtype=DT_F32, task_kind=TASK_CLASSIFY,
                           B=512, generations=3),
    "cfg2": WorkloadConfig("cfg2", pop=256, policy_kind=POLICY_CONVNET, dims=(8, 16, 10),
                           acts=(), dtype=DT_F32, task_kind=TASK_CLASSIFY, B=1024),
    "cfg3": WorkloadConfig("cfg3", pop=1024, policy_kind=POLICY_MLP, dims=(5, 64, 64, 1),
                           acts=(ACT_TANH, ACT_TANH, ACT_TANH), dtype=DT_F32,
                           task_kind=TASK_CARTPOLE, n_rollouts=16, steps=1000),
    "cfg4": WorkloadConfig("cfg4", pop=4096, policy_kind=POLICY_MLP, dims=(64, 256, 256, 16),
                           acts=(ACT_RELU, ACT_RELU, ACT_NONE), dtype=DT_BF16,
                           task_kind=TASK_REGRESS, B=64, shared_obs=False),
    "cfg5": WorkloadConfig("cfg5", pop=1024, policy_kind=POLICY_MLP, dims=(1 << 20,), acts=(),
                           dtype=DT_F32, task_kind=TASK_SPHERE, generations=10),
    # beyond the five named configurations: the paper's sequence-to-sequence example (Section 3), an
    # LSTM encoder-decoder of 145,674 parameters on strings of three-digit additions
    "seq2seq": WorkloadConfig("seq2seq", pop=1024, policy_kind=POLICY_LSTM_SEQ2SEQ, dims=(12, 128, 10), acts=(),
                              dtype=DT_F32, task_kind=TASK_SEQ2SEQ, B=128, digits=3),
    # the multi-agent scheme of Section 3's WaterWorld paragraph: the whole population lives in each of
    # n_rollouts shared worlds, one agent per member
    "forage": WorkloadConfig("forage", pop=1024, policy_kind=POLICY_MLP, dims=(8, 32, 32, 2),
                             acts=(ACT_TANH, ACT_TANH, ACT_TANH), dtype=DT_F32, task_kind=TASK_FORAGE,
                             n_rollouts=8, steps=500),
    # the single-agent form of the same world: every member alone in its own copy of each world
    "forage_solo": WorkloadConfig("forage_solo", pop=1024, policy_kind=POLICY_MLP, dims=(8, 32, 32, 2),
                                  acts=(ACT_TANH, ACT_TANH, ACT_TANH), dtype=DT_F32, task_kind=TASK_FORAGE_SOLO,
                                  n_rollouts=8, steps=500),
}
