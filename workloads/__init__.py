"""Seeded synthetic inputs for the IMPACT learner loss and its circular buffer.

This module only draws random tensors of the right shapes and value
distributions.  It contains none of the loss arithmetic: no log-probabilities,
no importance ratios, no returns.  Both the CPU oracle's tests and the GPU
path's tests and benchmark take their inputs from here, so the two sides see
bit-identical fp32 arrays.

The shapes follow the paper's experimental setups (Appendix B tables): Atari-like
categorical policies with up to 18 actions and 50-step worker batches, and
MuJoCo-like diagonal-Gaussian policies with 6 or 17 action dimensions.  The
simulators themselves are not used; the value distributions below stand in for
their logits, rewards and episode ends.

Tensor layout is time-major: ``[T, n, W]`` for distribution parameters
(``W = A`` logits for a categorical policy, ``W = 2*D`` for a Gaussian one, the
D means first and the D log standard deviations after them), ``[T, n]`` for
per-step scalars and ``[n]`` for the bootstrap value.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict

import numpy as np

BASE_SEED = 191200167

CATEGORICAL = "categorical"
GAUSSIAN = "gaussian"


@dataclass(frozen=True)
class LossHyper:
    """Scalars of the loss (Section 3.1, Algorithm 1, Appendix B tables)."""

    gamma: float = 0.99      # discount
    lam: float = 1.0         # GAE lambda inside the V-trace advantage
    rho_bar: float = 1.0     # V-trace truncation of the TD-error weight
    c_bar: float = 1.0       # V-trace truncation of the trace coefficient
    rho_clip: float = 2.0    # target-worker clipping rho of Section 3.1 (inf: ratio pi_theta/pi_target)
    eps: float = 0.2         # PPO clip parameter
    vf_coeff: float = 1.0
    ent_coeff: float = 0.01
    kl_coeff: float = 0.0
    ratio_mode: int = 0      # 0: target-worker clipping (R_3 of Section 4.1; R_1 when rho_clip = inf); 1: pi_theta / pi_worker (R_2)


@dataclass(frozen=True)
class Workload:
    name: str
    dist: str                # CATEGORICAL or GAUSSIAN
    T: int
    B: int
    A: int                   # number of actions, or action dimension D
    num_slots: int
    K: int
    storage: str = "f32"     # dtype of the buffer-resident float fields: "f32" or "bf16"
    hyper: LossHyper = field(default_factory=LossHyper)
    # value distributions
    learner_std: float = 1.0          # std of learner logits / means
    target_mode: str = "independent"  # "independent" | "learner_plus"
    target_noise: float = 0.0
    worker_mode: str = "independent"  # "independent" | "learner_plus" | "target_plus"
    worker_noise: float = 0.0
    logstd_lo: float = -1.5
    logstd_hi: float = 0.0
    logstd_mode: str = "per_policy"   # "per_policy": each policy's log-std drawn on its own | "offsets": like the means
    mean_mode: str = "offsets"        # "offsets": target/worker means a small offset away | "per_policy": drawn on their own
    reward_mode: str = "uniform"      # "uniform" | "sparse_sign" | "normal"
    reward_p_nonzero: float = 0.05
    done_p: float = 0.01
    config_id: int = 0

    @property
    def W(self) -> int:
        return self.A if self.dist == CATEGORICAL else 2 * self.A

    @property
    def steps(self) -> int:
        return self.T * self.B

    def with_batch(self, B: int, num_slots: int | None = None) -> "Workload":
        return replace(self, B=B, num_slots=self.num_slots if num_slots is None else num_slots)


# The five workloads.  Hyper-parameters per config: the tiny case uses eps 0.2;
# the Atari-like ones the discrete table of Appendix B (eps 0.3, entropy 0.01,
# KL 0, gamma 0.99); the MuJoCo-like ones the continuous table (eps 0.4,
# entropy 0, KL 1, gamma 0.995).  rho_clip = 2 in both tables.  The paper never
# gives the V-trace truncation levels; 1.0 is used.  lambda = 1 (plain V-trace).
C1 = Workload("C1-discrete-tiny", CATEGORICAL, T=20, B=32, A=6, num_slots=64, K=2,
              hyper=LossHyper(gamma=0.99, eps=0.2, ent_coeff=0.01, kl_coeff=0.0),
              learner_std=1.0, target_mode="independent", worker_mode="independent",
              reward_mode="uniform", done_p=0.01, config_id=1)
C2 = Workload("C2-discrete-atari", CATEGORICAL, T=50, B=512, A=18, num_slots=4096, K=4,
              hyper=LossHyper(gamma=0.99, eps=0.3, ent_coeff=0.01, kl_coeff=0.0),
              learner_std=2.0, target_mode="learner_plus", target_noise=0.1,
              worker_mode="learner_plus", worker_noise=0.1,
              reward_mode="sparse_sign", reward_p_nonzero=0.05, done_p=0.002, config_id=2)
C3 = Workload("C3-continuous-mujoco", GAUSSIAN, T=64, B=1024, A=6, num_slots=8192, K=2,
              hyper=LossHyper(gamma=0.995, eps=0.4, ent_coeff=0.0, kl_coeff=1.0),
              learner_std=1.0, target_mode="learner_plus", target_noise=0.1,
              worker_mode="learner_plus", worker_noise=0.1,
              logstd_lo=-1.5, logstd_hi=0.0, reward_mode="normal", done_p=0.001, config_id=3)
C4 = Workload("C4-discrete-large", CATEGORICAL, T=100, B=8192, A=18, num_slots=32768, K=8,
              hyper=LossHyper(gamma=0.99, eps=0.3, ent_coeff=0.01, kl_coeff=0.0),
              learner_std=2.0, target_mode="learner_plus", target_noise=0.1,
              worker_mode="target_plus", worker_noise=0.5,
              reward_mode="sparse_sign", reward_p_nonzero=0.05, done_p=0.002, config_id=4)
C5 = Workload("C5-continuous-large-bf16", GAUSSIAN, T=128, B=16384, A=17, num_slots=65536, K=4,
              storage="bf16",
              hyper=LossHyper(gamma=0.995, eps=0.4, ent_coeff=0.0, kl_coeff=1.0),
              learner_std=1.0, target_mode="learner_plus", target_noise=0.2,
              worker_mode="target_plus", worker_noise=0.2,
              logstd_lo=-2.0, logstd_hi=0.5, reward_mode="normal", done_p=0.001, config_id=5)

WORKLOADS: Dict[str, Workload] = {"C1": C1, "C2": C2, "C3": C3, "C4": C4, "C5": C5}


def _rng(wl: Workload, stream: int) -> np.random.Generator:
    # one independent stream per (workload, block of trajectories)
    return np.random.default_rng([BASE_SEED, wl.config_id, int(stream)])


def make_trajectories(wl: Workload, n: int, stream: int = 0) -> Dict[str, np.ndarray]:
    """Draw ``n`` synthetic trajectories of ``wl.T`` steps.

    Draw order: learner parameters, target noise, worker noise, values,
    bootstrap, rewards, dones, actions.  Returns fp32 arrays (int32 actions for
    a categorical policy, uint8 dones), C-contiguous, time-major.
    """
    T, A, W = wl.T, wl.A, wl.W
    g = _rng(wl, stream)
    f32 = np.float32

    def normal(shape, std):
        return (g.standard_normal(shape, dtype=np.float32) * f32(std)).astype(f32)

    def derive(mode, noise, learner_part, target_part):
        if mode == "independent":
            return normal(learner_part.shape, wl.learner_std)
        base = learner_part if mode == "learner_plus" else target_part
        return (base + normal(base.shape, noise)).astype(f32)

    if wl.dist == CATEGORICAL:
        learner = normal((T, n, A), wl.learner_std)
        target = derive(wl.target_mode, wl.target_noise, learner, None)
        worker = derive(wl.worker_mode, wl.worker_noise, learner, target)
    else:
        # Means: the learner's are drawn fresh, the target's and the worker's lie the stated small offsets
        # away (a target network is a lagged copy of the learner, a worker a lagged copy of either), or, with
        # mean_mode "per_policy", are drawn on their own.  Log standard deviations: uniform in the stated
        # range for each policy and element on its own ("per_policy"), or offsets like the means.
        l_mean = normal((T, n, A), wl.learner_std)
        l_lstd = g.uniform(wl.logstd_lo, wl.logstd_hi, (T, n, A)).astype(f32)
        own_means = wl.mean_mode == "per_policy"
        t_mean = derive("independent" if own_means else wl.target_mode, wl.target_noise, l_mean, None)
        w_mean = derive("independent" if own_means else wl.worker_mode, wl.worker_noise, l_mean, t_mean)

        def derive_lstd(mode, noise, target_part):
            if mode == "independent" or wl.logstd_mode == "per_policy":
                return g.uniform(wl.logstd_lo, wl.logstd_hi, (T, n, A)).astype(f32)
            base = l_lstd if mode == "learner_plus" else target_part
            return (base + normal(base.shape, noise)).astype(f32)

        t_lstd = derive_lstd(wl.target_mode, wl.target_noise, None)
        w_lstd = derive_lstd(wl.worker_mode, wl.worker_noise, t_lstd)
        learner = np.concatenate([l_mean, l_lstd], axis=2)
        target = np.concatenate([t_mean, t_lstd], axis=2)
        worker = np.concatenate([w_mean, w_lstd], axis=2)

    values = normal((T, n), 1.0)
    bootstrap = normal((n,), 1.0)

    if wl.reward_mode == "uniform":
        rewards = g.uniform(-1.0, 1.0, (T, n)).astype(f32)
    elif wl.reward_mode == "sparse_sign":
        nonzero = g.random((T, n)) < wl.reward_p_nonzero
        sign = np.where(g.random((T, n)) < 0.5, -1.0, 1.0)
        rewards = np.where(nonzero, sign, 0.0).astype(f32)
    else:
        rewards = normal((T, n), 1.0)

    dones = (g.random((T, n)) < wl.done_p).astype(np.uint8)

    if wl.dist == CATEGORICAL:
        # a ~ worker policy: arg-max of logits plus Gumbel noise draws from the
        # categorical distribution those logits define.
        gumbel = g.gumbel(size=(T, n, A))
        actions = np.argmax(worker.astype(np.float64) + gumbel, axis=2).astype(np.int32)
    else:
        noise = g.standard_normal((T, n, A))
        sigma_w = np.exp(worker[:, :, A:].astype(np.float64))
        actions = (worker[:, :, :A].astype(np.float64) + sigma_w * noise).astype(f32)

    out = dict(learner=learner, target=target, worker=worker, actions=actions,
               rewards=rewards, dones=dones, values=values, bootstrap=bootstrap)
    return {k: np.ascontiguousarray(v) for k, v in out.items()}


def make_batch(wl: Workload, stream: int = 0) -> Dict[str, np.ndarray]:
    """One time-major batch of ``wl.B`` trajectories."""
    return make_trajectories(wl, wl.B, stream)


def take_trajectories(trj: Dict[str, np.ndarray], index) -> Dict[str, np.ndarray]:
    """Select trajectories (axis 1; axis 0 for the bootstrap) — plain indexing."""
    out = {}
    for k, v in trj.items():
        out[k] = np.ascontiguousarray(v[index] if v.ndim == 1 else v[:, index])
    return out
