"""Seeded synthetic workloads for the PQL learner hot path.

This module only *draws inputs*: transition rows, initial network parameters and the
hyper-parameter constants of each workload.  It contains none of the method's
arithmetic (no returns, no network evaluation, no optimiser) so that both the HIP path
and the independent CPU checker can be fed from it without sharing any logic.

The paper evaluates on Isaac Gym tasks (Section 4.1, Table B.1).  The simulator is not
part of this code base, so transitions are synthetic: the dimensions, number of parallel
environments, replay size, batch size, n-step length and discount follow the paper's
hyper-parameter table (Table B.1) and the named robot tasks, while values are drawn from
simple distributions (standard normal observations / rewards, uniform actions, Bernoulli
terminations).

Parameter layout (shared convention, part of the C interface): a network is one flat fp32
vector; for each layer in order the weight matrix ``W[in, out]`` row-major (``y = x W + b``)
followed by the bias ``b[out]``.  Twin critics are two such vectors back to back.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np


def _f32(x: float) -> float:
    """Round a Python float to the nearest fp32 value (hyper-parameters cross the C
    interface as ``float``; both consumers must see the same number)."""
    return float(np.float32(x))


@dataclass(frozen=True)
class Workload:
    name: str
    obs_dim: int
    act_dim: int
    num_envs: int          # N parallel environments (Table B.1 default 4096)
    capacity: int          # replay size in transitions (Table B.1 default 5e6)
    batch: int             # batch size (Table B.1 default 8192)
    nstep: int             # n-step target (Table B.1 default 3)
    hidden: Tuple[int, ...]
    done_p: float          # Bernoulli termination probability of the synthetic data
    lr: float = _f32(5e-4)         # Table B.1 learning rates
    gamma: float = _f32(0.99)      # Table B.1 discount factor
    tau: float = _f32(0.05)        # Table B.1 target update rate
    sigma_min: float = _f32(0.05)  # Section 3.3 mixed exploration range
    sigma_max: float = _f32(0.8)
    beta1: float = _f32(0.9)
    beta2: float = _f32(0.999)
    eps: float = _f32(1e-8)
    critic_updates: int = 100
    actor_updates: int = 0
    index: int = 0
    max_grad_norm: float = 0.0     # Table B.1 gradient clipping (0.5 there); 0 = off
    obs_norm: bool = False         # Table B.1 normalized observations
    obs_norm_eps: float = _f32(1e-5)
    obs_loc: float = 0.0           # synthetic observations are obs_loc + obs_scale * N(0, 1)
    obs_scale: float = 1.0
    num_atoms: int = 0             # PQL-D: 51 atoms on (-10, 10); 0 = scalar critics
    v_min: float = -10.0
    v_max: float = 10.0
    sac: bool = False              # PQL + SAC: tanh-Gaussian policy, learnable temperature
    init_alpha: float = _f32(0.2)  # initial entropy coefficient (not given in the paper)

    @property
    def rows(self) -> int:
        """Ring rows T: one row holds one step of all N environments."""
        return self.capacity // self.num_envs

    @property
    def data_seed(self) -> int:
        return 1000 + self.index

    @property
    def param_seed(self) -> int:
        return 2000 + self.index

    @property
    def rng_seed(self) -> int:
        """Seed of the counter-based generator used for index sampling / exploration."""
        return 0x5EED0000 + self.index

    @property
    def target_entropy(self) -> float:
        return -float(self.act_dim)

    def actor_dims(self) -> List[Tuple[int, int]]:
        return layer_dims(self.obs_dim, self.hidden, 2 * self.act_dim if self.sac else self.act_dim)

    def critic_dims(self) -> List[Tuple[int, int]]:
        return layer_dims(self.obs_dim + self.act_dim, self.hidden, self.num_atoms if self.num_atoms >= 2 else 1)

    def replace(self, **kw) -> "Workload":
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


def layer_dims(n_in: int, hidden, n_out: int) -> List[Tuple[int, int]]:
    dims = []
    prev = n_in
    for h in hidden:
        dims.append((prev, int(h)))
        prev = int(h)
    dims.append((prev, n_out))
    return dims


def param_count(dims) -> int:
    return int(sum(i * o + o for i, o in dims))


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 8, 2, 64, 4096, 256, 3, (64, 64), 0.01,
                     lr=_f32(3e-4), critic_updates=1, actor_updates=1, index=0),
    "ant": Workload("ant", 60, 8, 4096, 1_000_000, 8192, 3, (256, 256), 0.01,
                    sigma_min=_f32(0.2), sigma_max=_f32(0.2),
                    critic_updates=100, actor_updates=10, index=1),
    "humanoid": Workload("humanoid", 108, 21, 16384, 2_000_000, 8192, 3, (512, 256, 128), 0.005,
                         critic_updates=100, index=2),
    "shadow": Workload("shadow", 211, 20, 16384, 4_000_000, 16384, 3, (512, 512, 256), 0.002,
                       critic_updates=100, index=3),
    "scale": Workload("scale", 211, 20, 32768, 8_000_000, 32768, 5, (1024, 512, 256), 0.002,
                      critic_updates=100, index=4),
}


def transition_rows(w: Workload, rng: np.random.Generator, rows: int = 1):
    """Draw ``rows`` synthetic actor steps, each one row of N transitions.

    Order of draws per row (fixed, so any consumer regenerates the same data):
    obs ~ N(0,1) [N,o]; act ~ U[-1,1) [N,a]; rew ~ N(0,1) [N]; next_obs ~ N(0,1) [N,o];
    done ~ Bernoulli(done_p) as 0.0/1.0 [N].  All fp32.  With a non-default obs_loc / obs_scale,
    dimension c of both observation fields becomes obs_loc * ((c mod 3) - 1) +
    obs_scale * (1 + c mod 4) * z (unequal units per dimension, as simulator observations have).
    """
    out = []
    N, o, a = w.num_envs, w.obs_dim, w.act_dim
    units = w.obs_loc != 0.0 or w.obs_scale != 1.0
    c = np.arange(o)
    loc = (w.obs_loc * ((c % 3) - 1)).astype(np.float32)
    scale = (w.obs_scale * (1 + c % 4)).astype(np.float32)
    for _ in range(rows):
        obs = rng.standard_normal((N, o), dtype=np.float32)
        act = rng.uniform(-1.0, 1.0, size=(N, a)).astype(np.float32)
        rew = rng.standard_normal((N,), dtype=np.float32)
        nxt = rng.standard_normal((N, o), dtype=np.float32)
        if units:
            obs = loc + scale * obs
            nxt = loc + scale * nxt
        done = (rng.random((N,)) < w.done_p).astype(np.float32)
        out.append(dict(obs=obs, act=act, rew=rew, next_obs=nxt, done=done))
    return out


def data_rng(w: Workload) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(w.data_seed))


def init_params(dims, rng: np.random.Generator) -> np.ndarray:
    """Flat fp32 parameter vector: every W and b ~ U(-1/sqrt(in), 1/sqrt(in))."""
    parts = []
    for n_in, n_out in dims:
        bound = 1.0 / np.sqrt(n_in)
        parts.append(rng.uniform(-bound, bound, size=(n_in * n_out,)).astype(np.float32))
        parts.append(rng.uniform(-bound, bound, size=(n_out,)).astype(np.float32))
    return np.concatenate(parts)


def init_networks(w: Workload):
    """Actor and twin-critic parameters (flat fp32), drawn actor, Q1, Q2 in that order."""
    rng = np.random.Generator(np.random.PCG64(w.param_seed))
    actor = init_params(w.actor_dims(), rng)
    q1 = init_params(w.critic_dims(), rng)
    q2 = init_params(w.critic_dims(), rng)
    return actor, np.concatenate([q1, q2])
