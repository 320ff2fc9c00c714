"""Plain CPU oracle for the Parallel Q-Learning (PQL) learner hot path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
learner path computes, written in NumPy float64 straight from the paper's description of
the method (Section 3, Algorithms 1-3, Table B.1).  Only the test-suite, the smoke check
and the benchmark's CPU-baseline leg may use it; the product never calls it and shares no
code with it.

Every function states the passage it follows.  Where the paper only names a technique
(DDPG, double Q-learning, n-step returns, Adam, mean-squared Bellman error) the textbook
definition of that technique is written out.

Conventions
-----------
* A network is one flat vector: per layer ``W[in, out]`` row-major then ``b[out]``
  (``y = x W + b``).  Hidden layers use ELU (alpha = 1); the critic output is linear and
  scalar, the actor output passes through tanh.  The critic input is ``concat(s, a)``.
* The replay memory is a ring of ``T`` rows; one row is one Actor step of all ``N``
  parallel environments (Section 3.1, "Data Transfer").  Slot = row * N + env.
* Random draws come from the counter-based generator Philox-4x32-10 (Salmon et al.,
  SC'11), implemented here from its published definition.

Parity status: the paper prints no numeric value of any loss, Q-value or parameter, so
agreement with the authors' own implementation is *parity unpinned*; every function below
is pinned by the definitional checks in ``tests/test_oracle_*.py``.
"""
from __future__ import annotations

import numpy as np

MASK32 = 0xFFFFFFFF
MASK64 = 0xFFFFFFFFFFFFFFFF

STREAM_SAMPLE = 1   # index sampling draws
STREAM_ACT = 2      # exploration-noise draws
STREAM_STATE = 3    # the P-learner's draws of states
STREAM_SAC_TARGET = 4   # PQL + SAC: action noise of the V-learner's target sample a' ~ pi^v(.|s')
STREAM_SAC_POLICY = 5   # PQL + SAC: action noise of the P-learner's reparameterised sample


# --------------------------------------------------------------------------------------
# Philox-4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3")
# --------------------------------------------------------------------------------------
_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85


def philox4x32_10(ctr, key):
    """Ten rounds of Philox-4x32 on arrays of counters.

    ``ctr``: four integer arrays (same shape), each value < 2**32.  ``key``: two Python
    ints < 2**32.  Returns four uint64 arrays holding 32-bit outputs.
    """
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & np.uint64(MASK32) for c in ctr)
    k0, k1 = int(key[0]) & MASK32, int(key[1]) & MASK32
    m32 = np.uint64(MASK32)
    s32 = np.uint64(32)
    for _ in range(10):
        p0 = np.uint64(_PHILOX_M0) * c0          # 32x32 -> 64 bit products
        p1 = np.uint64(_PHILOX_M1) * c2
        hi0, lo0 = p0 >> s32, p0 & m32
        hi1, lo1 = p1 >> s32, p1 & m32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _PHILOX_W0) & MASK32
        k1 = (k1 + _PHILOX_W1) & MASK32
    return c0, c1, c2, c3


def rng_words(seed: int, stream: int, call: int, k):
    """Four 32-bit words for element ``k`` of draw ``call`` on ``stream``.

    Counter = (k mod 2^32, stream, call mod 2^32, call >> 32); key = (seed mod 2^32,
    seed >> 32).  ``k`` is an integer array with values < 2**32.
    """
    k = np.asarray(k, dtype=np.uint64)
    one = np.ones_like(k)
    ctr = (k, one * np.uint64(stream & MASK32), one * np.uint64(call & MASK32),
           one * np.uint64((call >> 32) & MASK32))
    return philox4x32_10(ctr, (seed & MASK32, (seed >> 32) & MASK32))


# --------------------------------------------------------------------------------------
# Replay ring (Section 3.1: the V-learner keeps its replay buffer on the GPU; the Actor
# sends N tuples (s_t, a_t, s_{t+1}, r_t, d_{t+1}) per step)
# --------------------------------------------------------------------------------------
class ReplayRing:
    """Circular store of Actor steps.  Contents are kept in the dtype they arrive in
    (fp32): pushing is a copy, so stored values are bit-identical to the inputs."""

    def __init__(self, rows: int, num_envs: int, obs_dim: int, act_dim: int):
        self.T, self.N, self.o, self.a = int(rows), int(num_envs), int(obs_dim), int(act_dim)
        n = self.T * self.N
        self.obs = np.zeros((n, self.o), dtype=np.float32)
        self.act = np.zeros((n, self.a), dtype=np.float32)
        self.rew = np.zeros((n,), dtype=np.float32)
        self.next_obs = np.zeros((n, self.o), dtype=np.float32)
        self.done = np.zeros((n,), dtype=np.float32)
        self.head = 0     # row the next push writes
        self.count = 0    # number of valid rows

    def push(self, obs, act, rew, next_obs, done):
        """Algorithm 1 (the Actor appends one step of N tuples) / Algorithm 3 (the
        V-learner adds received tuples to its buffer); the oldest row is overwritten
        once the ring is full."""
        lo, hi = self.head * self.N, (self.head + 1) * self.N
        self.obs[lo:hi] = obs
        self.act[lo:hi] = act
        self.rew[lo:hi] = rew
        self.next_obs[lo:hi] = next_obs
        self.done[lo:hi] = done
        self.head = (self.head + 1) % self.T
        self.count = min(self.count + 1, self.T)

    def physical_row(self, j):
        """Chronological row j (0 = oldest valid) -> physical ring row."""
        return (self.head - self.count + j) % self.T


def sample_indices(ring: ReplayRing, nstep: int, batch: int, seed: int, call: int, stream: int = STREAM_SAMPLE):
    """I.i.d. uniform start slots, with replacement (Section 3.1: the V-learner samples
    "a batch of I.I.D. training data"; Algorithm 3).

    Valid starts are the (count - n + 1) * N (row, env) pairs whose n-row window lies
    entirely inside the valid, chronologically contiguous part of the ring.  Sample k:
    u = 64-bit word (w1 << 32 | w0) of the generator; p = floor(u * V / 2^64);
    chronological row j = p div N, env e = p mod N; result = physical_row(j) * N + e.
    """
    if ring.count < nstep:
        raise ValueError("not enough rows pushed for an n-step window")
    V = (ring.count - nstep + 1) * ring.N
    w0, w1, _, _ = rng_words(seed, stream, call, np.arange(batch, dtype=np.uint64))
    idx = np.empty(batch, dtype=np.int64)
    for k in range(batch):                      # exact big-integer arithmetic
        u = (int(w1[k]) << 32) | int(w0[k])
        p = (u * V) >> 64
        j, e = divmod(p, ring.N)
        idx[k] = ring.physical_row(j) * ring.N + e
    return idx


def gather_nstep(ring: ReplayRing, idx, nstep: int, gamma: float):
    """n-step return assembly with termination masking (Section 3: the scheme uses
    n-step returns [Sutton 1988]; d marks termination; Table B.1: n = 3).

    For start slot (row0, e) and rows row_k = row0 + k (mod T), k = 0..n-1:
        ret  = sum_k gamma^k * r[row_k, e] * alive_k,   alive_0 = 1,
               alive_{k+1} = alive_k * (1 - d[row_k, e])
        boot = gamma^n * alive_n
    s, a come from row_0; s' is the next-state of row_{n-1}.  The bootstrapped target is
    then ret + boot * Q'(s', .): once a termination occurs inside the window every later
    reward and the bootstrap are masked out.
    """
    idx = np.asarray(idx, dtype=np.int64)
    N, T = ring.N, ring.T
    row0, env = idx // N, idx % N
    B = idx.shape[0]
    ret = np.zeros(B, dtype=np.float64)
    alive = np.ones(B, dtype=np.float64)
    g = 1.0
    last = idx
    for k in range(nstep):
        slot = ((row0 + k) % T) * N + env
        ret += g * ring.rew[slot].astype(np.float64) * alive
        alive = alive * (1.0 - ring.done[slot].astype(np.float64))
        g *= gamma
        last = slot
    boot = g * alive
    return dict(idx=idx, obs=ring.obs[idx].copy(), act=ring.act[idx].copy(), ret=ret,
                next_obs=ring.next_obs[last].copy(), boot=boot)


def sample_states(ring: ReplayRing, batch: int, seed: int, call: int):
    """The P-learner's batch (Algorithm 2: "sample a batch of {s_t}"): i.i.d. uniform slots,
    with replacement, among all count * N stored transitions (a window of one row), drawn on
    a generator stream of their own; only the states are used.  Returns (slots, states)."""
    idx = sample_indices(ring, 1, batch, seed, call, stream=STREAM_STATE)
    return idx, ring.obs[idx].copy()


# --------------------------------------------------------------------------------------
# Running observation statistics (Table B.1: "Normalized Observations: True"; the paper
# does not describe the mechanism)
# --------------------------------------------------------------------------------------
class ObsNormalizer:
    """Per-dimension mean and population variance of every observation s_t handed to
    ``update`` so far, and the standardisation x -> (x - mean) / sqrt(var + eps).

    The statistics are those of the concatenation of all batches seen; they are carried
    as (count, mean, M2 = sum of squared deviations) and a new batch is merged with the
    pairwise formulas of Chan, Golub and LeVeque (1979).  Before the first batch the mean
    is 0 and the variance 1.
    """

    def __init__(self, dim: int, eps: float = 1e-5):
        self.count = 0
        self.mean = np.zeros(dim, dtype=np.float64)
        self.m2 = np.zeros(dim, dtype=np.float64)
        self.eps = float(eps)

    def update(self, obs):
        x = np.asarray(obs, dtype=np.float64)
        nb = x.shape[0]
        if nb == 0:
            return
        mean_b = x.mean(axis=0)
        m2_b = ((x - mean_b) ** 2).sum(axis=0)
        tot = self.count + nb
        delta = mean_b - self.mean
        self.mean = self.mean + delta * (nb / tot)
        self.m2 = self.m2 + m2_b + delta * delta * (self.count * nb / tot)
        self.count = tot

    @property
    def var(self):
        if self.count == 0:
            return np.ones_like(self.mean)
        return self.m2 / self.count

    def normalize(self, x):
        return (np.asarray(x, dtype=np.float64) - self.mean) / np.sqrt(self.var + self.eps)


def normalize_batch(batch, normalizer: ObsNormalizer):
    """A sampled batch with s and s' standardised by the statistics current at sampling
    time (the replay memory keeps raw observations)."""
    out = dict(batch)
    out["obs"] = normalizer.normalize(batch["obs"])
    out["next_obs"] = normalizer.normalize(batch["next_obs"])
    return out


# --------------------------------------------------------------------------------------
# Networks
# --------------------------------------------------------------------------------------
def unpack(params, dims):
    """Split a flat parameter vector into [(W[in,out], b[out]), ...] (float64 views)."""
    p = np.asarray(params, dtype=np.float64)
    layers, off = [], 0
    for n_in, n_out in dims:
        W = p[off:off + n_in * n_out].reshape(n_in, n_out)
        off += n_in * n_out
        b = p[off:off + n_out]
        off += n_out
        layers.append((W, b))
    assert off == p.size, "parameter vector length does not match the layer dims"
    return layers


def pack(layers):
    return np.concatenate([np.concatenate([W.reshape(-1), b.reshape(-1)]) for W, b in layers])


def elu(z):
    return np.where(z > 0, z, np.exp(np.minimum(z, 0.0)) - 1.0)


def elu_prime(z):
    return np.where(z > 0, 1.0, np.exp(np.minimum(z, 0.0)))


def mlp_forward(layers, x):
    """Returns (pre-activations z_l, activations h_l with h_0 = x).  Hidden layers ELU,
    last layer linear (the caller applies tanh for the actor)."""
    hs, zs = [np.asarray(x, dtype=np.float64)], []
    for li, (W, b) in enumerate(layers):
        z = hs[-1] @ W + b
        zs.append(z)
        hs.append(elu(z) if li < len(layers) - 1 else z)
    return zs, hs


def mlp_backward(layers, zs, hs, d_out):
    """Reverse-mode derivative of ``mlp_forward``.  ``d_out`` = dLoss/d(output).
    Returns (per-layer (dW, db), dLoss/d(input))."""
    grads = [None] * len(layers)
    delta = d_out
    for li in range(len(layers) - 1, -1, -1):
        W, _ = layers[li]
        grads[li] = (hs[li].T @ delta, delta.sum(axis=0))
        delta = delta @ W.T
        if li > 0:
            delta = delta * elu_prime(zs[li - 1])
    return grads, delta


def actor_forward(actor_params, actor_dims, obs):
    zs, hs = mlp_forward(unpack(actor_params, actor_dims), obs)
    return np.tanh(hs[-1])


def critic_forward(critic_params, critic_dims, obs, act):
    x = np.concatenate([np.asarray(obs, np.float64), np.asarray(act, np.float64)], axis=1)
    zs, hs = mlp_forward(unpack(critic_params, critic_dims), x)
    return hs[-1][:, 0]


def split_twin(twin_params):
    p = np.asarray(twin_params)
    half = p.size // 2
    return p[:half], p[half:]


# --------------------------------------------------------------------------------------
# V-learner: target and critic update (Algorithm 3; Section 3.2 "Third": the lagged local
# policy acts as the target policy; Q' is the target Q network; min over the twin critics
# as in Algorithm 2)
# --------------------------------------------------------------------------------------
def td_target(batch, actor_target_params, critic_target_params, actor_dims, critic_dims):
    """y = ret + boot * min_i Q'_i(s', pi^v(s'))."""
    a_next = actor_forward(actor_target_params, actor_dims, batch["next_obs"])
    t1, t2 = split_twin(critic_target_params)
    q1 = critic_forward(t1, critic_dims, batch["next_obs"], a_next)
    q2 = critic_forward(t2, critic_dims, batch["next_obs"], a_next)
    return np.asarray(batch["ret"], np.float64) + np.asarray(batch["boot"], np.float64) * np.minimum(q1, q2)


def critic_loss_and_grads(critic_params, critic_dims, batch, y):
    """Mean-squared Bellman error of both critics against the shared target y
    (Algorithm 3).  L_i = mean_b (Q_i(s_b, a_b) - y_b)^2; the optimised loss is L_1 + L_2;
    y is a constant.  Returns ([L_1, L_2], flat gradient in parameter layout)."""
    x = np.concatenate([np.asarray(batch["obs"], np.float64), np.asarray(batch["act"], np.float64)], axis=1)
    B = x.shape[0]
    losses, flat = [], []
    for p in split_twin(critic_params):
        layers = unpack(p, critic_dims)
        zs, hs = mlp_forward(layers, x)
        err = hs[-1][:, 0] - y
        losses.append(float(np.mean(err * err)))
        grads, _ = mlp_backward(layers, zs, hs, (2.0 * err / B)[:, None])
        flat.append(pack(grads))
    return np.array(losses), np.concatenate(flat)


# --------------------------------------------------------------------------------------
# P-learner: policy update (Algorithm 2: maximise min_i Q_i(s, pi(s)))
# --------------------------------------------------------------------------------------
def actor_loss_and_grads(actor_params, critic_params, actor_dims, critic_dims, obs):
    """J = -mean_b min(Q_1(s_b, pi(s_b)), Q_2(s_b, pi(s_b))); gradient w.r.t. the actor
    parameters only (the critics are constants here).  Ties go to Q_1."""
    obs = np.asarray(obs, np.float64)
    B = obs.shape[0]
    a_layers = unpack(actor_params, actor_dims)
    a_zs, a_hs = mlp_forward(a_layers, obs)
    a_pi = np.tanh(a_hs[-1])
    x = np.concatenate([obs, a_pi], axis=1)
    qs, caches = [], []
    for p in split_twin(critic_params):
        layers = unpack(p, critic_dims)
        zs, hs = mlp_forward(layers, x)
        qs.append(hs[-1][:, 0])
        caches.append((layers, zs, hs))
    pick1 = qs[0] <= qs[1]
    J = -float(np.mean(np.where(pick1, qs[0], qs[1])))
    d_act = np.zeros_like(a_pi)
    for sel, (layers, zs, hs) in zip((pick1, ~pick1), caches):
        d_q = np.where(sel, -1.0 / B, 0.0)[:, None]
        _, d_x = mlp_backward(layers, zs, hs, d_q)
        d_act += d_x[:, obs.shape[1]:]
    d_pre = d_act * (1.0 - a_pi * a_pi)           # tanh'
    grads, _ = mlp_backward(a_layers, a_zs, a_hs, d_pre)
    return J, pack(grads)


# --------------------------------------------------------------------------------------
# PQL-D: distributional critics (Section 3: distributional RL added to PQL; Appendix
# "Distributional critic update": categorical parameterisation over l = 51 fixed atoms on
# (-10, 10), categorical projection, cross-entropy; Bellemare, Dabney, Munos 2017)
# --------------------------------------------------------------------------------------
def atom_values(num_atoms: int, v_min: float, v_max: float):
    """z_j = v_min + j * (v_max - v_min) / (l - 1), j = 0..l-1."""
    return v_min + np.arange(num_atoms, dtype=np.float64) * ((v_max - v_min) / (num_atoms - 1))


def log_softmax(logits):
    x = np.asarray(logits, np.float64)
    x = x - x.max(axis=-1, keepdims=True)
    return x - np.log(np.exp(x).sum(axis=-1, keepdims=True))


def dist_critic_forward(critic_params, critic_dims, obs, act):
    """Logits over the atoms, [B, l]; the critic's last layer has l outputs."""
    x = np.concatenate([np.asarray(obs, np.float64), np.asarray(act, np.float64)], axis=1)
    zs, hs = mlp_forward(unpack(critic_params, critic_dims), x)
    return hs[-1]


def categorical_projection(p_next, ret, boot, z, v_min, v_max):
    """Projection of the shifted and shrunk distribution onto the fixed support
    (Bellemare et al. 2017, Eq. 7), with the n-step quantities of this path in place of
    (r, gamma): atom z_j of the next-state distribution moves to
    T z_j = clip(ret + boot * z_j, v_min, v_max) and its mass p_j is shared between the two
    neighbouring atoms in proportion to proximity:
        m_k = sum_j [1 - |T z_j - z_k| / dz]_0^1 * p_j."""
    p_next = np.asarray(p_next, np.float64)
    dz = (v_max - v_min) / (z.shape[0] - 1)
    tz = np.clip(np.asarray(ret, np.float64)[:, None] + np.asarray(boot, np.float64)[:, None] * z[None, :], v_min, v_max)
    w = np.clip(1.0 - np.abs(tz[:, :, None] - z[None, None, :]) / dz, 0.0, 1.0)        # [B, j, k]
    return np.einsum("bj,bjk->bk", p_next, w)


def dist_td_target(batch, actor_target_params, critic_target_params, actor_dims, critic_dims, v_min, v_max):
    """Target distribution m [B, l]: next action from the lagged policy pi^v (Section 3.2);
    of the twin target critics the one with the smaller expected value at (s', a') supplies
    the next-state distribution (the distributional form of min_i Q'_i; ties: Q'_1), which is
    then projected."""
    l = critic_dims[-1][1]
    z = atom_values(l, v_min, v_max)
    a_next = actor_forward(actor_target_params, actor_dims, batch["next_obs"])
    t1, t2 = split_twin(critic_target_params)
    p1 = np.exp(log_softmax(dist_critic_forward(t1, critic_dims, batch["next_obs"], a_next)))
    p2 = np.exp(log_softmax(dist_critic_forward(t2, critic_dims, batch["next_obs"], a_next)))
    pick1 = (p1 @ z) <= (p2 @ z)
    p_next = np.where(pick1[:, None], p1, p2)
    return categorical_projection(p_next, batch["ret"], batch["boot"], z, v_min, v_max)


def dist_critic_loss_and_grads(critic_params, critic_dims, batch, m):
    """Cross-entropy of each critic's distribution at (s, a) against the projected target:
    L_i = -mean_b sum_k m_bk log p_i,bk; optimised loss L_1 + L_2; m is a constant.
    Returns ([L_1, L_2], flat gradient)."""
    x = np.concatenate([np.asarray(batch["obs"], np.float64), np.asarray(batch["act"], np.float64)], axis=1)
    B = x.shape[0]
    losses, flat = [], []
    for p in split_twin(critic_params):
        layers = unpack(p, critic_dims)
        zs, hs = mlp_forward(layers, x)
        logp = log_softmax(hs[-1])
        losses.append(float(-np.mean(np.sum(m * logp, axis=1))))
        d_logits = (np.exp(logp) * m.sum(axis=1, keepdims=True) - m) / B      # d/dlogits of -sum_k m_k log p_k
        grads, _ = mlp_backward(layers, zs, hs, d_logits)
        flat.append(pack(grads))
    return np.array(losses), np.concatenate(flat)


def dist_actor_loss_and_grads(actor_params, critic_params, actor_dims, critic_dims, obs, v_min, v_max):
    """Policy objective with distributional critics: Q_i = sum_k p_i,k z_k (the mean of the
    distribution) takes the place of the scalar critic in J = -mean_b min_i Q_i(s, pi(s));
    ties go to Q_1; critics constant."""
    obs = np.asarray(obs, np.float64)
    B = obs.shape[0]
    z = atom_values(critic_dims[-1][1], v_min, v_max)
    a_layers = unpack(actor_params, actor_dims)
    a_zs, a_hs = mlp_forward(a_layers, obs)
    a_pi = np.tanh(a_hs[-1])
    x = np.concatenate([obs, a_pi], axis=1)
    qs, caches = [], []
    for p in split_twin(critic_params):
        layers = unpack(p, critic_dims)
        zs, hs = mlp_forward(layers, x)
        prob = np.exp(log_softmax(hs[-1]))
        qs.append(prob @ z)
        caches.append((layers, zs, hs, prob))
    pick1 = qs[0] <= qs[1]
    J = -float(np.mean(np.where(pick1, qs[0], qs[1])))
    d_act = np.zeros_like(a_pi)
    for sel, q, (layers, zs, hs, prob) in zip((pick1, ~pick1), qs, caches):
        d_q = np.where(sel, -1.0 / B, 0.0)[:, None]
        d_logits = d_q * prob * (z[None, :] - q[:, None])       # dQ/dlogit_k = p_k (z_k - Q)
        _, d_x = mlp_backward(layers, zs, hs, d_logits)
        d_act += d_x[:, obs.shape[1]:]
    d_pre = d_act * (1.0 - a_pi * a_pi)
    grads, _ = mlp_backward(a_layers, a_zs, a_hs, d_pre)
    return J, pack(grads)


# --------------------------------------------------------------------------------------
# Optimiser and target tracking (Table B.1: Adam, learning rate 5e-4, target update rate
# tau = 5e-2)
# --------------------------------------------------------------------------------------
def adam_step(theta, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One step of Adam (Kingma & Ba, Algorithm 1) with bias correction; ``t`` is the
    1-based step number.  Returns (theta, m, v)."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return theta - lr * m_hat / (np.sqrt(v_hat) + eps), m, v


def clip_grad_norm(g, max_norm):
    """Gradient clipping by global L2 norm (Table B.1: "Gradient Clipping 0.5"; the kind of
    clipping is not stated): the whole gradient of one optimiser step is rescaled so that
    its Euclidean norm does not exceed ``max_norm``; gradients inside the ball are left
    as they are.  Returns (clipped gradient, norm before clipping)."""
    g = np.asarray(g, dtype=np.float64)
    norm = float(np.sqrt(np.sum(g * g)))
    if max_norm is None or norm <= max_norm:
        return g, norm
    return g * (max_norm / norm), norm


def soft_update(src, dst, tau):
    """Polyak tracking of the target network: dst <- tau * src + (1 - tau) * dst.
    tau = 1 is the hard copy used to refresh the V-learner's lagged policy
    (Section 3.2)."""
    return tau * np.asarray(src, np.float64) + (1.0 - tau) * np.asarray(dst, np.float64)


# --------------------------------------------------------------------------------------
# Actor: exploration step (Section 3.3; Algorithm 1)
# --------------------------------------------------------------------------------------
def exploration_sigma(num_envs: int, sigma_min: float, sigma_max: float):
    """Mixed exploration: sigma_i = sigma_min + (i-1)/(N-1) (sigma_max - sigma_min),
    i = 1..N (returned 0-based).  N = 1 gives sigma_min."""
    if num_envs == 1:
        return np.array([sigma_min], dtype=np.float64)
    i = np.arange(num_envs, dtype=np.float64)
    return sigma_min + (i / (num_envs - 1)) * (sigma_max - sigma_min)


def gaussian_noise(seed: int, call: int, count: int, stream: int = STREAM_ACT):
    """Standard normal draws, one per element index 0..count-1: Box-Muller on two 24-bit
    uniforms u = ((word >> 8) + 0.5) / 2^24 taken from generator words 0 and 1."""
    w0, w1, _, _ = rng_words(seed, stream, call, np.arange(count, dtype=np.uint64))
    u1 = ((w0 >> np.uint64(8)).astype(np.float64) + 0.5) * 2.0 ** -24
    u2 = ((w1 >> np.uint64(8)).astype(np.float64) + 0.5) * 2.0 ** -24
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def actor_act(actor_params, actor_dims, obs, sigma_min, sigma_max, seed, call):
    """a = clip(pi(s) + sigma_i * eps, -1, 1), eps ~ N(0,1) independently per
    (environment, action dimension); element index = env * act_dim + dim."""
    mu = actor_forward(actor_params, actor_dims, obs)
    N, a = mu.shape
    eps = gaussian_noise(seed, call, N * a).reshape(N, a)
    sig = exploration_sigma(N, sigma_min, sigma_max)[:, None]
    return np.clip(mu + sig * eps, -1.0, 1.0)


# --------------------------------------------------------------------------------------
# PQL + SAC (Section 3: the scheme extends to SAC; appendix paragraph "PQL for SAC";
# Table B.1: learnable entropy coefficient).  The paper gives no formulas: the definitions
# are those of Haarnoja et al. 2018 (soft actor-critic with automatic temperature), written
# out for a tanh-squashed diagonal Gaussian policy.
# --------------------------------------------------------------------------------------
LOG_STD_MIN, LOG_STD_MAX = -5.0, 2.0


def sac_policy_sample(actor_params, actor_dims, obs, eps):
    """Stochastic policy: the network's last layer has 2a outputs (mu, raw log sigma);
    log sigma = clip(raw, -5, 2); u = mu + sigma * eps; a = tanh(u);
    log pi(a|s) = sum_d [-eps_d^2 / 2 - log sigma_d - log(2 pi) / 2 - log(1 - tanh(u_d)^2)],
    the last term evaluated as 2 (log 2 - u - softplus(-2u)).  Returns (a, log pi, cache)."""
    layers = unpack(actor_params, actor_dims)
    zs, hs = mlp_forward(layers, obs)
    a_dim = hs[-1].shape[1] // 2
    mu, raw = hs[-1][:, :a_dim], hs[-1][:, a_dim:]
    log_std = np.clip(raw, LOG_STD_MIN, LOG_STD_MAX)
    std = np.exp(log_std)
    u = mu + std * eps
    act = np.tanh(u)
    log_det = 2.0 * (np.log(2.0) - u - np.logaddexp(0.0, -2.0 * u))          # log(1 - tanh(u)^2)
    logp = np.sum(-0.5 * eps * eps - log_std - 0.5 * np.log(2.0 * np.pi) - log_det, axis=1)
    return act, logp, (layers, zs, hs, raw, std, u, act)


def sac_td_target(batch, actor_target_params, critic_target_params, actor_dims, critic_dims, log_alpha, eps):
    """Soft target with n-step quantities: a' ~ pi^v(.|s') (the V-learner's lagged policy,
    Section 3.2), y = ret + boot * (min_i Q'_i(s', a') - alpha log pi^v(a'|s'))."""
    a_next, logp, _ = sac_policy_sample(actor_target_params, actor_dims, batch["next_obs"], eps)
    t1, t2 = split_twin(critic_target_params)
    q = np.minimum(critic_forward(t1, critic_dims, batch["next_obs"], a_next),
                   critic_forward(t2, critic_dims, batch["next_obs"], a_next))
    return np.asarray(batch["ret"], np.float64) + np.asarray(batch["boot"], np.float64) * (q - np.exp(log_alpha) * logp)


def sac_actor_loss_and_grads(actor_params, critic_params, actor_dims, critic_dims, obs, log_alpha, eps):
    """J = mean_b [alpha log pi(a_b|s_b) - min_i Q_i(s_b, a_b)] with the reparameterised
    sample a_b = tanh(mu + sigma eps_b); alpha and the critics are constants; ties in the
    min go to Q_1; the clip of log sigma passes no gradient outside (-5, 2).
    Returns ((Q term, entropy term) of J, flat gradient, mean log pi)."""
    obs = np.asarray(obs, np.float64)
    B = obs.shape[0]
    alpha = np.exp(log_alpha)
    act, logp, (a_layers, a_zs, a_hs, raw, std, u, _) = sac_policy_sample(actor_params, actor_dims, obs, eps)
    x = np.concatenate([obs, act], axis=1)
    qs, caches = [], []
    for p in split_twin(critic_params):
        layers = unpack(p, critic_dims)
        zs, hs = mlp_forward(layers, x)
        qs.append(hs[-1][:, 0])
        caches.append((layers, zs, hs))
    pick1 = qs[0] <= qs[1]
    q_term = -float(np.mean(np.where(pick1, qs[0], qs[1])))
    ent_term = float(alpha * np.mean(logp))
    d_act = np.zeros_like(act)
    for sel, (layers, zs, hs) in zip((pick1, ~pick1), caches):
        _, d_x = mlp_backward(layers, zs, hs, np.where(sel, -1.0 / B, 0.0)[:, None])
        d_act += d_x[:, obs.shape[1]:]
    d_u = d_act * (1.0 - act * act) + (alpha / B) * 2.0 * act       # d log pi / du = 2 tanh(u)
    d_mu = d_u
    inside = (raw > LOG_STD_MIN) & (raw < LOG_STD_MAX)
    d_raw = np.where(inside, d_u * std * eps - alpha / B, 0.0)      # d log pi / d log sigma = -1 + 2 a sigma eps
    grads, _ = mlp_backward(a_layers, a_zs, a_hs, np.concatenate([d_mu, d_raw], axis=1))
    return (q_term, ent_term), pack(grads), float(np.mean(logp))


def sac_actor_act(actor_params, actor_dims, obs, seed, call):
    """The SAC Actor's step: a sample of the stochastic policy (its only exploration), noise
    element index = env * act_dim + dim on the exploration-noise stream."""
    N = np.asarray(obs).shape[0]
    a_dim = actor_dims[-1][1] // 2
    eps = gaussian_noise(seed, call, N * a_dim, STREAM_ACT).reshape(N, a_dim)
    return sac_policy_sample(actor_params, actor_dims, obs, eps)[0]


def sac_alpha_grad(log_alpha, mean_logp, target_entropy):
    """Temperature objective J(alpha) = -alpha * mean_b (log pi + H_target), alpha = exp(log alpha)
    optimised in log alpha: dJ / d log alpha = -alpha (mean log pi + H_target)."""
    return -np.exp(log_alpha) * (mean_logp + target_entropy)


# --------------------------------------------------------------------------------------
# A whole learner, for multi-step parity runs
# --------------------------------------------------------------------------------------
class Learner:
    """Holds the V-/P-learner state in float64 and applies the steps above in the order
    the paper's loops do.  Parameters enter as fp32 arrays and are promoted."""

    def __init__(self, actor_dims, critic_dims, actor_params, critic_params, lr, gamma, tau,
                 beta1=0.9, beta2=0.999, eps=1e-8, max_grad_norm=None, v_min=None, v_max=None,
                 sac=False, log_alpha=0.0, target_entropy=None, seed=0):
        self.actor_dims, self.critic_dims = actor_dims, critic_dims
        self.v_min, self.v_max = v_min, v_max         # set: PQL-D (critic outputs are logits over atoms)
        self.sac, self.seed = sac, seed               # PQL + SAC: stochastic policy, learnable temperature
        self.log_alpha, self.al_m, self.al_v = float(log_alpha), 0.0, 0.0
        self.target_entropy = target_entropy
        self.mean_logp = 0.0
        self.max_grad_norm = max_grad_norm            # None: no clipping
        self.critic_grad_norm = self.actor_grad_norm = 0.0
        self.actor = np.asarray(actor_params, np.float64).copy()
        self.actor_lag = self.actor.copy()            # pi^v, the V-learner's lagged policy
        self.critic = np.asarray(critic_params, np.float64).copy()
        self.critic_target = self.critic.copy()
        self.c_m = np.zeros_like(self.critic); self.c_v = np.zeros_like(self.critic); self.c_t = 0
        self.a_m = np.zeros_like(self.actor); self.a_v = np.zeros_like(self.actor); self.a_t = 0
        self.lr, self.gamma, self.tau = lr, gamma, tau
        self.beta1, self.beta2, self.eps = beta1, beta2, eps

    def critic_update(self, batch):
        if self.sac:
            a_dim = self.actor_dims[-1][1] // 2
            B = np.asarray(batch["ret"]).shape[0]
            eps_n = gaussian_noise(self.seed, self.c_t, B * a_dim, STREAM_SAC_TARGET).reshape(B, a_dim)
            y = sac_td_target(batch, self.actor_lag, self.critic_target, self.actor_dims, self.critic_dims,
                              self.log_alpha, eps_n)
            losses, g = critic_loss_and_grads(self.critic, self.critic_dims, batch, y)
        elif self.v_min is not None:
            m = dist_td_target(batch, self.actor_lag, self.critic_target, self.actor_dims, self.critic_dims,
                               self.v_min, self.v_max)
            losses, g = dist_critic_loss_and_grads(self.critic, self.critic_dims, batch, m)
        else:
            y = td_target(batch, self.actor_lag, self.critic_target, self.actor_dims, self.critic_dims)
            losses, g = critic_loss_and_grads(self.critic, self.critic_dims, batch, y)
        g, self.critic_grad_norm = clip_grad_norm(g, self.max_grad_norm)   # both critics: one step, one norm
        self.c_t += 1
        self.critic, self.c_m, self.c_v = adam_step(self.critic, g, self.c_m, self.c_v, self.c_t,
                                                    self.lr, self.beta1, self.beta2, self.eps)
        return losses, g

    def soft_update_targets(self):
        self.critic_target = soft_update(self.critic, self.critic_target, self.tau)

    def actor_update(self, obs):
        if self.sac:
            a_dim = self.actor_dims[-1][1] // 2
            B = np.asarray(obs).shape[0]
            eps_n = gaussian_noise(self.seed, self.a_t, B * a_dim, STREAM_SAC_POLICY).reshape(B, a_dim)
            J, g, self.mean_logp = sac_actor_loss_and_grads(self.actor, self.critic, self.actor_dims, self.critic_dims,
                                                            obs, self.log_alpha, eps_n)
        elif self.v_min is not None:
            J, g = dist_actor_loss_and_grads(self.actor, self.critic, self.actor_dims, self.critic_dims, obs,
                                             self.v_min, self.v_max)
        else:
            J, g = actor_loss_and_grads(self.actor, self.critic, self.actor_dims, self.critic_dims, obs)
        g, self.actor_grad_norm = clip_grad_norm(g, self.max_grad_norm)
        self.a_t += 1
        self.actor, self.a_m, self.a_v = adam_step(self.actor, g, self.a_m, self.a_v, self.a_t,
                                                   self.lr, self.beta1, self.beta2, self.eps)
        if self.sac:    # temperature step on the same batch, with the log-probabilities of the sampled actions
            ga = sac_alpha_grad(self.log_alpha, self.mean_logp, self.target_entropy)
            self.log_alpha, self.al_m, self.al_v = (float(x) for x in adam_step(
                self.log_alpha, ga, self.al_m, self.al_v, self.a_t, self.lr, self.beta1, self.beta2, self.eps))
        return J, g

    def sync_lagged_policy(self):
        self.actor_lag = soft_update(self.actor, self.actor_lag, 1.0)


# --------------------------------------------------------------------------------------
# The parallel scheme (Section 3.1, Section 3.2, Algorithms 1-3) as a deterministic schedule
# --------------------------------------------------------------------------------------
class ParallelScheme:
    """Actor, V-learner and P-learner with their local copies (pi^a, pi^v, Q^p), exchanging
    data and networks once per Actor iteration, as Algorithms 1-3 route every transfer
    through the Actor's loop.

    The paper's processes run asynchronously and are throttled by sleeping so that the
    update frequencies keep the ratios beta_a:v and beta_p:v (Section 3.2).  Here the same
    ratios are kept exactly: one *period* is one Actor iteration of ``horizon`` environment
    steps, ``v_updates`` critic updates and ``p_updates`` policy updates (1 : 8 and 1 : 2 by
    default give 1 step, 8 and 4).  Within a period the three parts only touch their local
    copies, so they are independent of each other and may run in any order or at the same
    time; at the period boundary
        * the V-learner receives the transitions the Actor produced during the period and
          the P-learner's policy (-> pi^v, the lagged target policy of Section 3.2);
        * the P-learner receives those states (here: it samples states from the same
          store, which then contains them) and the V-learner's critics (-> Q^p);
        * the Actor receives the P-learner's policy (-> pi^a).
    ``env_step(period, step, actions)`` plays the simulator: it returns the transition rows
    (obs, rew, next_obs, done) of that step; obs must not depend on the actions (synthetic
    data), the actions are stored with the transition.
    """

    def __init__(self, learner: Learner, ring: ReplayRing, nstep: int, batch: int, seed: int,
                 sigma_min: float, sigma_max: float, normalizer: ObsNormalizer = None,
                 horizon: int = 1, v_updates: int = 8, p_updates: int = 4):
        self.L, self.ring, self.nstep, self.batch, self.seed = learner, ring, nstep, batch, seed
        self.sigma_min, self.sigma_max, self.nz = sigma_min, sigma_max, normalizer
        self.horizon, self.v_updates, self.p_updates = horizon, v_updates, p_updates
        self.pi_a = learner.actor.copy()              # the Actor's local policy
        self.q_p = learner.critic.copy()              # the P-learner's local critics
        self.log_alpha_v = learner.log_alpha          # SAC variant: the V-learner's copy of the temperature
        learner.actor_lag = learner.actor.copy()      # pi^v
        self.sample_calls = self.state_calls = self.act_calls = 0
        self.period = 0
        self.trace = []                               # per period: what each part used

    def run_period(self, env_step, obs_rows):
        """obs_rows[t]: the observations s_t the Actor sees at step t of this period."""
        L = self.L
        rec = dict(pi_a=self.pi_a.copy(), pi_v=L.actor_lag.copy(), q_p=self.q_p.copy(), rows=self.ring.count,
                   log_alpha_v=self.log_alpha_v)
        # ---- Actor (Algorithm 1): roll out pi^a; the transitions are delivered at the boundary
        produced = []
        for t in range(self.horizon):
            s = obs_rows[t]
            seen = s if self.nz is None else self.nz.normalize(s)
            if L.sac:
                a = sac_actor_act(self.pi_a, L.actor_dims, seen, self.seed, self.act_calls)
            else:
                a = actor_act(self.pi_a, L.actor_dims, seen, self.sigma_min, self.sigma_max, self.seed, self.act_calls)
            self.act_calls += 1
            row = env_step(self.period, t, a)
            produced.append(dict(row, act=a.astype(np.float32)))
        # ---- V-learner (Algorithm 3): critic updates with the lagged policy pi^v (and its copy of the temperature)
        v_losses = []
        log_alpha_p = L.log_alpha
        L.log_alpha = self.log_alpha_v
        for _ in range(self.v_updates):
            b = gather_nstep(self.ring, sample_indices(self.ring, self.nstep, self.batch, self.seed, self.sample_calls),
                             self.nstep, L.gamma)
            self.sample_calls += 1
            rec["v_idx"] = b["idx"]                    # slots of the last batch, for inspection
            if self.nz is not None:
                b = normalize_batch(b, self.nz)
            losses, _ = L.critic_update(b)
            L.soft_update_targets()
            v_losses.append(losses)
        L.log_alpha = log_alpha_p
        # ---- P-learner (Algorithm 2): policy updates against its local critics Q^p
        q_v = L.critic
        L.critic = self.q_p
        p_losses = []
        for _ in range(self.p_updates):
            rec["p_idx"], states = sample_states(self.ring, self.batch, self.seed, self.state_calls)
            self.state_calls += 1
            if self.nz is not None:
                states = self.nz.normalize(states)
            J, _ = L.actor_update(states)
            p_losses.append(J)
        L.critic = q_v
        # ---- period boundary: data and network transfer
        for row in produced:
            self.ring.push(row["obs"], row["act"], row["rew"], row["next_obs"], row["done"])
            if self.nz is not None:
                self.nz.update(row["obs"])
        L.sync_lagged_policy()                        # pi^v <- pi^p
        self.pi_a = L.actor.copy()                    # pi^a <- pi^p
        self.q_p = L.critic.copy()                    # Q^p  <- Q^v
        self.log_alpha_v = L.log_alpha
        rec.update(v_losses=v_losses, p_losses=p_losses, actions=[r["act"] for r in produced])
        self.trace.append(rec)
        self.period += 1
        return rec
