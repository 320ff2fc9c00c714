"""Pins for the oracle's floating-point parts: networks, losses, gradients, Adam, Polyak,
exploration.  Independent evidence only: hand-computed small nets, central finite
differences, closed forms, PyTorch CPU autograd / optim as a library cross-check.
"""
import numpy as np
import pytest
import torch
from scipy import stats

from oracle import pql_oracle as O
from paper_2307_12983_amd import workloads as W


def _nets(o=5, a=3, hidden=(7, 6), seed=0):
    rng = np.random.default_rng(seed)
    ad, cd = W.layer_dims(o, hidden, a), W.layer_dims(o + a, hidden, 1)
    actor = W.init_params(ad, rng).astype(np.float64)
    critic = np.concatenate([W.init_params(cd, rng), W.init_params(cd, rng)]).astype(np.float64)
    return ad, cd, actor, critic


def _batch(B, o, a, seed=1):
    rng = np.random.default_rng(seed)
    return dict(obs=rng.standard_normal((B, o)), act=rng.uniform(-1, 1, (B, a)), ret=rng.standard_normal(B),
                next_obs=rng.standard_normal((B, o)), boot=rng.choice([0.0, 0.97], size=B, p=[0.2, 0.8]))


# ---------------------------------------------------------------- forward
def test_mlp_by_hand_single_hidden_layer():
    # 2 inputs -> 2 hidden (ELU) -> 1 output, all numbers worked out by hand
    Wm = np.array([[1.0, -1.0], [0.5, 2.0]]); b1 = np.array([0.0, -1.0])
    w2 = np.array([[2.0], [-3.0]]); b2 = np.array([0.25])
    flat = np.concatenate([Wm.ravel(), b1, w2.ravel(), b2])
    x = np.array([[1.0, 1.0], [-2.0, 0.0]])
    # row 0: z = (1.5, 0.0) -> h = (1.5, 0) -> q = 3.0 + 0.25
    # row 1: z = (-2, 1)    -> h = (e^-2 - 1, 1) -> q = 2(e^-2 - 1) - 3 + 0.25
    q = O.critic_forward(flat, [(2, 2), (2, 1)], x[:, :1], x[:, 1:])
    assert np.allclose(q, [3.25, 2 * (np.exp(-2.0) - 1) - 2.75], rtol=1e-14)
    pi = O.actor_forward(flat, [(2, 2), (2, 1)], x)
    assert np.allclose(pi[:, 0], np.tanh([3.25, 2 * (np.exp(-2.0) - 1) - 2.75]), rtol=1e-14)


def test_elu_special_values():
    z = np.array([0.0, -1e3, 3.0, -np.log(2.0)])
    assert np.allclose(O.elu(z), [0.0, -1.0, 3.0, -0.5])
    assert np.allclose(O.elu_prime(z), [1.0, 0.0, 1.0, 0.5])


def test_forward_matches_torch_modules():
    ad, cd, actor, critic = _nets()
    b = _batch(9, 5, 3)

    def torch_mlp(flat, dims, x, tanh):
        h, off = torch.tensor(x), 0
        for li, (i, o) in enumerate(dims):
            Wt = torch.tensor(flat[off:off + i * o]).reshape(i, o); off += i * o
            bt = torch.tensor(flat[off:off + o]); off += o
            h = h @ Wt + bt
            if li < len(dims) - 1:
                h = torch.nn.functional.elu(h)
        return torch.tanh(h) if tanh else h

    assert np.allclose(O.actor_forward(actor, ad, b["obs"]), torch_mlp(actor, ad, b["obs"], True).numpy(), rtol=1e-12)
    q1 = torch_mlp(critic[:critic.size // 2], cd, np.concatenate([b["obs"], b["act"]], 1), False)[:, 0]
    assert np.allclose(O.critic_forward(critic[:critic.size // 2], cd, b["obs"], b["act"]), q1.numpy(), rtol=1e-12)


def test_twin_critics_with_identical_parameters_agree():
    ad, cd, actor, critic = _nets()
    half = critic[:critic.size // 2]
    b = _batch(6, 5, 3)
    twin = np.concatenate([half, half])
    y = O.td_target(b, actor, twin, ad, cd)
    losses, g = O.critic_loss_and_grads(twin, cd, b, y)
    assert losses[0] == losses[1] and np.array_equal(g[:half.size], g[half.size:])


# ---------------------------------------------------------------- target
def test_target_properties():
    ad, cd, actor, critic = _nets()
    b = _batch(32, 5, 3)
    y = O.td_target(b, actor, critic, ad, cd)
    # boot = 0 -> y = ret whatever the networks are
    assert np.array_equal(y[b["boot"] == 0], b["ret"][b["boot"] == 0])
    # symmetric in the two target critics
    half = critic.size // 2
    y_swapped = O.td_target(b, actor, np.concatenate([critic[half:], critic[:half]]), ad, cd)
    assert np.array_equal(y, y_swapped)
    # explicit recomputation through the component calls
    a2 = O.actor_forward(actor, ad, b["next_obs"])
    q = np.minimum(O.critic_forward(critic[:half], cd, b["next_obs"], a2), O.critic_forward(critic[half:], cd, b["next_obs"], a2))
    assert np.allclose(y, b["ret"] + b["boot"] * q, rtol=1e-14)
    assert np.all(y <= b["ret"] + b["boot"] * O.critic_forward(critic[:half], cd, b["next_obs"], a2) + 1e-15)


# ---------------------------------------------------------------- gradients
def _central_diff(f, x, h=1e-6):
    g = np.zeros_like(x)
    for i in range(x.size):
        xp, xm = x.copy(), x.copy()
        xp[i] += h; xm[i] -= h
        g[i] = (f(xp) - f(xm)) / (2 * h)
    return g


def test_critic_gradient_matches_finite_differences():
    ad, cd, actor, critic = _nets(o=4, a=2, hidden=(5, 4))
    b = _batch(11, 4, 2)
    y = O.td_target(b, actor, critic, ad, cd)
    losses, g = O.critic_loss_and_grads(critic, cd, b, y)
    fd = _central_diff(lambda p: O.critic_loss_and_grads(p, cd, b, y)[0].sum(), critic)
    assert np.max(np.abs(g - fd)) / np.max(np.abs(fd)) < 1e-7
    assert np.allclose(g, fd, rtol=1e-5, atol=1e-9)


def test_actor_gradient_matches_finite_differences():
    ad, cd, actor, critic = _nets(o=4, a=2, hidden=(5, 4), seed=3)
    obs = _batch(13, 4, 2, seed=4)["obs"]
    # keep away from the kink of min(q1, q2)
    a_pi = O.actor_forward(actor, ad, obs)
    half = critic.size // 2
    gap = np.abs(O.critic_forward(critic[:half], cd, obs, a_pi) - O.critic_forward(critic[half:], cd, obs, a_pi))
    obs = obs[gap > 1e-3]
    assert obs.shape[0] >= 8
    J, g = O.actor_loss_and_grads(actor, critic, ad, cd, obs)
    fd = _central_diff(lambda p: O.actor_loss_and_grads(p, critic, ad, cd, obs)[0], actor)
    assert np.max(np.abs(g - fd)) / np.max(np.abs(fd)) < 1e-7
    assert np.allclose(g, fd, rtol=1e-5, atol=1e-9)


def _torch_params(flat, dims):
    ps, off = [], 0
    for i, o in dims:
        ps.append(torch.tensor(flat[off:off + i * o].reshape(i, o), requires_grad=True)); off += i * o
        ps.append(torch.tensor(flat[off:off + o].copy(), requires_grad=True)); off += o
    return ps


def _torch_mlp(ps, x):
    h = x
    for li in range(0, len(ps), 2):
        h = h @ ps[li] + ps[li + 1]
        if li < len(ps) - 2:
            h = torch.nn.functional.elu(h)
    return h


def test_critic_and_actor_gradients_match_torch_autograd():
    ad, cd, actor, critic = _nets(o=6, a=3, hidden=(16, 12, 8), seed=5)
    b = _batch(40, 6, 3, seed=6)
    y = O.td_target(b, actor, critic, ad, cd)
    losses, g = O.critic_loss_and_grads(critic, cd, b, y)
    half = critic.size // 2
    x = torch.tensor(np.concatenate([b["obs"], b["act"]], 1))
    for i, sl in enumerate((slice(0, half), slice(half, None))):
        ps = _torch_params(critic[sl], cd)
        loss = torch.nn.functional.mse_loss(_torch_mlp(ps, x)[:, 0], torch.tensor(y))
        loss.backward()
        assert np.isclose(loss.item(), losses[i], rtol=1e-12)
        tg = np.concatenate([p.grad.numpy().ravel() for p in ps])
        assert np.allclose(g[sl], tg, rtol=1e-10, atol=1e-14)
    # policy objective: -mean(min(Q1, Q2)(s, pi(s)))
    J, ga = O.actor_loss_and_grads(actor, critic, ad, cd, b["obs"])
    pa = _torch_params(actor, ad)
    s = torch.tensor(b["obs"])
    xa = torch.cat([s, torch.tanh(_torch_mlp(pa, s))], 1)
    q1 = _torch_mlp([p.detach() for p in _torch_params(critic[:half], cd)], xa)[:, 0]
    q2 = _torch_mlp([p.detach() for p in _torch_params(critic[half:], cd)], xa)[:, 0]
    Jt = -torch.minimum(q1, q2).mean()
    Jt.backward()
    assert np.isclose(Jt.item(), J, rtol=1e-12)
    assert np.allclose(ga, np.concatenate([p.grad.numpy().ravel() for p in pa]), rtol=1e-10, atol=1e-14)


# ---------------------------------------------------------------- Adam, Polyak
def test_adam_first_step_closed_form():
    rng = np.random.default_rng(0)
    theta, g = rng.standard_normal(50), rng.standard_normal(50) * 1e-3
    g[:3] = 0.0
    lr, eps = 5e-4, 1e-8
    t1, m, v = O.adam_step(theta, g, np.zeros(50), np.zeros(50), 1, lr, 0.9, 0.999, eps)
    assert np.allclose(t1 - theta, -lr * g / (np.abs(g) + eps), rtol=1e-9, atol=0)
    assert np.array_equal(t1[:3], theta[:3])
    # a constant gradient keeps producing the same step
    t2, m, v = O.adam_step(t1, g, m, v, 2, lr, 0.9, 0.999, eps)
    assert np.allclose(t2 - t1, -lr * g / (np.abs(g) + eps), rtol=1e-9, atol=0)


def test_adam_matches_torch_optim_over_several_steps():
    rng = np.random.default_rng(1)
    theta = rng.standard_normal(30)
    p = torch.tensor(theta.copy(), requires_grad=True)
    opt = torch.optim.Adam([p], lr=5e-4, betas=(0.9, 0.999), eps=1e-8)
    m, v = np.zeros(30), np.zeros(30)
    for t in range(1, 8):
        g = rng.standard_normal(30) * 10.0 ** rng.integers(-6, 1)
        p.grad = torch.tensor(g.copy())
        opt.step()
        theta, m, v = O.adam_step(theta, g, m, v, t, 5e-4, 0.9, 0.999, 1e-8)
        assert np.allclose(theta, p.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_polyak_pins():
    rng = np.random.default_rng(2)
    src, dst = rng.standard_normal(100).astype(np.float32), rng.standard_normal(100).astype(np.float32)
    assert np.array_equal(O.soft_update(src, dst, 1.0), src)        # hard copy, bitwise
    assert np.array_equal(O.soft_update(src, dst, 0.0), dst)        # identity, bitwise
    assert O.soft_update(np.array([1.0]), np.array([3.0]), 0.5)[0] == 2.0
    assert np.allclose(O.soft_update(src, src, 0.05), src, rtol=1e-15)
    out = O.soft_update(np.array([10.0]), np.array([0.0]), 0.05)    # moves 5% of the way to src
    assert np.isclose(out[0], 0.5)


# ---------------------------------------------------------------- exploration
def test_sigma_schedule_endpoints_and_linearity():
    s = O.exploration_sigma(4096, 0.05, 0.8)
    assert s[0] == 0.05 and np.isclose(s[-1], 0.8, rtol=1e-15) and s.size == 4096
    assert np.allclose(np.diff(s), (0.8 - 0.05) / 4095, rtol=1e-9)
    assert O.exploration_sigma(1, 0.05, 0.8).tolist() == [0.05]
    assert np.all(O.exploration_sigma(7, 0.2, 0.2) == 0.2)


def test_act_is_deterministic_policy_without_noise_and_bounded_with():
    ad, cd, actor, critic = _nets()
    obs = _batch(64, 5, 3)["obs"]
    assert np.array_equal(O.actor_act(actor, ad, obs, 0.0, 0.0, 1, 0), O.actor_forward(actor, ad, obs))
    a = O.actor_act(actor, ad, obs, 0.05, 0.8, 1, 0)
    assert a.min() >= -1.0 and a.max() <= 1.0 and (np.abs(a) == 1.0).any()
    assert np.array_equal(a, O.actor_act(actor, ad, obs, 0.05, 0.8, 1, 0))
    assert not np.array_equal(a, O.actor_act(actor, ad, obs, 0.05, 0.8, 1, 1))


def test_noise_is_standard_normal():
    e = O.gaussian_noise(seed=3, call=0, count=200_000)
    assert abs(e.mean()) < 0.01 and abs(e.var() - 1.0) < 0.01
    assert stats.kstest(e, "norm").pvalue > 1e-3
    assert abs(stats.kurtosis(e)) < 0.05
    # recover the residual of the clipped action: (a - pi(s)) / sigma_i on unclipped entries
    ad, cd, actor, critic = _nets()
    obs = _batch(4096, 5, 3)["obs"]
    a = O.actor_act(actor, ad, obs, 0.05, 0.3, 3, 7)
    mu = O.actor_forward(actor, ad, obs)
    sig = O.exploration_sigma(4096, 0.05, 0.3)[:, None]
    inside = np.abs(a) < 1.0
    resid = ((a - mu) / sig)
    assert np.allclose(resid[inside], O.gaussian_noise(3, 7, 4096 * 3).reshape(4096, 3)[inside], atol=1e-9)


# ---------------------------------------------------------------- whole update
def test_update_on_same_batch_decreases_loss():
    w = W.WORKLOADS["tiny"]
    actor, critic = W.init_networks(w)
    L = O.Learner(w.actor_dims(), w.critic_dims(), actor, critic, 1e-4, w.gamma, w.tau)
    b = _batch(256, w.obs_dim, w.act_dim)
    l0, _ = L.critic_update(b)
    l1, _ = L.critic_update(b)
    assert l1.sum() < l0.sum()
    j0, _ = L.actor_update(b["obs"])
    j1, _ = L.actor_update(b["obs"])
    assert j1 < j0
