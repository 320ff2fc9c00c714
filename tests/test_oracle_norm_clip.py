"""Pins for the oracle's running observation statistics and gradient-norm clipping
(Table B.1: "Normalized Observations", "Gradient Clipping 0.5").  Evidence independent of the
oracle's own formulas: statistics of the concatenated data, invariances, hand-worked numbers,
PyTorch's clipping routine and a PyTorch training step as library cross-checks.
"""
import numpy as np
import pytest
import torch

from oracle import pql_oracle as O
from paper_2307_12983_amd import workloads as W


def _pushes(seed, sizes, dim):
    rng = np.random.default_rng(seed)
    loc = rng.uniform(-50.0, 50.0, dim)
    scale = 10.0 ** rng.uniform(-2.0, 2.0, dim)
    return [loc + scale * rng.standard_normal((n, dim)) for n in sizes]


# ---------------------------------------------------------------- running statistics
@pytest.mark.parametrize("sizes", [(1,), (3,), (5, 1, 7), (64, 64, 64, 64), (1, 1, 1, 1, 1), (17, 256, 3)])
def test_statistics_are_those_of_the_concatenated_data(sizes):
    dim = 6
    batches = _pushes(3, sizes, dim)
    nz = O.ObsNormalizer(dim, eps=1e-5)
    for b in batches:
        nz.update(b)
    allx = np.concatenate(batches)
    assert nz.count == allx.shape[0]
    assert np.allclose(nz.mean, allx.mean(axis=0), rtol=1e-12, atol=0)
    # population variance (divide by the count): with 3 rows the two conventions differ by 50 %
    assert np.allclose(nz.var, allx.var(axis=0, ddof=0), rtol=1e-9, atol=1e-300)
    if allx.shape[0] > 1:
        assert not np.allclose(nz.var, allx.var(axis=0, ddof=1), rtol=1e-3)


def test_statistics_do_not_depend_on_how_the_data_was_split():
    dim = 4
    data = _pushes(5, (240,), dim)[0]
    ref = O.ObsNormalizer(dim)
    ref.update(data)
    for cuts in [(1, 239), (120, 120), (7, 100, 133), tuple([24] * 10)]:
        nz = O.ObsNormalizer(dim)
        pos = 0
        for c in cuts:
            nz.update(data[pos:pos + c])
            pos += c
        assert np.allclose(nz.mean, ref.mean, rtol=1e-13)
        assert np.allclose(nz.var, ref.var, rtol=1e-11)


def test_hand_worked_statistics():
    # column 0: 1, 2, 3, 6 -> mean 3, population variance (4 + 1 + 0 + 9) / 4 = 3.5
    # column 1: constant 5 -> variance 0
    nz = O.ObsNormalizer(2, eps=0.25)
    nz.update(np.array([[1.0, 5.0], [2.0, 5.0]]))
    nz.update(np.array([[3.0, 5.0]]))
    nz.update(np.array([[6.0, 5.0]]))
    assert nz.count == 4
    assert np.allclose(nz.mean, [3.0, 5.0], rtol=1e-15)
    assert np.allclose(nz.var, [3.5, 0.0], rtol=1e-15, atol=1e-30)
    out = nz.normalize(np.array([[7.0, 5.0], [3.0, 6.0]]))
    # (7 - 3) / sqrt(3.75), 0 ; 0, (6 - 5) / sqrt(0.25)
    assert np.allclose(out, [[4.0 / np.sqrt(3.75), 0.0], [0.0, 2.0]], rtol=1e-15)


def test_before_any_data_mean_is_zero_and_variance_one():
    nz = O.ObsNormalizer(3, eps=1e-5)
    x = np.array([[1.0, -2.0, 0.5]])
    assert np.allclose(nz.normalize(x), x / np.sqrt(1.0 + 1e-5), rtol=1e-15)
    nz.update(np.zeros((0, 3)))
    assert nz.count == 0


def test_normalized_data_is_standardised():
    dim = 5
    batches = _pushes(9, (100, 300, 50), dim)
    nz = O.ObsNormalizer(dim, eps=0.0)
    for b in batches:
        nz.update(b)
    z = nz.normalize(np.concatenate(batches))
    assert np.allclose(z.mean(axis=0), 0.0, atol=1e-10)
    assert np.allclose(z.var(axis=0), 1.0, rtol=1e-10)


def test_normalisation_is_invariant_to_an_affine_change_of_units():
    dim = 3
    batches = _pushes(11, (40, 60), dim)
    a, b = np.array([2.0, -0.5, 100.0]), np.array([1.0, 7.0, -3.0])
    n1, n2 = O.ObsNormalizer(dim, eps=0.0), O.ObsNormalizer(dim, eps=0.0)
    for x in batches:
        n1.update(x)
        n2.update(a * x + b)
    q = batches[0][:10]
    assert np.allclose(n2.normalize(a * q + b), np.sign(a) * n1.normalize(q), rtol=1e-9, atol=1e-12)


def test_normalize_batch_touches_only_observations():
    rng = np.random.default_rng(0)
    nz = O.ObsNormalizer(4)
    nz.update(3.0 + 2.0 * rng.standard_normal((50, 4)))
    batch = dict(idx=np.arange(6), obs=rng.standard_normal((6, 4)), act=rng.standard_normal((6, 2)),
                 ret=rng.standard_normal(6), next_obs=rng.standard_normal((6, 4)), boot=np.ones(6))
    out = O.normalize_batch(batch, nz)
    for k in ("idx", "act", "ret", "boot"):
        assert out[k] is batch[k]
    assert np.array_equal(out["obs"], nz.normalize(batch["obs"]))
    assert np.array_equal(out["next_obs"], nz.normalize(batch["next_obs"]))
    assert not np.allclose(out["obs"], batch["obs"])


# ---------------------------------------------------------------- gradient clipping
def test_clip_hand_example_and_identity_inside_the_ball():
    g, n = O.clip_grad_norm(np.array([3.0, 4.0]), 0.5)
    assert n == 5.0 and np.allclose(g, [0.3, 0.4], rtol=1e-15)
    small = np.array([0.3, -0.4])                       # norm exactly at the bound: unchanged
    g2, n2 = O.clip_grad_norm(small, 0.5)
    assert np.array_equal(g2, small) and abs(n2 - 0.5) < 1e-15
    g3, n3 = O.clip_grad_norm(np.zeros(4), 0.5)
    assert n3 == 0.0 and np.array_equal(g3, np.zeros(4))
    g4, _ = O.clip_grad_norm(np.array([3.0, 4.0]), None)
    assert np.array_equal(g4, [3.0, 4.0])


@pytest.mark.parametrize("scale", [1e-3, 0.1, 1.0, 50.0])
def test_clip_properties(scale):
    rng = np.random.default_rng(4)
    g = scale * rng.standard_normal(1000)
    c = 0.5
    gc, n = O.clip_grad_norm(g, c)
    assert np.isclose(n, np.linalg.norm(g), rtol=1e-14)
    assert np.isclose(np.linalg.norm(gc), min(n, c), rtol=1e-13)
    assert np.isclose(np.dot(gc, g), np.linalg.norm(gc) * n, rtol=1e-12)      # same direction


def test_clip_matches_torch_routine():
    # torch divides by (norm + 1e-6): agreement to ~2e-6 relative at a norm of order one
    rng = np.random.default_rng(5)
    parts = [rng.standard_normal((7, 5)), rng.standard_normal(5), rng.standard_normal((5, 1))]
    ps = [torch.nn.Parameter(torch.zeros(p.shape, dtype=torch.float64)) for p in parts]
    for p, g in zip(ps, parts):
        p.grad = torch.tensor(g)
    tn = torch.nn.utils.clip_grad_norm_(ps, 0.5)
    flat = np.concatenate([p.ravel() for p in parts])
    gc, n = O.clip_grad_norm(flat, 0.5)
    assert np.isclose(n, float(tn), rtol=1e-13)
    got = np.concatenate([p.grad.numpy().ravel() for p in ps])
    assert np.allclose(gc, got, rtol=1e-5, atol=0)


def _torch_params(flat, dims):
    out, pos = [], 0
    for (i, o) in dims:
        Wt = torch.tensor(flat[pos:pos + i * o].reshape(i, o), dtype=torch.float64, requires_grad=True); pos += i * o
        bt = torch.tensor(flat[pos:pos + o], dtype=torch.float64, requires_grad=True); pos += o
        out += [Wt, bt]
    return out


def _torch_mlp(ps, x):
    h = x
    n = len(ps) // 2
    for l in range(n):
        h = h @ ps[2 * l] + ps[2 * l + 1]
        if l < n - 1:
            h = torch.nn.functional.elu(h)
    return h


def test_learner_steps_with_clipping_and_normalised_batch_match_a_torch_training_loop():
    """Three critic updates and policy updates with clipping on a standardised batch, against
    torch autograd + clip_grad_norm_ + Adam written as a user of that library would."""
    o, a, hidden, B = 5, 3, (8, 6), 40
    rng = np.random.default_rng(21)
    ad, cd = W.layer_dims(o, hidden, a), W.layer_dims(o + a, hidden, 1)
    actor = W.init_params(ad, rng).astype(np.float64)
    critic = np.concatenate([W.init_params(cd, rng), W.init_params(cd, rng)]).astype(np.float64)
    nz = O.ObsNormalizer(o, eps=1e-5)
    nz.update(4.0 + 3.0 * rng.standard_normal((500, o)))
    lr, c = 1e-2, 0.5
    L = O.Learner(ad, cd, actor, critic, lr=lr, gamma=0.99, tau=0.05, max_grad_norm=c)

    half = critic.size // 2
    tq = [_torch_params(critic[:half], cd), _torch_params(critic[half:], cd)]
    tq_targ = [[p.detach().clone() for p in q] for q in tq]
    tpi = _torch_params(actor, ad)
    tpi_lag = [p.detach().clone() for p in tpi]
    opt_q = torch.optim.Adam(tq[0] + tq[1], lr=lr, eps=1e-8)
    opt_pi = torch.optim.Adam(tpi, lr=lr, eps=1e-8)
    mu_t, sd_t = torch.tensor(nz.mean), torch.sqrt(torch.tensor(nz.var) + 1e-5)

    clipped = 0
    for step in range(3):
        raw = dict(obs=4.0 + 3.0 * rng.standard_normal((B, o)), act=rng.uniform(-1, 1, (B, a)),
                   ret=5.0 * rng.standard_normal(B), next_obs=4.0 + 3.0 * rng.standard_normal((B, o)),
                   boot=rng.choice([0.0, 0.97], size=B, p=[0.2, 0.8]))
        batch = O.normalize_batch(raw, nz)
        L.critic_update(batch)
        L.soft_update_targets()
        L.actor_update(batch["obs"])
        L.sync_lagged_policy()
        clipped += int(L.critic_grad_norm > c) + int(L.actor_grad_norm > c)

        s = (torch.tensor(raw["obs"]) - mu_t) / sd_t
        s2 = (torch.tensor(raw["next_obs"]) - mu_t) / sd_t
        act_t, ret_t, boot_t = torch.tensor(raw["act"]), torch.tensor(raw["ret"]), torch.tensor(raw["boot"])
        with torch.no_grad():
            a2 = torch.tanh(_torch_mlp(tpi_lag, s2))
            x2 = torch.cat([s2, a2], dim=1)
            y = ret_t + boot_t * torch.minimum(_torch_mlp(tq_targ[0], x2), _torch_mlp(tq_targ[1], x2))[:, 0]
        x = torch.cat([s, act_t], dim=1)
        loss = sum(((_torch_mlp(q, x)[:, 0] - y) ** 2).mean() for q in tq)
        opt_q.zero_grad(); loss.backward()
        torch.nn.utils.clip_grad_norm_(tq[0] + tq[1], c)
        opt_q.step()
        with torch.no_grad():
            for q, qt in zip(tq, tq_targ):
                for p, pt in zip(q, qt):
                    pt.mul_(0.95).add_(0.05 * p)
        xa = torch.cat([s, torch.tanh(_torch_mlp(tpi, s))], dim=1)
        J = -torch.minimum(_torch_mlp(tq[0], xa), _torch_mlp(tq[1], xa)).mean()
        opt_pi.zero_grad()
        for q in tq:
            for p in q:
                p.grad = None
        J.backward()
        torch.nn.utils.clip_grad_norm_(tpi, c)
        opt_pi.step()
        with torch.no_grad():
            for p, pl in zip(tpi, tpi_lag):
                pl.copy_(p)

    assert clipped >= 2                                     # the clip was active, not a no-op
    got_c = np.concatenate([np.concatenate([p.detach().numpy().ravel() for p in q]) for q in tq])
    got_a = np.concatenate([p.detach().numpy().ravel() for p in tpi])
    # torch's 1e-6 in the clip coefficient perturbs the clipped gradient by ~1e-6 relative
    assert np.allclose(L.critic, got_c, rtol=0, atol=3 * lr * 1e-4)
    assert np.allclose(L.actor, got_a, rtol=0, atol=3 * lr * 1e-4)
    assert np.abs(L.critic - critic).max() > 10 * lr * 1e-4
