"""Shared helpers of the GPU parity tests: run the same seeded inputs through the HIP path
(LearnerSession -> C-ABI) and through the CPU oracle, and compare tensor by tensor."""
from __future__ import annotations

import numpy as np

from oracle import pql_oracle as O
from paper_2307_12983_amd import workloads as W

TOL_ONE_STEP = 1e-4     # max relative error after one step (per tensor, max-norm)
TOL_100_STEPS = 1e-3    # after 100 steps


def rel_err(x, ref):
    """max_i |x_i - ref_i| / max(max_i |ref_i|, 1e-30): the per-tensor max-norm relative error.
    Element-wise relative error is meaningless for gradients that pass through zero."""
    x = np.asarray(x, np.float64).ravel()
    ref = np.asarray(ref, np.float64).ravel()
    assert x.shape == ref.shape
    if x.size == 0:
        return 0.0
    return float(np.max(np.abs(x - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def split_tensors(flat, dims, nets=1):
    """Flat vector(s) -> list of (name, array) per W_l / b_l of each network."""
    flat = np.asarray(flat)
    out, off = [], 0
    for n in range(nets):
        for li, (i, o) in enumerate(dims):
            out.append(("net%d.W%d" % (n, li), flat[off:off + i * o])); off += i * o
            out.append(("net%d.b%d" % (n, li), flat[off:off + o])); off += o
    assert off == flat.size
    return out


def joint_scales(ref, dims, nets):
    """Reference scale of every tensor for the max-norm relative error: max |ref| of the tensor itself,
    except for one-element tensors (the scalar critic's output bias).  There the max-norm rule would
    degenerate to the relative error of a single number, and for the gradient that number is
    sum_b delta_b, which can cancel to orders of magnitude below its terms (and below the fp32 rounding of
    the q_b it is made of).  A bias is the weight of a constant input 1: the one-element tensor is judged
    as that extra row of its layer's weight matrix, i.e. on the scale max(max |W_l|, |b_l|)."""
    tensors = split_tensors(ref, dims, nets)
    scales = []
    for k, (name, r) in enumerate(tensors):
        sc = float(np.max(np.abs(np.asarray(r, np.float64)))) if r.size else 0.0
        if r.size == 1 and ".b" in name:
            sc = max(sc, float(np.max(np.abs(np.asarray(tensors[k - 1][1], np.float64)))))    # W_l precedes b_l
        scales.append(max(sc, 1e-30))
    return scales


def assert_params_close(got, ref, dims, nets, tol, what):
    worst = 0.0
    scales = joint_scales(ref, dims, nets)
    for (name, g), (_, r), sc in zip(split_tensors(got, dims, nets), split_tensors(ref, dims, nets), scales):
        e = float(np.max(np.abs(np.asarray(g, np.float64) - np.asarray(r, np.float64)))) / sc if r.size else 0.0
        worst = max(worst, e)
        assert e <= tol, "%s %s: rel err %.3e > %.1e" % (what, name, e, tol)
    return worst


def assert_first_step_params(theta, theta_ref, g, g_ref, dims, nets, lr, eps, tol, what, from_grad):
    """Parameters after the FIRST Adam step (m = v = 0 before it), where the update is
    -lr * g / (|g| + eps).  That map has slope lr * eps / (|g| + eps)^2, i.e. up to lr / eps = 5e4
    for gradient entries that happen to be ~0: a gradient error dg far inside the fp32 rounding
    of the batch reduction moves such a parameter by up to 2 lr (the sign of the entry), which is more
    than `tol` of the largest weight of a layer.  Entries whose guaranteed bound
    lr * eps * dg / (max(|g| - dg, 0) + eps)^2 (dg = measured max gradient error of the tensor,
    itself required to be within tolerance) stays below half the tolerance must agree with the
    oracle's parameters to `tol`.  For the others the oracle's parameters say nothing about the
    optimiser (they follow a gradient entry that differs in sign or by its own magnitude), so they
    are compared, to the same `tol`, with what the ORACLE's step makes of the gradient the GPU itself
    reports: ``from_grad(g)`` returns those parameters for a flat gradient vector (oracle code:
    adam_step, and soft_update for target networks).  Their gradient entries are covered by the
    gradient comparison; their count is returned.  One-element tensors take their scale from
    joint_scales()."""
    total = exempt_total = 0
    worst = worst_exempt = 0.0
    scales = joint_scales(theta_ref, dims, nets)
    theta_own = from_grad(np.asarray(g, np.float64))
    for (name, t), (_, tr), (_, to), (_, gg), (_, gr), scale in zip(
            split_tensors(theta, dims, nets), split_tensors(theta_ref, dims, nets), split_tensors(theta_own, dims, nets),
            split_tensors(g, dims, nets), split_tensors(g_ref, dims, nets), scales):
        t, tr, to, gg, gr = (np.asarray(x, np.float64) for x in (t, tr, to, gg, gr))
        dg = float(np.max(np.abs(gg - gr)))
        amp = lr * eps * dg / (np.maximum(np.abs(gr) - dg, 0.0) + eps) ** 2
        exempt = amp > 0.5 * tol * scale
        total += t.size
        exempt_total += int(exempt.sum())
        if (~exempt).any():
            e = float(np.abs(t - tr)[~exempt].max()) / scale
            worst = max(worst, e)
            assert e <= tol, "%s %s: rel err %.3e > %.1e" % (what, name, e, tol)
        if exempt.any():
            e = float(np.abs(t - to)[exempt].max()) / scale
            worst_exempt = max(worst_exempt, e)
            assert e <= tol, "%s %s: near-zero-gradient entry: rel err %.3e to the step on the reported gradient" % (what, name, e)
    return dict(rel=worst, near_zero_grad_entries=exempt_total, of=total, rel_there=worst_exempt)


def oracle_ring(w: W.Workload):
    return O.ReplayRing(w.rows, w.num_envs, w.obs_dim, w.act_dim)


def oracle_learner(w: W.Workload, actor, critic):
    return O.Learner(w.actor_dims(), w.critic_dims(), actor, critic, w.lr, w.gamma, w.tau, w.beta1, w.beta2, w.eps,
                     max_grad_norm=(w.max_grad_norm if w.max_grad_norm > 0 else None),
                     v_min=(w.v_min if w.num_atoms >= 2 else None), v_max=(w.v_max if w.num_atoms >= 2 else None),
                     sac=w.sac, log_alpha=float(np.float32(np.log(np.float64(w.init_alpha)))),
                     target_entropy=w.target_entropy, seed=w.rng_seed)


def oracle_normalizer(w: W.Workload):
    return O.ObsNormalizer(w.obs_dim, w.obs_norm_eps) if w.obs_norm else None


def fill_both(sess, ring, w: W.Workload, rows: int, rng=None, normalizer=None):
    """Pushes the same `rows` synthetic Actor steps into the device ring and the oracle ring (and
    the pushed observations into the oracle's running statistics, when given)."""
    rng = rng or W.data_rng(w)
    for row in W.transition_rows(w, rng, rows):
        sess.push(row)
        ring.push(row["obs"], row["act"], row["rew"], row["next_obs"], row["done"])
        if normalizer is not None:
            normalizer.update(row["obs"])
    return rng


def oracle_batch(ring, w: W.Workload, batch_size, call, normalizer=None):
    b = O.gather_nstep(ring, O.sample_indices(ring, w.nstep, batch_size, w.rng_seed, call), w.nstep, w.gamma)
    return b if normalizer is None else O.normalize_batch(b, normalizer)


def batch_to_numpy(batch, B):
    return dict(idx=batch.idx[:B].cpu().numpy(), obs=batch.obs[:B].cpu().numpy(), act=batch.act[:B].cpu().numpy(),
                ret=batch.ret[:B].cpu().numpy(), next_obs=batch.next_obs[:B].cpu().numpy(),
                boot=batch.boot[:B].cpu().numpy())


def assert_batch_matches(got, ref, normalized=False, ring=None, normalizer=None):
    """Copies are bit-exact; standardised observations (normalized=True) are fp32 arithmetic on
    one subtraction and one product per element: 1e-6 of the tensor's largest value, plus - when the
    oracle's `normalizer` is given - what the fp32 rounding of the running mean costs after the
    division by the standard deviation, 4 * 2^-24 |mean_j| / sqrt(var_j + eps) per column (it matters
    when a column's spread is small against its mean, e.g. statistics of two observations).  The n-step
    return is a sum of at most n terms gamma^k r_k that may cancel: it is judged on the scale of its
    terms (the largest |r| stored in `ring`) when that exceeds the largest return of the batch, which
    it does for a batch of one row whose rewards happen to cancel."""
    assert np.array_equal(got["idx"], ref["idx"]), "sampled indices differ"
    for k in ("obs", "act", "next_obs"):
        if normalized and k != "act":
            x, r = np.asarray(got[k], np.float64), np.asarray(ref[k], np.float64)
            if r.size == 0:
                continue
            bound = 1e-6 * max(float(np.max(np.abs(r))), 1e-30) * np.ones(r.shape[1])
            if normalizer is not None:
                bound = bound + 4.0 * 2.0 ** -24 * np.abs(normalizer.mean) / np.sqrt(normalizer.var + normalizer.eps)
            worst = float(np.max(np.abs(x - r) / bound))
            assert worst <= 1.0, "standardised %s: error %.2f times its bound" % (k, worst)
            continue
        assert np.array_equal(got[k], ref[k]), "gathered %s differs (must be bit-exact)" % k
    ret, ret_ref = np.asarray(got["ret"], np.float64), np.asarray(ref["ret"], np.float64)
    if ret_ref.size:
        scale = float(np.max(np.abs(ret_ref)))
        if ring is not None:
            scale = max(scale, float(np.max(np.abs(ring.rew))))
        err = float(np.max(np.abs(ret - ret_ref)))
        assert err <= 1e-6 * max(scale, 1e-30), "n-step return: error %.3e on scale %.3e" % (err, scale)
    assert rel_err(got["boot"], ref["boot"]) <= 1e-6
    assert np.array_equal(got["boot"] == 0.0, ref["boot"] == 0.0)
