"""Pins for the oracle's statement of the parallel scheme (Section 3.1 / 3.2, Algorithms 1-3):
the P-learner's state sampling, who sees which copy of which network when, and reductions of
the scheme to loops of already pinned single steps.
"""
import numpy as np
import pytest
from scipy import stats

from oracle import pql_oracle as O
from paper_2307_12983_amd import workloads as W

SMALL = W.WORKLOADS["tiny"].replace(name="scheme", obs_dim=6, act_dim=3, num_envs=16, capacity=16 * 12, batch=48,
                                    hidden=(12, 10), index=20)


def _setup(w, v_updates=8, p_updates=4, horizon=1, norm=False, clip=None, prefill=None):
    rng = W.data_rng(w)
    ring = O.ReplayRing(w.rows, w.num_envs, w.obs_dim, w.act_dim)
    nz = O.ObsNormalizer(w.obs_dim, 1e-5) if norm else None
    for row in W.transition_rows(w, rng, prefill or (w.nstep + 1)):
        ring.push(row["obs"], row["act"], row["rew"], row["next_obs"], row["done"])
        if nz is not None:
            nz.update(row["obs"])
    actor, critic = W.init_networks(w)
    L = O.Learner(w.actor_dims(), w.critic_dims(), actor, critic, 5e-3, w.gamma, w.tau, max_grad_norm=clip)
    S = O.ParallelScheme(L, ring, w.nstep, w.batch, w.rng_seed, 0.05, 0.8, normalizer=nz, horizon=horizon,
                         v_updates=v_updates, p_updates=p_updates)
    env_rows = W.transition_rows(w, rng, 64)
    return S, L, ring, env_rows


def _run(S, env_rows, periods):
    ends = []
    for p in range(periods):
        base = p * S.horizon
        S.run_period(lambda period, t, a: env_rows[period * S.horizon + t],
                     [env_rows[base + t]["obs"] for t in range(S.horizon)])
        ends.append(dict(actor=S.L.actor.copy(), critic=S.L.critic.copy()))
    return ends


# ---------------------------------------------------------------- state sampling (Algorithm 2)
def test_state_sampling_covers_every_stored_slot_uniformly():
    ring = O.ReplayRing(5, 8, 2, 1)
    for r in range(7):                                    # wrapped: all 5 rows valid
        ring.push(np.full((8, 2), float(r)), np.zeros((8, 1)), np.zeros(8), np.zeros((8, 2)), np.zeros(8))
    idx, states = O.sample_states(ring, 40000, seed=5, call=0)
    assert idx.min() == 0 and idx.max() == 39
    assert np.array_equal(states, ring.obs[idx])
    chi = stats.chisquare(np.bincount(idx, minlength=40))
    assert chi.pvalue > 1e-3
    # a window of one row: the newest row is a valid draw (it is not for n = 3)
    newest = ring.physical_row(ring.count - 1)
    assert np.any(idx // 8 == newest)
    idx3 = O.sample_indices(ring, 3, 40000, seed=5, call=0)
    assert not np.any(idx3 // 8 == newest)


def test_state_sampling_uses_its_own_generator_stream():
    ring = O.ReplayRing(6, 4, 1, 1)
    for r in range(6):
        ring.push(np.zeros((4, 1)), np.zeros((4, 1)), np.zeros(4), np.zeros((4, 1)), np.zeros(4))
    a, _ = O.sample_states(ring, 256, seed=9, call=3)
    b = O.sample_indices(ring, 1, 256, seed=9, call=3)    # transition sampling, same call number
    assert not np.array_equal(a, b)
    w0, w1, _, _ = O.rng_words(9, 3, 3, np.arange(256, dtype=np.uint64))
    expect = [(((int(hi) << 32) | int(lo)) * 24) >> 64 for lo, hi in zip(w0, w1)]
    assert np.array_equal(a, [ring.physical_row(p // 4) * 4 + p % 4 for p in expect])
    assert not np.array_equal(a, O.sample_states(ring, 256, seed=9, call=4)[0])


def test_partially_filled_ring_only_yields_written_slots():
    ring = O.ReplayRing(10, 4, 1, 1)
    for r in range(3):
        ring.push(np.zeros((4, 1)), np.zeros((4, 1)), np.zeros(4), np.zeros((4, 1)), np.zeros(4))
    idx, _ = O.sample_states(ring, 5000, seed=1, call=0)
    assert idx.min() == 0 and idx.max() == 11


# ---------------------------------------------------------------- who sees what, when
@pytest.mark.parametrize("horizon", [1, 2])
def test_local_copies_lag_by_exactly_one_period(horizon):
    w = SMALL
    S, L, ring, env_rows = _setup(w, horizon=horizon)
    init_actor, init_critic, rows0 = L.actor.copy(), L.critic.copy(), ring.count
    ends = _run(S, env_rows, 4)
    for p, rec in enumerate(S.trace):
        prev_actor = init_actor if p == 0 else ends[p - 1]["actor"]
        prev_critic = init_critic if p == 0 else ends[p - 1]["critic"]
        assert np.array_equal(rec["pi_a"], prev_actor)        # Actor: policy as of the last boundary
        assert np.array_equal(rec["pi_v"], prev_actor)        # V-learner's lagged target policy
        assert np.array_equal(rec["q_p"], prev_critic)        # P-learner's critics
        assert rec["rows"] == rows0 + p * horizon             # data arrives at the boundary
        assert len(rec["v_losses"]) == 8 and len(rec["p_losses"]) == 4
        for t, a in enumerate(rec["actions"]):                # exploration with pi^a, one noise draw per step
            ref = O.actor_act(prev_actor, w.actor_dims(), env_rows[p * horizon + t]["obs"], 0.05, 0.8, w.rng_seed,
                              p * horizon + t)
            assert np.array_equal(a, ref.astype(np.float32))
    # the stored actions are the Actor's, the rest is what the environment returned
    last = ring.physical_row(ring.count - 1) * w.num_envs
    assert np.array_equal(ring.act[last:last + w.num_envs], S.trace[-1]["actions"][-1])
    assert np.array_equal(ring.obs[last:last + w.num_envs], env_rows[4 * horizon - 1]["obs"])
    assert not np.array_equal(ends[0]["actor"], ends[1]["actor"]) and not np.array_equal(ends[0]["critic"], ends[1]["critic"])


def test_parts_of_one_period_do_not_influence_each_other():
    w = SMALL
    full = _setup(w)
    only_v = _setup(w, p_updates=0)
    only_p = _setup(w, v_updates=0)
    e_full, e_v, e_p = _run(full[0], full[3], 2), _run(only_v[0], only_v[3], 2), _run(only_p[0], only_p[3], 2)
    # period 0: every part works on the initial copies, whatever the others do
    assert np.array_equal(e_full[0]["critic"], e_v[0]["critic"])
    assert np.array_equal(e_full[0]["actor"], e_p[0]["actor"])
    assert np.array_equal(full[0].trace[0]["actions"][0], only_v[0].trace[0]["actions"][0])
    # period 1: the exchanged networks matter
    assert not np.array_equal(e_full[1]["critic"], e_v[1]["critic"])
    assert not np.array_equal(e_full[1]["actor"], e_p[1]["actor"])


# ---------------------------------------------------------------- reductions to pinned single steps
def test_value_part_alone_is_the_plain_critic_loop():
    """Without policy updates the scheme is: 8 critic updates + Polyak per period on a ring that
    grows by one Actor step per period, with the (constant) policy as target policy."""
    w = SMALL
    S, L, ring, env_rows = _setup(w, p_updates=0, norm=True, clip=0.5)
    ref_S, ref_L, ref_ring, _ = _setup(w, p_updates=0, norm=True, clip=0.5)
    nz = ref_S.nz
    _run(S, env_rows, 3)
    call = 0
    for p in range(3):
        a = O.actor_act(ref_L.actor, w.actor_dims(), nz.normalize(env_rows[p]["obs"]), 0.05, 0.8, w.rng_seed, p)
        for _ in range(8):
            b = O.gather_nstep(ref_ring, O.sample_indices(ref_ring, w.nstep, w.batch, w.rng_seed, call), w.nstep, w.gamma)
            call += 1
            ref_L.critic_update(O.normalize_batch(b, nz))
            ref_L.soft_update_targets()
        r = env_rows[p]
        ref_ring.push(r["obs"], a.astype(np.float32), r["rew"], r["next_obs"], r["done"])
        nz.update(r["obs"])
    assert np.array_equal(L.critic, ref_L.critic) and np.array_equal(L.critic_target, ref_L.critic_target)
    assert np.array_equal(ring.act, ref_ring.act) and ring.head == ref_ring.head
    assert np.array_equal(S.nz.mean, nz.mean) and S.nz.count == nz.count


def test_policy_part_alone_is_the_plain_policy_loop_on_sampled_states():
    w = SMALL
    S, L, ring, env_rows = _setup(w, v_updates=0)
    _, ref_L, ref_ring, _ = _setup(w, v_updates=0)
    _run(S, env_rows, 3)
    call = 0
    for p in range(3):
        a = O.actor_act(ref_L.actor, w.actor_dims(), env_rows[p]["obs"], 0.05, 0.8, w.rng_seed, p)
        for _ in range(4):
            _, states = O.sample_states(ref_ring, w.batch, w.rng_seed, call)
            call += 1
            ref_L.actor_update(states)
        r = env_rows[p]
        ref_ring.push(r["obs"], a.astype(np.float32), r["rew"], r["next_obs"], r["done"])
    assert np.array_equal(L.actor, ref_L.actor)
    assert np.array_equal(L.critic, ref_L.critic)            # untouched
    assert np.array_equal(ring.act, ref_ring.act)


def test_sac_variant_hands_the_temperature_over_like_the_policy():
    w = SMALL.replace(sac=True)
    rng = W.data_rng(w)
    ring = O.ReplayRing(w.rows, w.num_envs, w.obs_dim, w.act_dim)
    for row in W.transition_rows(w, rng, w.nstep + 1):
        ring.push(row["obs"], row["act"], row["rew"], row["next_obs"], row["done"])
    actor, critic = W.init_networks(w)
    L = O.Learner(w.actor_dims(), w.critic_dims(), actor, critic, 5e-3, w.gamma, w.tau, sac=True,
                  log_alpha=np.log(0.2), target_entropy=-3.0, seed=w.rng_seed)
    S = O.ParallelScheme(L, ring, w.nstep, w.batch, w.rng_seed, 0.05, 0.8)
    env_rows = W.transition_rows(w, rng, 8)
    alphas = [L.log_alpha]
    for p in range(3):
        rec = S.run_period(lambda period, t, a: env_rows[period], [env_rows[p]["obs"]])
        alphas.append(L.log_alpha)
        assert rec["log_alpha_v"] == alphas[p]                 # the V-learner's copy: the value at the last boundary
        # the Actor's exploration is a sample of its policy copy
        ref = O.sac_actor_act(rec["pi_a"], w.actor_dims(), env_rows[p]["obs"], w.rng_seed, p)
        assert np.array_equal(rec["actions"][0], ref.astype(np.float32))
    assert len(set(alphas)) == 4                               # the P-learner moved it in every period
