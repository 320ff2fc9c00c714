"""GPU parity of the concurrent Actor / V-learner / P-learner schedule (Section 3.1, 3.2,
Algorithms 1-3) against the oracle's sequential statement of the same schedule, and bit-equality
of the three-stream run with the single-stream run of the same calls (any missing event between
the streams shows up as a difference).
"""
import sys

import numpy as np
import pytest

from oracle import pql_oracle as O
from paper_2307_12983_amd import workloads as W

from parity_util import (TOL_100_STEPS, TOL_ONE_STEP, assert_params_close, fill_both, oracle_learner,
                         oracle_normalizer, oracle_ring, rel_err)

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    return torch


def cases():
    Wk = W.WORKLOADS
    return {
        "tiny": Wk["tiny"],
        "ragged": Wk["tiny"].replace(name="ragged", obs_dim=13, act_dim=3, num_envs=50, capacity=50 * 11, batch=333,
                                     hidden=(96, 40), index=10),
        "ant_s": Wk["ant"].replace(name="ant_s", num_envs=96, capacity=96 * 13, batch=1000),
        "tiny_defaults": Wk["tiny"].replace(name="tiny_defaults", max_grad_norm=0.5, obs_norm=True, obs_loc=3.0,
                                            obs_scale=2.0, index=13),
        "ragged_dist": Wk["tiny"].replace(name="ragged_dist", obs_dim=13, act_dim=3, num_envs=50, capacity=50 * 11,
                                          batch=333, hidden=(96, 40), index=14, num_atoms=51),
        "ragged_sac": Wk["tiny"].replace(name="ragged_sac", obs_dim=13, act_dim=3, num_envs=50, capacity=50 * 11,
                                         batch=333, hidden=(96, 40), index=15, sac=True),
    }


CASES = cases()


def build(torch, w, concurrent, horizon=1, fold=False):
    from paper_2307_12983_amd.scheme import ParallelSchemeSession
    from paper_2307_12983_amd.session import LearnerSession
    s, ring, nz = LearnerSession(w), oracle_ring(w), oracle_normalizer(w)
    if fold:                # Polyak step and transposed weights carried by the optimiser kernels
        s.fold_followups()
    rng = fill_both(s, ring, w, w.nstep + 1, normalizer=nz)
    env_host = W.transition_rows(w, rng, 6)
    env_dev = [s.to_device(r) for r in env_host]
    ps = ParallelSchemeSession(s, env_dev, horizon=horizon, concurrent=concurrent)
    return s, ps, ring, nz, env_host


@pytest.mark.parametrize("case,horizon,fold", [("tiny", 1, False), ("ragged", 2, False), ("ant_s", 1, False), ("tiny_defaults", 1, False),
                                               ("ragged_dist", 1, False), ("ragged_sac", 1, False), ("ant_s", 1, True),
                                               ("tiny_defaults", 2, True)])
def test_scheme_matches_oracle(torch_cuda, case, horizon, fold):
    torch = torch_cuda
    w = CASES[case]
    periods = 4
    s, ps, ring, nz, env_host = build(torch, w, True, horizon, fold)
    L = oracle_learner(w, s.actor_init, s.critic_init)
    S = O.ParallelScheme(L, ring, w.nstep, w.batch, w.rng_seed, w.sigma_min, w.sigma_max, normalizer=nz, horizon=horizon)
    for p in range(periods):
        say(case, "period", p)
        ps.run_period()
        ps.finish()
        torch.cuda.synchronize()
        base = p * horizon
        rec = S.run_period(lambda period, t, a: env_host[(period * horizon + t) % len(env_host)],
                           [env_host[(base + t) % len(env_host)]["obs"] for t in range(horizon)])
        # actions of this period: produced with pi^a, the policy of the last boundary
        for t in range(horizon):
            e = rel_err(ps.staged_act[p % 2][t].cpu().numpy(), rec["actions"][t])
            assert e <= TOL_ONE_STEP, "period %d step %d actions: %.2e" % (p, t, e)
        # the last batches drawn by both learners: same slots
        assert np.array_equal(s.batch.idx[:w.batch].cpu().numpy(), rec["v_idx"])
        assert np.array_equal(ps.p_idx[:w.batch].cpu().numpy(), rec["p_idx"])
        e_loss = rel_err(s.critic_loss.cpu().numpy(), rec["v_losses"][-1])
        if w.sac:
            out, Jr = s.actor_out.cpu().numpy(), rec["p_losses"][-1]
            e_J = max(abs(out[0] - Jr[0]) / abs(Jr[0]), abs(out[2] - Jr[1]) / abs(Jr[1]))
        else:
            e_J = abs(float(s.actor_loss.cpu()[0]) - rec["p_losses"][-1]) / abs(rec["p_losses"][-1])
        say("  last losses: critic %.2e policy %.2e" % (e_loss, e_J))
        assert e_loss <= TOL_100_STEPS and e_J <= TOL_100_STEPS
    st = s.ctx.get_state()
    assert st[2] == w.nstep + 1 + (periods - 1) * horizon          # the last period's data is still staged
    assert st[3] == 8 * periods and st[7] == 4 * periods and st[4] == periods * horizon
    assert st[5] == 8 * periods and st[6] == 4 * periods
    res = dict(
        critic=assert_params_close(s.critic.cpu().numpy(), L.critic, w.critic_dims(), 2, TOL_100_STEPS, "critic"),
        target=assert_params_close(s.critic_target.cpu().numpy(), L.critic_target, w.critic_dims(), 2, TOL_100_STEPS, "target"),
        actor=assert_params_close(s.actor.cpu().numpy(), L.actor, w.actor_dims(), 1, TOL_100_STEPS, "actor"),
        pi_a=assert_params_close(ps.pi_snap[(periods - 1) % 2].cpu().numpy(), S.pi_a, w.actor_dims(), 1, TOL_100_STEPS, "pi^a"),
        q_p=assert_params_close(ps.q_snap[(periods - 1) % 2].cpu().numpy(), S.q_p, w.critic_dims(), 2, TOL_100_STEPS, "Q^p"))
    if w.sac:
        assert abs(float(s.temperature.cpu()[0]) - L.log_alpha) <= TOL_100_STEPS * abs(L.log_alpha)
        assert abs(float(ps.alpha_snap[(periods - 1) % 2].cpu()[0]) - S.log_alpha_v) <= TOL_100_STEPS * abs(S.log_alpha_v)
    say(case, res)


@pytest.mark.parametrize("case,fold", [("ragged", False), ("ant_s", False), ("tiny_defaults", False), ("ragged_sac", False),
                                       ("ant_s", True), ("ragged", True)])
def test_three_streams_equal_one_stream_bit_for_bit(torch_cuda, case, fold):
    torch = torch_cuda
    w = CASES[case]
    out = []
    for concurrent in (False, True):
        s, ps, _, _, _ = build(torch, w, concurrent, horizon=2, fold=fold)
        for p in range(6):
            ps.run_period()
        ps.finish()
        torch.cuda.synchronize()
        out.append(dict(critic=s.critic.clone(), target=s.critic_target.clone(), actor=s.actor.clone(),
                        c_m=s.c_m.clone(), a_v=s.a_v.clone(), ring_act=s.storage.act.clone(), ring_obs=s.storage.obs.clone(),
                        pi0=ps.pi_snap[0].clone(), q1=ps.q_snap[1].clone(), losses=s.critic_out.clone(),
                        J=s.actor_out.clone(), p_idx=ps.p_idx.clone(), v_idx=s.batch.idx.clone(),
                        stats=None if s.obs_stats is None else s.obs_stats.clone(), state=s.ctx.get_state()))
    a, b = out
    assert a["state"] == b["state"]
    for k in a:
        if k == "state" or a[k] is None:
            continue
        assert torch.equal(a[k], b[k]), "%s differs between the one-stream and the three-stream run" % k
    say(case, "bit-identical over 6 periods; critic moved by", float((a["critic"] - torch.from_numpy(s.critic_init).cuda()).abs().max()))


def test_two_contexts_driven_from_two_threads(torch_cuda):
    """Two learners with their own contexts, buffers and streams, driven from two host threads at the same time
    (ctypes releases the interpreter lock during a call, so the library's calls do overlap), must end where
    the same two learners end when run one after the other: the library keeps nothing per process that one
    context's calls could disturb for another's."""
    import threading
    torch = torch_cuda
    from paper_2307_12983_amd.session import LearnerSession
    shapes = [CASES["ant_s"], CASES["ragged"]]

    def learner(w):
        s = LearnerSession(w)
        for row in W.transition_rows(w, W.data_rng(w), w.nstep + 4):
            s.push(row)
        torch.cuda.synchronize()
        return s

    def run(s, stream, steps=24):
        w = s.w
        with torch.cuda.stream(stream):
            for it in range(steps):
                s.sample(w.batch)
                s.critic_update(w.batch)
                s.soft_update_targets()
                if it % 2 == 1:
                    s.actor_update(None, w.batch)
                    s.sync_lagged_policy()
            stream.synchronize()

    def state(s):
        return [t.clone() for t in (s.critic, s.critic_target, s.actor, s.actor_lag, s.c_m, s.c_v, s.a_m, s.a_v)]

    # one after the other, each on a stream of its own
    ref = []
    for w in shapes:
        s = learner(w)
        run(s, torch.cuda.Stream())
        ref.append(state(s))
    # both at once, one host thread each
    sessions = [learner(w) for w in shapes]
    errors = []

    def worker(s):
        try:
            run(s, torch.cuda.Stream())
        except Exception as e:      # reported by the main thread
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(s,)) for s in sessions]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
        assert not t.is_alive(), "a learner thread did not finish"
    assert not errors, errors
    torch.cuda.synchronize()
    for s, r in zip(sessions, ref):
        for got, want in zip(state(s), r):
            assert torch.equal(got, want)
