"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle on identical
seeded inputs.  Integer / copy work must be bit-exact; floats within the per-tensor max-norm
relative error 1e-4 after one step and 1e-3 after 100 steps.
"""
import sys

import numpy as np
import pytest

from oracle import pql_oracle as O
from paper_2307_12983_amd import workloads as W

from parity_util import (TOL_100_STEPS, TOL_ONE_STEP, assert_batch_matches, assert_first_step_params,
                         assert_params_close, batch_to_numpy, fill_both, oracle_batch, oracle_learner,
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


def make_session(w, **kw):
    from paper_2307_12983_amd.session import LearnerSession
    return LearnerSession(w, **kw)


# Reduced cases: the network shapes of each workload at batch sizes the oracle handles in well
# under a second, chosen so that rows/columns are not multiples of the 32/64/128 tile sizes.
def small_cases():
    Wk = W.WORKLOADS
    return {
        "tiny": Wk["tiny"],
        "ragged": Wk["tiny"].replace(name="ragged", obs_dim=13, act_dim=3, num_envs=50, capacity=50 * 11, batch=333,
                                     hidden=(96, 40), index=10),
        "ant_s": Wk["ant"].replace(name="ant_s", num_envs=96, capacity=96 * 13, batch=1000),
        "humanoid_s": Wk["humanoid"].replace(name="humanoid_s", num_envs=64, capacity=64 * 9, batch=777),
        "shadow_s": Wk["shadow"].replace(name="shadow_s", num_envs=40, capacity=40 * 10, batch=640),
        "scale_s": Wk["scale"].replace(name="scale_s", num_envs=48, capacity=48 * 12, batch=520),
        # shapes that take the row-tile fused kernels (all widths multiples of 32, at most 256) with one
        # and with three hidden layers, odd input widths and a batch that is not a multiple of 32
        "fused_l1": Wk["tiny"].replace(name="fused_l1", obs_dim=37, act_dim=5, num_envs=70, capacity=70 * 9, batch=333,
                                       hidden=(160,), index=11),
        "fused_l3": Wk["tiny"].replace(name="fused_l3", obs_dim=45, act_dim=11, num_envs=33, capacity=33 * 12, batch=451,
                                       hidden=(128, 96, 64), index=12),
        # contraction lengths of the row-tile kernels: several whole 32-chunks plus a short tail (211 = 6 * 32 + 19),
        # a tail only (20), whole chunks only (64, 32), layers narrower than the eight wavefronts' 256 columns
        "fused_wide_in": Wk["tiny"].replace(name="fused_wide_in", obs_dim=211, act_dim=20, num_envs=40, capacity=40 * 10,
                                            batch=300, hidden=(192, 128), index=16),
        "fused_k64": Wk["tiny"].replace(name="fused_k64", obs_dim=64, act_dim=32, num_envs=36, capacity=36 * 9, batch=200,
                                        hidden=(64, 64), index=17),
        # layers too wide for the chained kernels but with enough rows for the row-tile layer kernel (forward
        # and backward data products of the layered path) and the narrow one (policy output, action gradient),
        # single-network launches included: a ragged last row tile (8195 = 256 * 32 + 3, an odd number of row
        # tiles: the 128-column layer pairs row tiles per workgroup and the last pair is half empty), output
        # widths that are no multiple of 32 or 256 (300, 136), contraction lengths with and without a tail
        "layer_tiles": Wk["tiny"].replace(name="layer_tiles", obs_dim=41, act_dim=13, num_envs=40, capacity=40 * 8,
                                          batch=8195, hidden=(300, 136, 128), index=19),
    }


SMALL = small_cases()
ROW_TILE_CASES = ["tiny", "ant_s", "fused_l1", "fused_l3", "fused_wide_in", "fused_k64"]


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["tiny", "ragged", "shadow_s"])
def test_push_ring_contents_bit_exact(torch_cuda, case):
    w = SMALL[case]
    say("case", case, "push 2.5*T rows, T =", w.rows)
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, int(2.5 * w.rows) + 1)
    torch_cuda.cuda.synchronize()
    st = s.ctx.get_state()
    assert st[0] == ring.head and st[1] == ring.count and st[2] == int(2.5 * w.rows) + 1
    for f in ("obs", "act", "rew", "next_obs", "done"):
        assert np.array_equal(getattr(s.storage, f).cpu().numpy(), getattr(ring, f)), f


@pytest.mark.parametrize("case", ["tiny", "ragged", "ant_s", "shadow_s", "scale_s"])
@pytest.mark.parametrize("fill", ["partial", "wrapped"])
def test_sample_nstep_indices_and_gather(torch_cuda, case, fill):
    w = SMALL[case]
    rows = w.nstep + 2 if fill == "partial" else 2 * w.rows + 3
    say("case", case, fill, "rows pushed", rows)
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, rows)
    for call in range(3):
        Bsz = w.batch if call < 2 else 7
        s.sample(Bsz)
        ref = O.gather_nstep(ring, O.sample_indices(ring, w.nstep, Bsz, w.rng_seed, call), w.nstep, w.gamma)
        assert_batch_matches(batch_to_numpy(s.batch, Bsz), ref, ring=ring)
    assert s.ctx.get_state()[3] == 3


def test_gather_with_given_indices_and_degenerate_window(torch_cuda):
    w = SMALL["ragged"]
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, w.nstep)          # exactly one valid start row
    s.sample(64)
    ref_idx = O.sample_indices(ring, w.nstep, 64, w.rng_seed, 0)
    assert np.all(ref_idx // w.num_envs == ring.physical_row(0))
    assert_batch_matches(batch_to_numpy(s.batch, 64), O.gather_nstep(ring, ref_idx, w.nstep, w.gamma), ring=ring)
    idx = np.arange(w.num_envs, dtype=np.int64)[::-1].copy()
    s.gather(torch_cuda.from_numpy(idx).cuda())
    got = batch_to_numpy(s.batch, idx.size)
    got["idx"] = idx
    assert_batch_matches(got, O.gather_nstep(ring, idx, w.nstep, w.gamma), ring=ring)
    assert s.ctx.get_state()[3] == 1        # gather does not advance the sample counter


def test_sample_errors_leave_state_unchanged(torch_cuda):
    from paper_2307_12983_amd.binding import PqlError
    w = SMALL["tiny"]
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, w.nstep - 1)
    before = s.ctx.get_state()
    with pytest.raises(PqlError) as e:
        s.sample(16)
    assert e.value.code == -3
    with pytest.raises(PqlError) as e:
        s.ctx.pql_sample_nstep(s.storage, s.max_batch + 1, s.batch)
    assert e.value.code == -4
    assert s.ctx.get_state() == before


# ---------------------------------------------------------------------------------------------
def test_soft_update_pins_and_values(torch_cuda):
    torch = torch_cuda
    s = make_session(SMALL["tiny"])
    g = torch.Generator(device="cpu").manual_seed(0)
    for n in (1, 3, 4, 1023, 4096 + 5, 300001):
        src = torch.randn(n + 1, generator=g).cuda()
        dst = torch.randn(n + 1, generator=g).cuda()
        for off in (0, 1):                   # 16-byte aligned and unaligned views
            a, b = src[off:off + n], dst[off:off + n].clone()
            b0 = b.clone()
            s.ctx.pql_soft_update(a, b, n, 1.0)
            assert torch.equal(a, b)
            b = b0.clone()
            s.ctx.pql_soft_update(a, b, n, 0.0)
            assert torch.equal(b, b0)
            b = b0.clone()
            s.ctx.pql_soft_update(a, b, n, 0.05)
            ref = O.soft_update(a.cpu().numpy(), b0.cpu().numpy(), float(np.float32(0.05)))
            assert rel_err(b.cpu().numpy(), ref) <= 1e-6


def test_adam_step_on_oracle_gradients(torch_cuda):
    """The Adam kernel in isolation, fed gradients that do not come from the GPU: several steps
    with gradients spanning ten orders of magnitude (and exact zeros) against the oracle."""
    torch = torch_cuda
    s = make_session(SMALL["tiny"])
    rng = np.random.default_rng(3)
    n = 70001
    theta0 = rng.standard_normal(n).astype(np.float32)
    theta, m, v = torch.from_numpy(theta0).cuda(), torch.zeros(n).cuda(), torch.zeros(n).cuda()
    rt, rm, rv = theta0.astype(np.float64), np.zeros(n), np.zeros(n)
    opt = s.opt
    for t in range(1, 6):
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-10, 1, size=n)).astype(np.float32)
        g[::97] = 0.0
        s.ctx.pql_adam_step(theta, torch.from_numpy(g).cuda(), m, v, n, opt, t)
        rt, rm, rv = O.adam_step(rt, g.astype(np.float64), rm, rv, t, opt.lr, opt.beta1, opt.beta2, opt.eps)
        # fp32 storage rounding of theta (half an ulp per step) plus a 1e-5 share of the largest
        # possible update (lr)
        assert np.all(np.abs(theta.cpu().numpy() - rt) <= t * 1e-7 * np.abs(rt) + 1e-5 * opt.lr)
        assert rel_err(m.cpu().numpy(), rm) <= 1e-6 and rel_err(v.cpu().numpy(), rv) <= 1e-6
    assert rel_err(theta.cpu().numpy(), rt) <= 1e-6


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", list(small_cases()))
def test_actor_act_matches_oracle(torch_cuda, case):
    torch = torch_cuda
    w = SMALL[case]
    s = make_session(w)
    rng = np.random.default_rng(7)
    # (the last call of layer_tiles is large enough for the row-tile layer kernels, noise epilogue included)
    for call, num in enumerate((w.num_envs, 1, min(s.max_batch, 333)) + ((s.max_batch,) if case == "layer_tiles" else ())):
        obs = rng.standard_normal((num, w.obs_dim), dtype=np.float32)
        got = s.act(torch.from_numpy(obs).cuda(), 0.05, 0.8).cpu().numpy()
        ref = O.actor_act(s.actor_init, w.actor_dims(), obs, float(np.float32(0.05)), float(np.float32(0.8)),
                          w.rng_seed, call)
        e = rel_err(got, ref)
        say(case, "act call", call, "num", num, "rel err %.2e" % e)
        assert e <= TOL_ONE_STEP and got.min() >= -1.0 and got.max() <= 1.0
    obs = rng.standard_normal((w.num_envs, w.obs_dim), dtype=np.float32)
    got = s.act(torch.from_numpy(obs).cuda(), 0.0, 0.0).cpu().numpy()
    assert rel_err(got, O.actor_forward(s.actor_init, w.actor_dims(), obs)) <= TOL_ONE_STEP


@pytest.mark.parametrize("name", ["ant", "humanoid", "scale"])
def test_actor_act_at_the_workloads_own_num_envs(torch_cuda, name):
    """The Actor step at the number of environments each workload names (4096 / 16384 / 32768: the
    launch shapes the benchmark times), with the mixed noise scales of Section 3.3 (sigma_i from 0.05
    to 0.8, linear in the environment index): two calls (two call numbers of the generator), then
    sigma = 0, which must give the deterministic policy."""
    torch = torch_cuda
    w = W.WORKLOADS[name]
    s = make_session(w)
    rng = np.random.default_rng(11)
    lo, hi = float(np.float32(0.05)), float(np.float32(0.8))
    for call in range(2):
        obs = rng.standard_normal((w.num_envs, w.obs_dim), dtype=np.float32)
        s.ctx.pql_profile_begin(64)
        got = s.act(torch.from_numpy(obs).cuda(), lo, hi).cpu().numpy()
        names = {k["name"] for k in s.ctx.pql_profile_end()}
        ref = O.actor_act(s.actor_init, w.actor_dims(), obs, lo, hi, w.rng_seed, call)
        e = rel_err(got, ref)
        # per environment: the noise scale is the one of ITS index (a wrong sigma_i or element counter shows in
        # the rows it belongs to, whatever the tensor-wide maximum is)
        row_err = np.abs(got.astype(np.float64) - ref).max(axis=1)
        say(name, "act call", call, "N", w.num_envs, "rel err %.2e" % e, "worst row", int(row_err.argmax()), sorted(names))
        assert e <= TOL_ONE_STEP and row_err.max() <= TOL_ONE_STEP and got.min() >= -1.0 and got.max() <= 1.0
        if name == "ant":
            assert names == {"fused_act16_kernel"}           # 4096 environments: 256 tiles of 16 rows
        elif name == "humanoid":
            assert names == {"chain_act_kernel"}
        else:
            assert {"layer_rowtile_kernel", "narrow_rowtile_kernel"} <= names
    sig = O.exploration_sigma(w.num_envs, lo, hi)
    assert sig[0] == lo and abs(sig[-1] - hi) <= 1e-15 and sig.shape == (w.num_envs,)
    obs = rng.standard_normal((w.num_envs, w.obs_dim), dtype=np.float32)
    got = s.act(torch.from_numpy(obs).cuda(), 0.0, 0.0).cpu().numpy()
    assert rel_err(got, O.actor_forward(s.actor_init, w.actor_dims(), obs)) <= TOL_ONE_STEP
    assert s.ctx.get_state()[4] == 3


@pytest.mark.parametrize("case,num,kernel", [("ant_s", 4096, "fused_act16_kernel"), ("ant_s", 4097, "fused_act_kernel"),
                                             ("ant_s", 6001, "fused_act_kernel"), ("fused_l3", 4000, "fused_act16_kernel"),
                                             ("fused_wide_in", 2049, "fused_act16_kernel"), ("fused_k64", 4099, "fused_act_kernel")])
def test_actor_act_tile_heights(torch_cuda, case, num, kernel):
    """Up to 4096 environments the Actor step of narrow networks runs on 16-row tiles, above on 32-row tiles:
    both sides of the switch, ragged last tiles, odd input widths (45, 211), 32 action columns (fused_k64),
    with mixed noise scales and, for the second call, standardised observations."""
    torch = torch_cuda
    w = SMALL[case].replace(batch=num, obs_norm=True, obs_loc=1.0, obs_scale=2.0)
    s, nz = make_session(w), oracle_normalizer(w)
    row = W.transition_rows(w, W.data_rng(w), 1)[0]
    rng = np.random.default_rng(13)
    lo, hi = float(np.float32(0.05)), float(np.float32(0.8))
    for call in range(2):
        if call == 1:                      # statistics of one pushed row: the second call standardises with them
            s.push(row)
            nz.update(row["obs"])
        obs = (1.0 + 2.0 * rng.standard_normal((num, w.obs_dim))).astype(np.float32)
        s.ctx.pql_profile_begin(16)
        got = s.act(torch.from_numpy(obs).cuda(), lo, hi).cpu().numpy()
        names = {k["name"] for k in s.ctx.pql_profile_end()}
        ref = O.actor_act(s.actor_init, w.actor_dims(), nz.normalize(obs), lo, hi, w.rng_seed, call)
        err = np.abs(got.astype(np.float64) - ref).max()
        say(case, "num", num, "call", call, sorted(names), "max abs err %.2e" % err)
        assert names == {kernel}
        assert err <= TOL_ONE_STEP and np.abs(got).max() <= 1.0


# ---------------------------------------------------------------------------------------------
def one_step(torch, w, rows, check_all=True):
    """One sample + critic update + Polyak + policy update + sync on both sides.  The workload's
    switches decide whether batches are standardised and gradients clipped (Table B.1)."""
    s, ring, nz = make_session(w), oracle_ring(w), oracle_normalizer(w)
    fill_both(s, ring, w, rows, normalizer=nz)
    L = oracle_learner(w, s.actor_init, s.critic_init)
    Bsz = w.batch
    s.sample(Bsz)
    batch = oracle_batch(ring, w, Bsz, 0, nz)
    assert_batch_matches(batch_to_numpy(s.batch, Bsz), batch, normalized=nz is not None, ring=ring, normalizer=nz)
    # critic update
    s.critic_update(Bsz)
    losses, g = L.critic_update(batch)
    res = {}
    res["loss"] = rel_err(s.critic_loss.cpu().numpy(), losses)
    if w.max_grad_norm > 0:
        res["c_norm"] = abs(float(s.critic_grad_norm.cpu()[0]) - L.critic_grad_norm) / L.critic_grad_norm
        res["c_clipped"] = L.critic_grad_norm > w.max_grad_norm
        assert res["c_norm"] <= 1e-5
    else:
        assert float(s.critic_grad_norm.cpu()[0]) == 0.0
    res["grad"] = assert_params_close(s.c_g.cpu().numpy(), g, w.critic_dims(), 2, TOL_ONE_STEP, "critic grad")
    c0 = np.asarray(s.critic_init, np.float64)

    def critic_from(gg):        # the oracle's first step on a given gradient
        return O.adam_step(c0, gg, 0.0, 0.0, 1, w.lr, w.beta1, w.beta2, w.eps)[0]

    res["theta"] = assert_first_step_params(s.critic.cpu().numpy(), L.critic, s.c_g.cpu().numpy(), g, w.critic_dims(), 2,
                                            w.lr, w.eps, TOL_ONE_STEP, "critic params", critic_from)
    res["m"] = assert_params_close(s.c_m.cpu().numpy(), L.c_m, w.critic_dims(), 2, TOL_ONE_STEP, "critic adam m")
    res["v"] = assert_params_close(s.c_v.cpu().numpy(), L.c_v, w.critic_dims(), 2, TOL_ONE_STEP, "critic adam v")
    assert res["loss"] <= TOL_ONE_STEP
    # Polyak
    s.soft_update_targets()
    L.soft_update_targets()
    # theta' = tau * theta + (1 - tau) * theta' is linear in theta: the target inherits tau times the deviation
    # of each parameter, so the near-zero-gradient entries of the first Adam step get the same treatment with
    # lr * tau in place of lr (tau * 2 lr is NOT below 1e-4 of the largest weight of a wide layer); the targets
    # start as copies of the critics
    res["target"] = assert_first_step_params(s.critic_target.cpu().numpy(), L.critic_target, s.c_g.cpu().numpy(), g,
                                             w.critic_dims(), 2, w.lr * w.tau, w.eps, TOL_ONE_STEP, "critic target",
                                             lambda gg: O.soft_update(critic_from(gg), c0, w.tau))
    # policy update on the sampled states, then hard sync of the lagged policy
    s.actor_update(None, Bsz)
    J, ga = L.actor_update(batch["obs"])
    if w.sac:       # J = Q term + entropy term, reported separately; then the temperature step
        out = s.actor_out.cpu().numpy().astype(np.float64)
        res["J"] = max(abs(out[0] - J[0]) / abs(J[0]), abs(out[2] - J[1]) / abs(J[1]), abs(out[3] - L.mean_logp) / abs(L.mean_logp))
        res["log_alpha"] = abs(float(s.temperature.cpu()[0]) - L.log_alpha)
        assert res["log_alpha"] <= TOL_ONE_STEP * abs(L.log_alpha)
        assert abs(float(s.temperature.cpu()[1]) - L.al_m) <= TOL_ONE_STEP * abs(L.al_m)
    else:
        res["J"] = abs(float(s.actor_loss.cpu().numpy()[0]) - J) / max(abs(J), 1e-30)
    if w.max_grad_norm > 0:
        res["a_norm"] = abs(float(s.actor_grad_norm.cpu()[0]) - L.actor_grad_norm) / L.actor_grad_norm
        res["a_clipped"] = L.actor_grad_norm > w.max_grad_norm
        assert res["a_norm"] <= 1e-5
    else:
        assert float(s.actor_grad_norm.cpu()[0]) == 0.0
    res["a_grad"] = assert_params_close(s.a_g.cpu().numpy(), ga, w.actor_dims(), 1, TOL_ONE_STEP, "actor grad")
    a0 = np.asarray(s.actor_init, np.float64)
    res["a_theta"] = assert_first_step_params(s.actor.cpu().numpy(), L.actor, s.a_g.cpu().numpy(), ga, w.actor_dims(), 1,
                                              w.lr, w.eps, TOL_ONE_STEP, "actor params",
                                              lambda gg: O.adam_step(a0, gg, 0.0, 0.0, 1, w.lr, w.beta1, w.beta2, w.eps)[0])
    assert res["J"] <= TOL_ONE_STEP
    s.sync_lagged_policy()
    assert torch.equal(s.actor, s.actor_lag)
    st = s.ctx.get_state()
    assert st[5] == 1 and st[6] == 1
    return res


@pytest.mark.parametrize("case", list(SMALL))
def test_one_update_small_cases(torch_cuda, case):
    w = SMALL[case]
    say("case", case, "B", w.batch, "hidden", w.hidden)
    res = one_step(torch_cuda, w, min(w.rows, w.nstep + 4))
    say(case, res)


def workspace_rows(s, what, B):
    """y (0), Q_1 (1) or Q_2 (2) of the last update, read from the workspace at the offset the library names."""
    off = s.ctx.workspace_view(what)
    assert off % 4 == 0
    return s.workspace[off // 4: off // 4 + B].cpu().numpy()


@pytest.mark.parametrize("case,Bsz", [("ant_s", 1000), ("humanoid_s", 1200), ("layer_tiles", 8195)])
def test_td_target_and_q_values_row_by_row(torch_cuda, case, Bsz):
    """Algorithm 3's target y_b and both critics' Q_i(s_b, a_b), and Algorithm 2's Q_i(s_b, pi(s_b)), compared
    row by row with the oracle (the update tests see them only through batch means and weighted sums):
    the row-tile kernels (ant_s), the per-layer path with the grouped GEMMs (humanoid_s) and with the
    row-tile layer kernels (layer_tiles)."""
    w = SMALL[case].replace(batch=Bsz, done_p=0.05)        # enough terminations for some windows to hold one
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, min(w.rows, w.nstep + 4))
    s.sample(Bsz)
    batch = oracle_batch(ring, w, Bsz, 0)
    critic0 = s.critic.cpu().numpy().copy()
    s.critic_update(Bsz)
    y_ref = O.td_target(batch, s.actor_init, s.critic_init, w.actor_dims(), w.critic_dims())
    y = workspace_rows(s, 0, Bsz)
    q_ref = [O.critic_forward(p, w.critic_dims(), batch["obs"], batch["act"]) for p in O.split_twin(critic0)]
    q = [workspace_rows(s, 1 + i, Bsz) for i in range(2)]
    errs = dict(y=rel_err(y, y_ref), q1=rel_err(q[0], q_ref[0]), q2=rel_err(q[1], q_ref[1]))
    # rows whose window holds a termination: the target is the reward sum alone
    term = batch["boot"] == 0.0
    assert term.any() and not term.all()
    assert np.array_equal(y[term], s.batch.ret[:Bsz].cpu().numpy()[term])
    s.actor_update(None, Bsz)
    critic1 = s.critic.cpu().numpy()
    a_pi = O.actor_forward(s.actor_init, w.actor_dims(), batch["obs"])
    qp_ref = [O.critic_forward(p, w.critic_dims(), batch["obs"], a_pi) for p in O.split_twin(critic1)]
    qp = [workspace_rows(s, 1 + i, Bsz) for i in range(2)]
    errs.update(qpi1=rel_err(qp[0], qp_ref[0]), qpi2=rel_err(qp[1], qp_ref[1]))
    say(case, "B", Bsz, {k: "%.2e" % v for k, v in errs.items()}, "terminal rows", int(term.sum()))
    assert max(errs.values()) <= TOL_ONE_STEP


def test_cancelling_output_bias_gradient(torch_cuda):
    """A fixed case in which the scalar critic's output-bias gradient sum_b delta_b cancels to 1e-4 of the
    largest gradient entry (found by a sweep over random shapes): its relative error as a single number was
    1e-3 with an absolute error of 3e-8.  The one-element rule of parity_util.joint_scales judges it on the
    scale of its layer, and here the sum is also held to what its conditioning allows:
    |error| <= 1e-6 * sum_b |delta_b|."""
    w = W.WORKLOADS["tiny"].replace(name="cancel", obs_dim=82, act_dim=16, num_envs=46, capacity=414, batch=100,
                                    hidden=(128, 128, 192, 64), index=108, nstep=1)
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, min(w.rows, w.nstep + 3))
    L = oracle_learner(w, s.actor_init, s.critic_init)
    s.sample(w.batch)
    batch = oracle_batch(ring, w, w.batch, 0)
    assert_batch_matches(batch_to_numpy(s.batch, w.batch), batch, ring=ring)
    y = O.td_target(batch, s.actor_init, s.critic_init, w.actor_dims(), w.critic_dims())
    s.critic_update(w.batch)
    losses, g = L.critic_update(batch)
    got = s.c_g.cpu().numpy().astype(np.float64)
    Pc = g.size // 2
    for i, p in enumerate(O.split_twin(s.critic_init)):
        delta = 2.0 * (O.critic_forward(p, w.critic_dims(), batch["obs"], batch["act"]) - y) / w.batch
        ref_b = g[(i + 1) * Pc - 1]
        assert abs(ref_b - delta.sum()) <= 1e-12 * np.abs(delta).sum()
        err = abs(got[(i + 1) * Pc - 1] - ref_b)
        say("critic", i, "db_out", ref_b, "sum |delta|", np.abs(delta).sum(), "abs err %.2e" % err,
            "as a single number %.2e" % (err / abs(ref_b)), "max |g| %.3f" % np.abs(g[i * Pc:(i + 1) * Pc]).max())
        assert err <= 1e-6 * np.abs(delta).sum()
    assert rel_err(s.critic_loss.cpu().numpy(), losses) <= TOL_ONE_STEP
    assert_params_close(got, g, w.critic_dims(), 2, TOL_ONE_STEP, "critic grad")


SWEEP_FINDS = {
    # a batch of one row whose three rewards nearly cancel: the n-step return as a single number missed 1e-6
    # (it is judged on the scale of its terms, parity_util.assert_batch_matches)
    "cancelling_return": dict(obs_dim=117, act_dim=32, num_envs=40, capacity=480, batch=1, hidden=(320, 512, 40),
                              index=62, nstep=3, num_atoms=51, v_min=-2.0, v_max=3.0),
    # a batch of one row (the gradient is an outer product): 0.54 % of the critics' entries have a gradient so
    # close to zero that the first Adam step follows its rounding; they are held to the oracle's step on the
    # gradient the GPU reports (parity_util.assert_first_step_params)
    "many_near_zero_gradients": dict(obs_dim=36, act_dim=2, num_envs=51, capacity=357, batch=1, hidden=(32, 128),
                                     index=91, nstep=1, num_atoms=51, v_min=-2.0, v_max=3.0),
    "near_zero_gradients_batch_512": dict(obs_dim=158, act_dim=31, num_envs=23, capacity=23 * 9, batch=512, hidden=(128,),
                                          index=75, nstep=3),
}


@pytest.mark.parametrize("case", list(SWEEP_FINDS))
def test_cases_found_by_sweeps_over_random_shapes(torch_cuda, case):
    """Fixed configurations on which an earlier form of a comparison rule failed although the results were
    right (sweeps over seeded random shapes; see the rules named in SWEEP_FINDS)."""
    w = W.WORKLOADS["tiny"].replace(name=case, **SWEEP_FINDS[case])
    res = one_step(torch_cuda, w, min(w.rows, w.nstep + 3))
    say(case, {k: v for k, v in res.items() if isinstance(v, dict)})
    if case == "many_near_zero_gradients":
        assert res["theta"]["near_zero_grad_entries"] > 0.003 * res["theta"]["of"]      # the case still is what it was found as


@pytest.mark.parametrize("name", ["ant", "humanoid", "shadow", "scale"])
def test_one_update_full_size(torch_cuda, name):
    """Full batch and network sizes of each workload.  The ring keeps its full number of rows
    but only n + 8 of them are filled, which bounds host memory and generation time."""
    w = W.WORKLOADS[name]
    say("workload", name, "B", w.batch, "hidden", w.hidden, "rows filled", w.nstep + 8)
    res = one_step(torch_cuda, w, w.nstep + 8)
    say(name, res)


# ---------------------------------------------------------------------------------------------
# Networks with a layer of 512 columns at batches of at least 4096 rows: the row-tile chain kernels (one launch
# per learner step, the networks pass through the tile one after the other, 512-column layers as two halves)
def chain_cases():
    t = W.WORKLOADS["tiny"]
    return {
        # the humanoid-shaped networks, a ragged last row tile (4100 = 128 * 32 + 4)
        "chain_humanoid": W.WORKLOADS["humanoid"].replace(name="chain_humanoid", num_envs=64, capacity=64 * 9, batch=4100),
        # two 512-column layers in a row (the widest pair of tiles), a wide observation with a short tail chunk
        "chain_shadow": W.WORKLOADS["shadow"].replace(name="chain_shadow", num_envs=40, capacity=40 * 10, batch=4097),
        # two hidden layers (the last one, at most 256 wide, is the scalar heads' input); the most action columns
        "chain_l2": t.replace(name="chain_l2", obs_dim=41, act_dim=32, num_envs=50, capacity=50 * 8, batch=4128,
                              hidden=(512, 96), index=41),
        # a narrow layer before a wide one, four layers (tiles alternate twice), one action column
        "chain_l4": t.replace(name="chain_l4", obs_dim=77, act_dim=1, num_envs=33, capacity=33 * 9, batch=4500,
                              hidden=(64, 512, 32, 256), index=42, nstep=2),
    }


CHAIN = chain_cases()


@pytest.mark.parametrize("case", list(CHAIN))
def test_one_update_chain_kernels(torch_cuda, case):
    w = CHAIN[case]
    say("case", case, "B", w.batch, "hidden", w.hidden)
    s = make_session(w)
    for row in W.transition_rows(w, W.data_rng(w), w.nstep + 2):
        s.push(row)
    s.sample(w.batch)
    s.ctx.pql_profile_begin(256)
    s.critic_update(w.batch)
    s.actor_update(None, w.batch)
    s.act(s.batch.obs[:w.batch])
    torch_cuda.cuda.synchronize()
    names = {k["name"] for k in s.ctx.pql_profile_end()}
    say(case, sorted(names))
    assert {"chain_critic_kernel", "chain_policy_kernel", "chain_act_kernel"} <= names
    assert not any(n.startswith(("gemm_grouped_n", "layer_rowtile", "narrow_rowtile", "head_kernel")) for n in names)
    res = one_step(torch_cuda, w, min(w.rows, w.nstep + 4))
    say(case, res)


@pytest.mark.parametrize("case", ["chain_humanoid", "chain_l4"])
def test_chain_kernels_row_by_row_and_actor_step(torch_cuda, case):
    """y_b, Q_i(s_b, a_b) and Q_i(s_b, pi(s_b)) of the chain kernels row by row, and the Actor step at a number
    of environments that takes the chain kernel (two call numbers, then sigma = 0)."""
    torch = torch_cuda
    w = CHAIN[case].replace(done_p=0.05)
    Bsz = w.batch
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, min(w.rows, w.nstep + 4))
    s.sample(Bsz)
    batch = oracle_batch(ring, w, Bsz, 0)
    s.critic_update(Bsz)
    y = workspace_rows(s, 0, Bsz)
    q = [workspace_rows(s, 1 + i, Bsz) for i in range(2)]
    y_ref = O.td_target(batch, s.actor_init, s.critic_init, w.actor_dims(), w.critic_dims())
    q_ref = [O.critic_forward(p, w.critic_dims(), batch["obs"], batch["act"]) for p in O.split_twin(s.critic_init)]
    errs = dict(y=rel_err(y, y_ref), q1=rel_err(q[0], q_ref[0]), q2=rel_err(q[1], q_ref[1]))
    term = batch["boot"] == 0.0
    assert term.any() and np.array_equal(y[term], s.batch.ret[:Bsz].cpu().numpy()[term])
    critic1 = s.critic.cpu().numpy()
    s.actor_update(None, Bsz)
    a_pi = O.actor_forward(s.actor_init, w.actor_dims(), batch["obs"])
    qp_ref = [O.critic_forward(p, w.critic_dims(), batch["obs"], a_pi) for p in O.split_twin(critic1)]
    qp = [workspace_rows(s, 1 + i, Bsz) for i in range(2)]
    errs.update(qpi1=rel_err(qp[0], qp_ref[0]), qpi2=rel_err(qp[1], qp_ref[1]))
    say(case, {k: "%.2e" % v for k, v in errs.items()}, "terminal rows", int(term.sum()))
    assert max(errs.values()) <= TOL_ONE_STEP
    rng = np.random.default_rng(5)
    lo, hi = float(np.float32(0.05)), float(np.float32(0.8))
    a0 = s.actor.cpu().numpy()
    for call in range(2):
        obs = rng.standard_normal((Bsz, w.obs_dim), dtype=np.float32)
        got = s.act(torch.from_numpy(obs).cuda(), lo, hi).cpu().numpy()
        ref = O.actor_act(a0, w.actor_dims(), obs, lo, hi, w.rng_seed, call)
        assert np.abs(got - ref).max() <= TOL_ONE_STEP and np.abs(got).max() <= 1.0
    got = s.act(torch.from_numpy(obs).cuda(), 0.0, 0.0).cpu().numpy()
    assert rel_err(got, O.actor_forward(a0, w.actor_dims(), obs)) <= TOL_ONE_STEP


# ---------------------------------------------------------------------------------------------
def many_steps(torch, w, rows, steps, actor_every=0, must_run=(), must_not_run=(), fold=False):
    """`must_run` / `must_not_run`: kernels that the library's own per-launch profile must / must not name
    during the first iteration that holds every kind of update.  `fold`: the Polyak step, the policy copy
    and the transposes ride on the optimiser kernels (LearnerSession.fold_followups)."""
    s, ring, nz = make_session(w), oracle_ring(w), oracle_normalizer(w)
    fill_both(s, ring, w, rows, normalizer=nz)
    if fold:
        s.fold_followups()
    L = oracle_learner(w, s.actor_init, s.critic_init)
    Bsz = w.batch
    worst_loss = 0.0
    prof_it = (actor_every - 1) if actor_every else 0
    for it in range(steps):
        if must_run and it == prof_it:
            s.ctx.pql_profile_begin(512)
        s.sample(Bsz)
        s.critic_update(Bsz)
        s.soft_update_targets()
        batch = oracle_batch(ring, w, Bsz, it, nz)
        losses, _ = L.critic_update(batch)
        L.soft_update_targets()
        if actor_every and (it + 1) % actor_every == 0:
            s.actor_update(None, Bsz)
            s.sync_lagged_policy()
            L.actor_update(batch["obs"])
            L.sync_lagged_policy()
        if must_run and it == prof_it:
            torch.cuda.synchronize()
            ran = {k["name"]: k["launches"] for k in s.ctx.pql_profile_end()}
            say("  kernels of iteration", it, ran)
            assert set(must_run) <= set(ran), "expected kernels did not run: %s" % sorted(set(must_run) - set(ran))
            assert not (set(must_not_run) & set(ran)), "kernels that should be gone: %s" % sorted(set(must_not_run) & set(ran))
        if it % 10 == 9 or it == steps - 1:
            e = rel_err(s.critic_loss.cpu().numpy(), losses)
            worst_loss = max(worst_loss, e)
            say("  step", it + 1, "loss", losses, "rel err %.2e" % e)
    assert np.array_equal(s.batch.idx[:Bsz].cpu().numpy(), batch["idx"])
    res = dict(loss=worst_loss)
    res["theta"] = assert_params_close(s.critic.cpu().numpy(), L.critic, w.critic_dims(), 2, TOL_100_STEPS, "critic params")
    res["target"] = assert_params_close(s.critic_target.cpu().numpy(), L.critic_target, w.critic_dims(), 2, TOL_100_STEPS, "critic target")
    res["actor"] = assert_params_close(s.actor.cpu().numpy(), L.actor, w.actor_dims(), 1, TOL_100_STEPS, "actor params")
    assert worst_loss <= TOL_100_STEPS
    if w.sac:
        res["log_alpha"] = abs(float(s.temperature.cpu()[0]) - L.log_alpha) / abs(L.log_alpha)
        assert res["log_alpha"] <= TOL_100_STEPS
    return res


def test_100_updates_tiny(torch_cuda):
    w = W.WORKLOADS["tiny"]
    res = many_steps(torch_cuda, w, w.rows, 100, actor_every=2)
    say("tiny 100 steps", res)


def test_100_critic_10_actor_updates_ant_full_batch(torch_cuda):
    w = W.WORKLOADS["ant"]
    res = many_steps(torch_cuda, w, w.nstep + 8, 100, actor_every=10)
    say("ant 100 steps", res)


@pytest.mark.parametrize("name", ["humanoid", "shadow", "scale"])
def test_100_updates_reduced_batch(torch_cuda, name):
    """100 critic updates with the full network shapes at batch 1024 (the full-batch float64
    oracle would need minutes per workload; full batch is covered by the one-step test)."""
    w = W.WORKLOADS[name].replace(num_envs=256, capacity=256 * 16, batch=1024)
    res = many_steps(torch_cuda, w, w.rows, 100, actor_every=0)
    say(name, "100 steps", res)


@pytest.mark.parametrize("name,Bsz,actor_every,steps", [("humanoid", 8192, 10, 100), ("shadow", 16384, 0, 100),
                                                        ("scale", 8192, 0, 100), ("scale", 32768, 0, 16)])
def test_100_updates_through_the_row_tile_layer_kernels(torch_cuda, name, Bsz, actor_every, steps):
    """Many critic updates with the networks of the large workloads on the kernels the benchmark runs them on:
    humanoid (batch 8192, with a policy update every 10th step, so the policy path's launches are covered too)
    and shadow (batch 16384) at their own batch sizes for 100 steps; scale for 100 steps at batch 8192 instead of
    32768 (the float64 oracle needs 0.8 s per update there and 3 s at 32768) and for 16 steps at its own batch.
    Every launch of the critic update has at least the 256 row tiles from which the row-tile kernels are used;
    the library's per-launch profile must name them.  (The ring is shortened to 1024 environments: the
    full rings are covered by the one-step tests.)"""
    base = W.WORKLOADS[name]
    w = base.replace(num_envs=1024, capacity=1024 * (base.nstep + 9), batch=Bsz)
    need = (("chain_critic_kernel",) + (("chain_policy_kernel",) if actor_every else ()) if name != "scale" else
            ("layer_rowtile_kernel", "narrow_rowtile_kernel")) + ("gemm_tn_stream_kernel",)
    res = many_steps(torch_cuda, w, w.rows, steps, actor_every=actor_every, must_run=need)
    say(name, "batch", Bsz, steps, "steps", res)


def test_100_updates_row_tile_layers(torch_cuda):
    """100 critic and 20 policy updates at a batch and widths that take the row-tile layer kernel
    (forward and backward data products of the layered path)."""
    w = SMALL["layer_tiles"]
    res = many_steps(torch_cuda, w, w.rows, 100, actor_every=5)
    say("layer_tiles 100 steps", res)


# ---------------------------------------------------------------------------------------------
# Table B.1 defaults left off in the five workloads: observation standardisation and gradient clipping
def paper_defaults(w, bound=0.5):
    return w.replace(max_grad_norm=float(np.float32(bound)), obs_norm=True, obs_loc=3.0, obs_scale=2.0)


@pytest.mark.parametrize("case", ["tiny", "ragged", "fused_l3", "shadow_s"])
def test_running_observation_statistics(torch_cuda, case):
    """Count exact; mean and sum of squared deviations are double-precision sums in a different
    association than the oracle's (chunks of 64 rows): 1e-12 / 1e-10; the fp32 mean and
    1/sqrt(var + eps) that the kernels read: fp32 rounding of the oracle's values."""
    w = paper_defaults(SMALL[case])
    s, ring, nz = make_session(w), oracle_ring(w), oracle_normalizer(w)
    cnt, mean, m2, mean32, rstd32 = s.obs_statistics()
    assert cnt == 0 and not mean.any() and not m2.any() and not mean32.any()
    assert np.allclose(rstd32, 1.0 / np.sqrt(1.0 + w.obs_norm_eps), rtol=1e-7)
    rng = None
    for rows in (1, 2, w.rows + 3):                     # statistics keep growing after the ring wraps
        rng = fill_both(s, ring, w, rows, rng=rng, normalizer=nz)
        cnt, mean, m2, mean32, rstd32 = s.obs_statistics()
        assert cnt == nz.count
        e_mean, e_m2 = rel_err(mean, nz.mean), rel_err(m2, nz.m2)
        e32 = max(rel_err(mean32, nz.mean), rel_err(rstd32, 1.0 / np.sqrt(nz.var + nz.eps)))
        say(case, "rows", nz.count // w.num_envs, "mean %.1e m2 %.1e fp32 %.1e" % (e_mean, e_m2, e32))
        assert e_mean <= 1e-12 and e_m2 <= 1e-10 and e32 <= 1e-7


@pytest.mark.parametrize("case", ["tiny", "ragged", "ant_s", "fused_l1", "scale_s"])
def test_standardised_sampling_and_actor_step(torch_cuda, case):
    torch = torch_cuda
    w = paper_defaults(SMALL[case])
    s, ring, nz = make_session(w), oracle_ring(w), oracle_normalizer(w)
    fill_both(s, ring, w, w.nstep + 3, normalizer=nz)
    for call in range(2):
        Bsz = w.batch if call == 0 else 7
        s.sample(Bsz)
        assert_batch_matches(batch_to_numpy(s.batch, Bsz), oracle_batch(ring, w, Bsz, call, nz), normalized=True, ring=ring, normalizer=nz)
    idx = np.arange(w.num_envs, dtype=np.int64)
    s.gather(torch.from_numpy(idx).cuda())
    got = batch_to_numpy(s.batch, idx.size)
    got["idx"] = idx
    assert_batch_matches(got, O.normalize_batch(O.gather_nstep(ring, idx, w.nstep, w.gamma), nz), normalized=True, ring=ring, normalizer=nz)
    assert np.array_equal(s.storage.obs.cpu().numpy(), ring.obs)          # the ring keeps raw observations
    row = W.transition_rows(w, np.random.default_rng(3), 1)[0]
    for call, num in enumerate((w.num_envs, 5)):
        obs = row["obs"][:num]
        got = s.act(torch.from_numpy(obs).cuda(), 0.05, 0.8).cpu().numpy()
        ref = O.actor_act(s.actor_init, w.actor_dims(), nz.normalize(obs), float(np.float32(0.05)),
                          float(np.float32(0.8)), w.rng_seed, call)
        e = rel_err(got, ref)
        say(case, "standardised act, num", num, "rel err %.2e" % e)
        assert e <= TOL_ONE_STEP
    # detaching restores the raw path bit for bit
    s.ctx.pql_obs_norm_attach(None, 0.0)
    s.sample(w.batch)
    assert_batch_matches(batch_to_numpy(s.batch, w.batch), oracle_batch(ring, w, w.batch, 2, None), ring=ring)


@pytest.mark.parametrize("case,bound", [("tiny", 0.5), ("ragged", 0.5), ("ant_s", 0.5), ("fused_l3", 0.01),
                                        ("humanoid_s", 0.01), ("tiny", 1e6)])
def test_one_update_with_clipping_and_standardisation(torch_cuda, case, bound):
    """bound 0.5: the critic gradient is clipped, the policy gradient is inside the ball;
    0.01: both are clipped; 1e6: neither (the two-kernel clipped step must then equal the plain one)."""
    w = paper_defaults(SMALL[case], bound)
    res = one_step(torch_cuda, w, min(w.rows, w.nstep + 4))
    say(case, bound, res)
    assert res["c_clipped"] == (bound < 1.0) and res["a_clipped"] == (bound < 0.02)


@pytest.mark.parametrize("case", ["tiny", "ant_s"])
def test_100_updates_with_clipping_and_standardisation(torch_cuda, case):
    w = paper_defaults(SMALL[case])
    res = many_steps(torch_cuda, w, w.rows, 100, actor_every=2)
    say(case, "100 clipped steps", res)


def test_ant_full_batch_paper_defaults(torch_cuda):
    w = paper_defaults(W.WORKLOADS["ant"])
    res = one_step(torch_cuda, w, w.nstep + 8)
    say("ant, clipping + standardisation", res)


# ---------------------------------------------------------------------------------------------
# PQL-D: distributional critics (51 atoms on (-10, 10) in the paper's appendix)
def distributional(w, atoms=51, v_min=-10.0, v_max=10.0):
    return w.replace(num_atoms=atoms, v_min=float(np.float32(v_min)), v_max=float(np.float32(v_max)))


DIST_CASES = {
    "tiny_d": (SMALL["tiny"], 51, -10.0, 10.0),
    "ragged_d": (SMALL["ragged"], 11, -4.0, 4.0),          # few atoms on a narrow support: much clipping at the bounds
    "ant_s_d": (SMALL["ant_s"], 51, -10.0, 10.0),
    "shadow_s_d": (SMALL["shadow_s"], 64, -10.0, 10.0),    # the largest supported atom count
    "fused_l3_d": (SMALL["fused_l3"], 2, -1.0, 1.0),       # the smallest
    # row-tile path, two layers of 128 / 224 columns: the LDS scratch of the logit products is longer than one
    # activation tile here and reaches into the tile that holds the second critic's last hidden layer
    "fused_mid_d": (SMALL["fused_wide_in"].replace(name="fused_mid", obs_dim=109, act_dim=32, hidden=(128, 224), index=18),
                    51, -2.0, 3.0),
    "fused_mid4_d": (SMALL["fused_wide_in"].replace(name="fused_mid4", obs_dim=45, act_dim=7, hidden=(160, 192, 128, 160),
                                                    index=19), 33, -3.0, 3.0),
}


@pytest.mark.parametrize("case", list(DIST_CASES))
def test_one_update_distributional(torch_cuda, case):
    base, atoms, lo, hi = DIST_CASES[case]
    w = distributional(base, atoms, lo, hi)
    say("case", case, "atoms", atoms, "critic dims", w.critic_dims())
    res = one_step(torch_cuda, w, min(w.rows, w.nstep + 4))
    say(case, res)


def test_one_update_distributional_with_paper_defaults(torch_cuda):
    w = paper_defaults(distributional(SMALL["ant_s"]))
    res = one_step(torch_cuda, w, w.nstep + 4)
    say("ant_s, 51 atoms, clipping + standardisation", res)


@pytest.mark.parametrize("case", ["tiny_d", "ant_s_d"])
def test_100_updates_distributional(torch_cuda, case):
    base, atoms, lo, hi = DIST_CASES[case]
    w = distributional(base, atoms, lo, hi)
    res = many_steps(torch_cuda, w, w.rows, 100, actor_every=2)
    say(case, "100 steps", res)


def test_distributional_full_batch_ant(torch_cuda):
    w = distributional(W.WORKLOADS["ant"])
    res = one_step(torch_cuda, w, w.nstep + 8)
    say("ant, 51 atoms, batch 8192", res)


# ---------------------------------------------------------------------------------------------
# PQL + SAC: tanh-Gaussian policy, soft target, learnable temperature
def with_sac(w):
    return w.replace(sac=True)


@pytest.mark.parametrize("case", ["tiny", "ragged", "ant_s", "humanoid_s", "fused_l1"])
def test_sac_actor_step_is_a_policy_sample(torch_cuda, case):
    torch = torch_cuda
    w = with_sac(SMALL[case])
    s = make_session(w)
    rng = np.random.default_rng(7)
    # (the last call of layer_tiles is large enough for the row-tile layer kernels, noise epilogue included)
    for call, num in enumerate((w.num_envs, 1, min(s.max_batch, 333)) + ((s.max_batch,) if case == "layer_tiles" else ())):
        obs = rng.standard_normal((num, w.obs_dim), dtype=np.float32)
        got = s.act(torch.from_numpy(obs).cuda()).cpu().numpy()
        ref = O.sac_actor_act(s.actor_init, w.actor_dims(), obs, w.rng_seed, call)
        e = rel_err(got, ref)
        say(case, "SAC act call", call, "num", num, "rel err %.2e" % e)
        assert e <= TOL_ONE_STEP and np.abs(got).max() <= 1.0


@pytest.mark.parametrize("case", ["tiny", "ragged", "ant_s", "humanoid_s", "fused_l3"])
def test_one_update_sac(torch_cuda, case):
    w = with_sac(SMALL[case])
    say("case", case, "actor dims", w.actor_dims())
    res = one_step(torch_cuda, w, min(w.rows, w.nstep + 4))
    say(case, res)


def test_one_update_sac_with_paper_defaults(torch_cuda):
    w = paper_defaults(with_sac(SMALL["ant_s"]))
    res = one_step(torch_cuda, w, w.nstep + 4)
    say("ant_s SAC, clipping + standardisation", res)


@pytest.mark.parametrize("case", ["tiny", "ant_s"])
def test_100_updates_sac(torch_cuda, case):
    w = with_sac(SMALL[case])
    s_res = many_steps(torch_cuda, w, w.rows, 100, actor_every=2)
    say(case, "100 SAC steps", s_res)


def test_sac_full_batch_ant(torch_cuda):
    w = with_sac(W.WORKLOADS["ant"])
    res = one_step(torch_cuda, w, w.nstep + 8)
    say("ant SAC, batch 8192", res)


# ---------------------------------------------------------------------------------------------
# degenerate and boundary sizes
@pytest.mark.parametrize("case", ["tiny", "ragged"])
@pytest.mark.parametrize("Bsz", [1, 33])
def test_updates_on_one_row_and_on_one_row_more_than_a_tile(torch_cuda, case, Bsz):
    """Batch 1 (every mean is over one sample) and batch 33 (a 32-row tile plus one row), through the
    row-tile kernels (tiny) and the grouped GEMMs (ragged)."""
    w = SMALL[case].replace(batch=Bsz)
    res = one_step(torch_cuda, w, w.nstep + 2)
    say(case, "batch", Bsz, res)


@pytest.mark.parametrize("variant", ["scalar", "dist", "sac"])
@pytest.mark.parametrize("widths", [(64,) * 8, (96, 40, 96, 40, 96, 40, 96, 40)])
def test_deepest_network(torch_cuda, widths, variant):
    """Eight hidden layers (the most the interface takes): the row-tile kernels (widths 64) and the grouped
    GEMMs (widths 96 / 40), with every variant of critic and policy."""
    w = SMALL["ragged"].replace(hidden=widths, batch=150, index=30)
    if variant == "dist":
        w = distributional(w)
    if variant == "sac":
        w = with_sac(w)
    res = one_step(torch_cuda, w, w.nstep + 2)
    say("8 layers", widths[:2], variant, res)


@pytest.mark.parametrize("variant", ["scalar", "dist64", "sac31"])
def test_widest_inputs_and_outputs(torch_cuda, variant):
    """Wide observation and action vectors (more than one 32-column tile of actions), the most atoms with a
    last hidden layer too narrow for the row-tile path, the widest stochastic policy (31 actions)."""
    base = SMALL["ragged"].replace(obs_dim=300, act_dim=40, hidden=(128, 64), batch=200, num_envs=37, capacity=37 * 8, index=31)
    if variant == "dist64":
        w = distributional(base.replace(hidden=(128, 32)), 64)
    elif variant == "sac31":
        w = with_sac(base.replace(act_dim=31))
    else:
        w = base
    res = one_step(torch_cuda, w, w.nstep + 2)
    say("wide", variant, res)
    torch = torch_cuda
    s = make_session(w)
    obs = np.random.default_rng(5).standard_normal((w.num_envs, w.obs_dim), dtype=np.float32)
    got = s.act(torch.from_numpy(obs).cuda(), 0.05, 0.8).cpu().numpy()
    ref = (O.sac_actor_act(s.actor_init, w.actor_dims(), obs, w.rng_seed, 0) if w.sac else
           O.actor_act(s.actor_init, w.actor_dims(), obs, float(np.float32(0.05)), float(np.float32(0.8)), w.rng_seed, 0))
    assert rel_err(got, ref) <= TOL_ONE_STEP


def test_empty_batch_and_single_environment(torch_cuda):
    torch = torch_cuda
    w = SMALL["tiny"]
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, w.nstep + 1)
    before = {k: getattr(s.batch, k).clone() for k in ("idx", "obs", "act", "ret", "next_obs", "boot")}
    s.ctx.pql_sample_nstep(s.storage, 0, s.batch)      # nothing to draw: nothing is written, the draw is still counted
    torch.cuda.synchronize()
    for k, v in before.items():
        assert torch.equal(getattr(s.batch, k), v), k
    assert s.ctx.get_state()[3] == 1
    s.sample(w.batch)                                  # the next draw is call number 1 on both sides
    assert_batch_matches(batch_to_numpy(s.batch, w.batch), oracle_batch(ring, w, w.batch, 1), ring=ring)
    # one environment: its noise scale is sigma_min (Section 3.3 with N = 1)
    obs = np.random.default_rng(2).standard_normal((1, w.obs_dim), dtype=np.float32)
    got = s.act(torch.from_numpy(obs).cuda(), 0.3, 0.9).cpu().numpy()
    ref = O.actor_act(s.actor_init, w.actor_dims(), obs, float(np.float32(0.3)), float(np.float32(0.9)), w.rng_seed, 0)
    assert rel_err(got, ref) <= TOL_ONE_STEP
    mu = O.actor_forward(s.actor_init, w.actor_dims(), obs)
    eps = O.gaussian_noise(w.rng_seed, 0, w.act_dim)
    assert np.allclose(ref, np.clip(mu + float(np.float32(0.3)) * eps, -1, 1), rtol=1e-12)


def test_every_transition_terminal(torch_cuda):
    """done = 1 everywhere: boot = 0 for every window, the target is the first reward alone and the
    target networks drop out of the update."""
    torch = torch_cuda
    w = SMALL["ant_s"].replace(done_p=1.0, batch=200)
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, w.nstep + 3)
    s.sample(w.batch)
    got = batch_to_numpy(s.batch, w.batch)
    assert not got["boot"].any()
    assert np.array_equal(got["ret"], ring.rew[got["idx"]])            # later rewards are masked out exactly
    s.critic_update(w.batch)
    loss_a = s.critic_loss.cpu().numpy().copy()
    s2 = make_session(w)
    fill_both(s2, oracle_ring(w), w, w.nstep + 3)
    s2.critic_target.mul_(3.0)                                          # different target critics and lagged policy: no influence
    s2.actor_lag.mul_(-2.0)
    s2.sample(w.batch)
    s2.critic_update(w.batch)
    assert np.array_equal(s2.critic_loss.cpu().numpy(), loss_a)
    assert torch.equal(s.critic, s2.critic)
    L = oracle_learner(w, s.actor_init, s.critic_init)
    losses, _ = L.critic_update(oracle_batch(ring, w, w.batch, 0))
    assert rel_err(loss_a, losses) <= TOL_ONE_STEP


# ---------------------------------------------------------------------------------------------
def test_ant_full_ring_as_benchmarked(torch_cuda):
    """The benchmark's launch configuration: ant-shaped workload with the whole ring filled and
    wrapped (T = 244 rows of 4096 environments), batch 8192: sampled indices and gathered rows
    bit-exact, one critic update and one policy update within tolerance."""
    w = W.WORKLOADS["ant"]
    say("filling", w.rows + 5, "rows of", w.num_envs, "environments")
    res = one_step(torch_cuda, w, w.rows + 5)
    say("ant full ring", res)


def test_runs_are_bit_reproducible_and_resumable(torch_cuda):
    """All reductions have a fixed order: two runs from the same seed agree bit for bit, and a run
    resumed through pql_get_state / pql_set_state on the same device buffers continues identically."""
    torch = torch_cuda
    w = SMALL["ant_s"]

    def run(steps, resume_at=None):
        s = make_session(w)
        for row in W.transition_rows(w, W.data_rng(w), w.rows):
            s.push(row)
        for it in range(steps):
            if resume_at is not None and it == resume_at:
                from paper_2307_12983_amd import binding as Bn
                state = s.ctx.get_state()
                s.ctx.close()
                s.ctx = Bn.Context(s.cfg)            # fresh context, same device buffers
                s.ctx.set_state(state)
            s.sample(w.batch)
            s.critic_update(w.batch)
            s.soft_update_targets()
            if it % 2 == 1:
                s.actor_update(None, w.batch)
                s.sync_lagged_policy()
        torch.cuda.synchronize()
        return [t.clone() for t in (s.critic, s.critic_target, s.actor, s.c_m, s.c_v, s.a_m, s.a_v, s.batch.idx)]

    a, b, c = run(6), run(6), run(6, resume_at=3)
    for x, y, z in zip(a, b, c):
        assert torch.equal(x, y), "two identical runs differ"
        assert torch.equal(x, z), "resumed run differs"


def transposed_blocks(s, w):
    """What the block of transposed weights must hold for the session's current parameters, in the order
    the library lays it out (each matrix starts on a 256-byte boundary)."""
    torch = s.torch
    up = lambda n: (n + 63) // 64 * 64
    out, off = [], 0
    Pc = s.critic.numel() // 2
    o, a, H = w.obs_dim, w.act_dim, w.hidden
    outs = w.num_atoms if w.num_atoms >= 2 else 1
    for i in range(2):
        q = s.critic[i * Pc:(i + 1) * Pc]
        pos = (o + a) * H[0] + H[0]
        for l in range(1, len(H)):
            out.append((off, q[pos:pos + H[l - 1] * H[l]].view(H[l - 1], H[l]).t().contiguous().view(-1)))
            off += up(H[l - 1] * H[l]); pos += H[l - 1] * H[l] + H[l]
        out.append((off, q[o * H[0]:(o + a) * H[0]].view(a, H[0]).t().contiguous().view(-1)))
        off += up(a * H[0])
        if w.num_atoms >= 2:
            out.append((off, q[pos:pos + H[-1] * outs].view(H[-1], outs).t().contiguous().view(-1)))
        off += up(outs * H[-1])
    pos = o * H[0] + H[0]
    aw = 2 * a if w.sac else a
    for l in range(1, len(H) + 1):
        cols = H[l] if l < len(H) else aw
        out.append((off, s.actor[pos:pos + H[l - 1] * cols].view(H[l - 1], cols).t().contiguous().view(-1)))
        off += up(H[l - 1] * cols); pos += H[l - 1] * cols + cols
    return out, off


FOLD_CASES = {
    "ant_s": lambda: SMALL["ant_s"],
    "fused_l3": lambda: SMALL["fused_l3"],
    "humanoid_s": lambda: SMALL["humanoid_s"],
    "layer_tiles": lambda: SMALL["layer_tiles"].replace(batch=8195),
    "fused_l3_dist": lambda: distributional(SMALL["fused_l3"], 33, -3.0, 3.0),
    "ragged_dist": lambda: distributional(SMALL["ragged"], 11, -4.0, 4.0),
    "ant_s_sac": lambda: with_sac(SMALL["ant_s"]),
    "ant_s_clipped": lambda: paper_defaults(SMALL["ant_s"]),
    "humanoid_s_clipped": lambda: paper_defaults(SMALL["humanoid_s"], 0.01),
    "chain_humanoid": lambda: CHAIN["chain_humanoid"],
    "chain_l4": lambda: CHAIN["chain_l4"],
}


@pytest.mark.parametrize("case", list(FOLD_CASES))
def test_folded_followups_equal_the_separate_calls(torch_cuda, case):
    """pql_track_attach + pql_weight_cache_*: the Polyak step of the target critics, the hard copy into the
    lagged policy and the transposed weights ride on the optimiser kernels.  Against a second session that
    makes the separate calls (pql_soft_update twice, transposes inside every update): every parameter,
    target, moment and loss bit for bit over six critic and three policy updates, and the block of
    transposed weights equals the transposes of the current parameters after every step."""
    torch = torch_cuda
    w = FOLD_CASES[case]()
    a, b = make_session(w), make_session(w)
    nz = oracle_normalizer(w)
    fill_both(a, oracle_ring(w), w, min(w.rows, w.nstep + 4), normalizer=nz)
    fill_both(b, oracle_ring(w), w, min(w.rows, w.nstep + 4))
    b.fold_followups()
    assert b.ctx.weight_cache_bytes() == 4 * transposed_blocks(b, w)[1]
    for it in range(6):
        for s in (a, b):
            s.sample(w.batch)
            s.critic_update(w.batch)
            s.soft_update_targets()                       # a: pql_soft_update; b: nothing left to do
            if it % 2 == 1:
                s.actor_update(None, w.batch)
                s.sync_lagged_policy()
        torch.cuda.synchronize()
        for name in ("critic", "critic_target", "actor", "actor_lag", "c_m", "c_v", "c_g", "a_m", "a_v", "a_g",
                     "critic_out", "actor_out"):
            assert torch.equal(getattr(a, name), getattr(b, name)), "%s differs after step %d" % (name, it)
        for off, ref in transposed_blocks(b, w)[0]:
            assert torch.equal(b.weight_cache[off:off + ref.numel()], ref), "transposed weights at %d, step %d" % (off, it)
    # a parameter vector changed behind the library's back needs a refresh; after it the two agree again
    for s in (a, b):
        s.critic.mul_(0.5)
        s.actor.mul_(-1.0)
    b.ctx.pql_weight_cache_refresh(b.critic, b.actor)
    for s in (a, b):
        s.sample(w.batch)
        s.critic_update(w.batch)
        s.soft_update_targets()
        s.actor_update(None, w.batch)
        s.sync_lagged_policy()
    torch.cuda.synchronize()
    for name in ("critic", "critic_target", "actor", "actor_lag"):
        assert torch.equal(getattr(a, name), getattr(b, name)), "%s differs after the refresh" % name
    # another parameter vector (a snapshot) is not served from the block
    snap = b.critic.clone()
    b.ctx.pql_actor_update(b.actor, snap, b.a_m, b.a_v, b.a_g, b.batch.obs, w.batch, b.opt, b.actor_loss, b.workspace)
    a.ctx.pql_actor_update(a.actor, a.critic, a.a_m, a.a_v, a.a_g, a.batch.obs, w.batch, a.opt, a.actor_loss, a.workspace)
    a.sync_lagged_policy()
    torch.cuda.synchronize()
    assert torch.equal(a.actor, b.actor) and torch.equal(a.actor_lag, b.actor_lag)


def test_folded_followups_100_steps_against_the_oracle(torch_cuda):
    """The benchmark's configuration of the calls (follow-ups folded into the optimiser kernels) through 100
    critic and 10 policy updates of the ant-shaped workload at batch 8192 against the oracle."""
    w = W.WORKLOADS["ant"]
    res = many_steps(torch_cuda, w, w.nstep + 8, 100, actor_every=10, fold=True,
                     must_run=("fused_critic_kernel", "fused_policy_kernel", "adam_reduce_kernel"),
                     must_not_run=("soft_update_kernel", "copy_kernel", "transpose_kernel"))
    say("ant 100 steps, folded follow-ups", res)


def test_kernel_profile_reports_launches_and_work(torch_cuda):
    torch = torch_cuda
    w = SMALL["ant_s"]
    s = make_session(w)
    for row in W.transition_rows(w, W.data_rng(w), w.nstep + 2):
        s.push(row)
    s.sample(w.batch)
    s.critic_update(w.batch)
    torch.cuda.synchronize()
    s.ctx.pql_profile_begin(64)
    s.sample(w.batch)
    s.critic_update(w.batch)
    s.soft_update_targets()
    torch.cuda.synchronize()
    stats = {k["name"]: k for k in s.ctx.pql_profile_end()}
    say(sorted(stats))
    assert stats["sample_kernel"]["launches"] == 1 and stats["adam_reduce_kernel"]["launches"] == 1
    assert stats["soft_update_kernel"]["bytes"] == 12.0 * s.critic.numel()
    flops = sum(k["flops"] for k in stats.values())
    pc = sum(i * o for i, o in w.critic_dims())
    pa = sum(i * o for i, o in w.actor_dims())
    first = w.critic_dims()[0][0] * w.critic_dims()[0][1]
    # target path (policy + twin targets) + twin forward + weight gradients of the hidden layers (the
    # output layer's come from the head reductions) + backward data path of all but the first layer
    expect = w.batch * 2 * (pa + 2 * pc + 2 * pc + 2 * (pc - w.critic_dims()[-1][0]) + 2 * (pc - first))
    assert abs(flops - expect) <= 0.02 * expect, (flops, expect)
    assert all(k["total_ms"] > 0 for k in stats.values())
    from paper_2307_12983_amd.binding import PqlError
    with pytest.raises(PqlError):
        s.ctx.pql_profile_end()


@pytest.mark.parametrize("case", list(SMALL))
def test_which_cases_take_the_row_tile_kernels(torch_cuda, case):
    """The cases meant to cover the row-tile kernels really run them (and the others the layered path):
    the library's own per-kernel profile names what was launched."""
    w = SMALL[case]
    s, ring = make_session(w), oracle_ring(w)
    fill_both(s, ring, w, w.nstep + 2)
    s.sample(w.batch)
    s.ctx.pql_profile_begin(256)
    s.critic_update(w.batch)
    s.actor_update(None, w.batch)
    s.act(s.batch.obs[:min(w.num_envs, w.batch)])
    torch_cuda.cuda.synchronize()
    names = {k["name"] for k in s.ctx.pql_profile_end()}
    say(case, sorted(names))
    fused = {"fused_critic_kernel", "fused_policy_kernel", "fused_act16_kernel"}     # (few environments: 16-row tiles)
    if case in ROW_TILE_CASES:
        assert fused <= names and not any(n.startswith("gemm_grouped_n") for n in names)
    else:
        assert not ((fused | {"fused_act_kernel"}) & names)
    assert ("layer_rowtile_kernel" in names) == (case == "layer_tiles")
    assert ("narrow_rowtile_kernel" in names) == (case == "layer_tiles")


# ---------------------------------------------------------------------------------------------
# Seeded random shapes.  The hand-picked cases above miss combinations (a distributional critic with
# an even number of 128- to 224-wide layers once computed wrong hidden-layer gradients for its second
# network); here widths, depths, input sizes, batch sizes, n and the variant are drawn from a seeded
# generator.  Only what is robust for any shape is compared: the sampled batch, the losses and every
# gradient tensor of one critic and one policy update (max-norm, 1e-4).
def random_shape(rnd, it, wide=False):
    row_tile = rnd.random() < 0.6 and not wide         # all widths multiples of 32 and at most 256: the row-tile kernels
    depth = rnd.choice([1, 2, 2, 3, 4])
    if wide:                                           # a layer too wide for them and a batch large enough for the row-tile layer kernel
        hidden = tuple(rnd.choice([128, 136, 160, 200, 260, 288, 300, 320, 384, 512, 516, 640]) for _ in range(depth))
        if max(hidden) <= 256 and all(h % 32 == 0 for h in hidden):
            hidden = hidden[:-1] + (300,)
        act = rnd.randint(1, 40)
    elif row_tile:
        hidden = tuple(32 * rnd.randint(1, 8) for _ in range(depth))
        act = rnd.randint(1, 32)
    else:
        hidden = tuple(rnd.choice([40, 72, 100, 200, 288, 320, 512]) for _ in range(depth))
        act = rnd.randint(1, 40)
    variant = rnd.choice(["scalar", "scalar", "dist", "sac", "defaults"])
    if variant == "sac":
        act = min(act, 15)
    nstep = rnd.choice([1, 2, 3, 3, 5])
    envs = rnd.randint(5, 70)
    kw = dict(name="rand%d" % it, obs_dim=rnd.randint(3, 230), act_dim=act, num_envs=envs,
              capacity=envs * rnd.randint(nstep + 4, nstep + 10),
              batch=rnd.choice([2753, 4096, 4100, 5510, 8192, 8195] if wide else [31, 33, 64, 100, 257, 333, 512, 777, 1500]),
              hidden=hidden, index=60 + it, nstep=nstep)
    if variant == "dist":
        kw.update(num_atoms=rnd.choice([2, 11, 51, 64]), v_min=float(np.float32(-2.0)), v_max=float(np.float32(3.0)))
    if variant == "sac":
        kw.update(sac=True)
    if variant == "defaults":
        kw.update(max_grad_norm=float(np.float32(0.5)), obs_norm=True, obs_loc=1.0, obs_scale=2.0)
    return variant, W.WORKLOADS["tiny"].replace(**kw)


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_gradients_on_random_shapes(torch_cuda, seed):
    import random
    rnd = random.Random(seed)
    wide = seed == 14
    for it in range(24 if wide else 40):
        variant, w = random_shape(rnd, it, wide)
        say(seed, it, variant, "obs", w.obs_dim, "act", w.act_dim, "envs", w.num_envs, "B", w.batch, "n", w.nstep, "hidden", w.hidden,
            "atoms", w.num_atoms)
        s, ring, nz = make_session(w), oracle_ring(w), oracle_normalizer(w)
        fill_both(s, ring, w, min(w.rows, w.nstep + 3), normalizer=nz)
        L = oracle_learner(w, s.actor_init, s.critic_init)
        s.sample(w.batch)
        batch = oracle_batch(ring, w, w.batch, 0, nz)
        assert_batch_matches(batch_to_numpy(s.batch, w.batch), batch, normalized=nz is not None, ring=ring, normalizer=nz)
        s.critic_update(w.batch)
        losses, g = L.critic_update(batch)
        assert rel_err(s.critic_loss.cpu().numpy(), losses) <= TOL_ONE_STEP
        assert_params_close(s.c_g.cpu().numpy(), g, w.critic_dims(), 2, TOL_ONE_STEP, "critic grad")
        s.actor_update(None, w.batch)
        _, ga = L.actor_update(batch["obs"])
        assert_params_close(s.a_g.cpu().numpy(), ga, w.actor_dims(), 1, TOL_ONE_STEP, "actor grad")
