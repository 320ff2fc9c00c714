"""The V-learner step on the library's own scratch array (pql_critic_update_static), called through
the C-ABI, against pql_critic_update with a caller-owned workspace: two calls in a row on the same
GPU, the second with a smaller batch, every output bit for bit (both entry points enqueue the same
kernels with the same arguments; only the scratch address differs), and the first also against the
CPU oracle to the one-step tolerance."""
import numpy as np
import pytest

from paper_2307_12983_amd import workloads as W

from parity_util import (TOL_ONE_STEP, assert_params_close, fill_both, oracle_batch, oracle_learner, oracle_ring,
                         rel_err)

pytestmark = pytest.mark.gpu


def _session(w):
    from paper_2307_12983_amd.session import LearnerSession
    return LearnerSession(w)


@pytest.mark.parametrize("case", ["row_tile", "layered"])
def test_static_scratch_entry_point_matches_workspace_entry_point(case):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    base = W.WORKLOADS["ant"]
    if case == "row_tile":      # the chained row-tile kernels
        w = base.replace(name="static_a", num_envs=96, capacity=96 * 13, batch=1000)
    else:                       # a layer wider than 256: the per-layer path with its many scratch buffers
        w = W.WORKLOADS["humanoid"].replace(name="static_h", num_envs=64, capacity=64 * 9, batch=777)
    a, b, ring = _session(w), _session(w), oracle_ring(w)
    assert a.ctx.workspace_bytes() <= a.ctx.static_scratch_bytes()
    fill_both(a, ring, w, w.nstep + 4)
    fill_both(b, oracle_ring(w), w, w.nstep + 4)
    L = oracle_learner(w, a.actor_init, a.critic_init)
    for call, Bsz in enumerate((w.batch, 333)):              # the second call is smaller than the first
        print("case", case, "call", call, "batch", Bsz, flush=True)
        a.sample(Bsz)
        b.sample(Bsz)
        assert torch.equal(a.batch.obs, b.batch.obs)
        a.ctx.pql_critic_update(a.critic, a.critic_target, a.actor_lag, a.c_m, a.c_v, a.c_g, a.batch, Bsz, a.opt,
                                a.critic_loss, a.workspace)
        b.ctx.pql_critic_update_static(b.critic, b.critic_target, b.actor_lag, b.c_m, b.c_v, b.c_g, b.batch, Bsz, b.opt,
                                       b.critic_loss)
        torch.cuda.synchronize()
        for name in ("critic", "c_m", "c_v", "c_g", "critic_out"):
            assert torch.equal(getattr(a, name), getattr(b, name)), "%s differs on call %d" % (name, call)
        assert a.ctx.get_state() == b.ctx.get_state()
        batch = oracle_batch(ring, w, Bsz, call)
        losses, g = L.critic_update(batch)
        assert rel_err(b.critic_loss.cpu().numpy(), losses) <= TOL_ONE_STEP
        assert_params_close(b.c_g.cpu().numpy(), g, w.critic_dims(), 2, TOL_ONE_STEP, "critic grad (static scratch)")
        a.soft_update_targets(); b.soft_update_targets(); L.soft_update_targets()
    # the array is shared by every context on the GPU: a second context right after the first works on it too
    c = _session(w)
    fill_both(c, oracle_ring(w), w, w.nstep + 4)
    c.sample(200)
    c.ctx.pql_critic_update_static(c.critic, c.critic_target, c.actor_lag, c.c_m, c.c_v, c.c_g, c.batch, 200, c.opt,
                                   c.critic_loss)
    L2 = oracle_learner(w, c.actor_init, c.critic_init)
    losses, g = L2.critic_update(oracle_batch(ring, w, 200, 0))
    assert rel_err(c.critic_loss.cpu().numpy(), losses) <= TOL_ONE_STEP
    assert_params_close(c.c_g.cpu().numpy(), g, w.critic_dims(), 2, TOL_ONE_STEP, "critic grad (second context)")


def test_static_scratch_entry_point_refuses_large_configurations():
    import torch
    from paper_2307_12983_amd.binding import PqlError
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    w = W.WORKLOADS["humanoid"].replace(num_envs=64, capacity=64 * 9)       # batch 8192: 290 MB of scratch
    s = _session(w)
    before = s.ctx.get_state()
    with pytest.raises(PqlError) as e:
        s.ctx.pql_critic_update_static(s.critic, s.critic_target, s.actor_lag, s.c_m, s.c_v, s.c_g, s.batch, 64, s.opt,
                                       s.critic_loss)
    assert e.value.code == -7 and s.ctx.get_state() == before
