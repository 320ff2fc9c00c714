"""The C-ABI driven from C: tests/c_client/pql_client.c (plain C99, hipMalloc'd buffers, no Python or torch in its
process; built by `python -m paper_2307_12983_amd.build`) runs one learner iteration and one Actor step on a
problem this test writes to a file.  Its results must be the Python session's bit for bit (the same library,
the same calls, other owners of the memory), and the losses the oracle's."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import pql_oracle as O
from paper_2307_12983_amd import workloads as W
from parity_util import TOL_ONE_STEP, oracle_batch, oracle_learner, oracle_ring, rel_err

pytestmark = pytest.mark.gpu



@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    return torch


CLIENT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_client", "pql_client")

CASES = {
    "tiny": W.WORKLOADS["tiny"],
    # ragged everything: no dimension a multiple of a tile, ring of 7 rows, layered path
    "ragged": W.WORKLOADS["tiny"].replace(name="ragged_c", obs_dim=13, act_dim=3, num_envs=37, capacity=37 * 7 + 5, batch=101,
                                          hidden=(48, 72), index=7),
    "ant_small_batch": W.WORKLOADS["ant"].replace(name="ant_c", num_envs=96, capacity=96 * 12, batch=1000),
}


@pytest.mark.parametrize("case", list(CASES))
def test_c_client_matches_the_python_session(torch_cuda, tmp_path, case):
    torch = torch_cuda
    from paper_2307_12983_amd.session import LearnerSession
    assert os.path.exists(CLIENT), "tests/c_client/pql_client is missing: run `python -m paper_2307_12983_amd.build`"
    w = CASES[case]
    rows = w.nstep + 3
    s = LearnerSession(w)
    data = W.transition_rows(w, W.data_rng(w), rows)
    act_obs = np.random.default_rng(11).standard_normal((w.num_envs, w.obs_dim), dtype=np.float32)
    hidden = list(w.hidden) + [0] * (8 - len(w.hidden))
    problem = tmp_path / "problem.bin"
    with open(problem, "wb") as f:
        f.write(struct.pack("<15i", w.obs_dim, w.act_dim, w.num_envs, w.nstep, len(w.hidden), *hidden, w.batch, rows))
        f.write(struct.pack("<qQ", w.capacity, w.rng_seed))
        f.write(np.asarray([w.gamma, w.lr, w.beta1, w.beta2, w.eps, w.tau, w.sigma_min, w.sigma_max], np.float32).tobytes())
        f.write(np.ascontiguousarray(s.actor_init, np.float32).tobytes())
        f.write(np.ascontiguousarray(s.critic_init, np.float32).tobytes())
        for row in data:
            for k in ("obs", "act", "rew", "next_obs", "done"):
                f.write(np.ascontiguousarray(row[k], np.float32).tobytes())
        f.write(act_obs.tobytes())
    result = tmp_path / "result.bin"
    print("case", case, "running", CLIENT, flush=True)
    run = subprocess.run([CLIENT, str(problem), str(result)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, "client failed (%d): %s %s" % (run.returncode, run.stdout, run.stderr)
    assert run.stdout.split() == ("pushes %d samples 1 acts 1 critic steps 1 policy steps 1" % rows).split()

    # the same calls through the Python session
    ring = oracle_ring(w)
    for row in data:
        s.push(row)
        ring.push(row["obs"], row["act"], row["rew"], row["next_obs"], row["done"])
    s.sample(w.batch)
    s.critic_update(w.batch)
    s.soft_update_targets()
    s.actor_update(None, w.batch)
    s.sync_lagged_policy()
    actions = s.act(torch.from_numpy(act_obs).cuda()).cpu().numpy()
    torch.cuda.synchronize()

    raw = open(result, "rb").read()
    Pa, Pc2, B = s.actor.numel(), s.critic.numel(), w.batch
    idx = np.frombuffer(raw, np.int64, B, 0)
    fl = np.frombuffer(raw, np.float32, offset=8 * B)
    assert fl.size == 3 + 2 * Pc2 + 2 * Pa + w.num_envs * w.act_dim
    losses, J = fl[:2], fl[2]
    off = 3
    got = {}
    for name, n in (("critic", Pc2), ("critic_target", Pc2), ("actor", Pa), ("actor_lag", Pa), ("actions", w.num_envs * w.act_dim)):
        got[name] = fl[off:off + n]
        off += n
    assert np.array_equal(idx, s.batch.idx[:B].cpu().numpy())
    assert np.array_equal(losses, s.critic_loss.cpu().numpy()) and J == float(s.actor_loss.cpu()[0])
    for name, t in (("critic", s.critic), ("critic_target", s.critic_target), ("actor", s.actor), ("actor_lag", s.actor_lag)):
        assert np.array_equal(got[name], t.cpu().numpy()), name
    assert np.array_equal(got["actions"], actions.ravel())

    # and against the oracle: sampled indices, losses before the step, the policy objective, the actions
    L = oracle_learner(w, s.actor_init, s.critic_init)
    batch = oracle_batch(ring, w, B, 0)
    assert np.array_equal(idx, batch["idx"])
    ref_losses, _ = L.critic_update(batch)
    L.soft_update_targets()
    ref_J, _ = L.actor_update(batch["obs"])
    assert rel_err(losses, ref_losses) <= TOL_ONE_STEP and abs(J - ref_J) <= TOL_ONE_STEP * abs(ref_J)
    ref_act = O.actor_act(L.actor, w.actor_dims(), act_obs, w.sigma_min, w.sigma_max, w.rng_seed, 0)
    assert rel_err(got["actions"], ref_act.ravel()) <= TOL_ONE_STEP
