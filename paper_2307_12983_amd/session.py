"""Device-memory plumbing for one learner: allocates the caller-owned buffers the C interface
expects (replay ring, batch, parameters, Adam moments, gradients, workspace) with torch and
forwards each step to the C entry point of the same name.  No arithmetic happens here.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

from . import binding as B
from .workloads import Workload, init_networks


class LearnerSession:
    def __init__(self, w: Workload, device: str = "cuda", max_batch: Optional[int] = None, seed: Optional[int] = None):
        import torch
        self.torch = torch
        self.w = w
        self.device = device
        self.max_batch = int(max_batch or max(w.batch, w.num_envs))
        self.cfg = B.make_config(w.obs_dim, w.act_dim, w.num_envs, w.capacity, w.nstep, w.gamma, w.hidden,
                                 self.max_batch, w.rng_seed if seed is None else seed, w.num_atoms, w.v_min, w.v_max,
                                 1 if w.sac else 0)
        self.ctx = B.Context(self.cfg)
        self.rows = self.ctx.replay_rows()
        self.storage = B.Storage(self.rows, w.num_envs, w.obs_dim, w.act_dim, device)
        self.batch = B.Batch(self.max_batch, w.obs_dim, w.act_dim, device)
        actor, critic = init_networks(w)
        self.actor_init, self.critic_init = actor, critic
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
        self.actor = t(actor)
        self.actor_lag = t(actor)            # pi^v: the V-learner's lagged copy of the policy
        self.critic = t(critic)
        self.critic_target = t(critic)
        z = lambda n: torch.zeros(n, dtype=torch.float32, device=device)
        self.c_m, self.c_v, self.c_g = z(critic.size), z(critic.size), z(critic.size)
        self.a_m, self.a_v, self.a_g = z(actor.size), z(actor.size), z(actor.size)
        self.critic_out, self.actor_out = z(3), z(4)      # losses, then the gradient norm before clipping (SAC: two more)
        self.critic_loss, self.critic_grad_norm = self.critic_out[:2], self.critic_out[2:]
        self.actor_loss, self.actor_grad_norm = self.actor_out[:1], self.actor_out[1:]
        self.workspace = torch.zeros(self.ctx.workspace_bytes() // 4 + 64, dtype=torch.float32, device=device)
        assert self.workspace.data_ptr() % 256 == 0
        self.act_out = torch.zeros((self.max_batch, w.act_dim), dtype=torch.float32, device=device)
        self.opt = B.PqlAdam(w.lr, w.beta1, w.beta2, w.eps, w.max_grad_norm)
        self.temperature = None
        if w.sac:
            self.temperature = torch.tensor([float(np.log(np.float64(w.init_alpha))), 0.0, 0.0, 0.0], dtype=torch.float32,
                                            device=device)
            self.ctx.pql_sac_attach(self.temperature, w.target_entropy)
        self.folded = False
        self.obs_stats = None
        if w.obs_norm:
            self.obs_stats = torch.zeros(self.ctx.obs_norm_bytes() // 8 + 32, dtype=torch.float64, device=device)
            assert self.obs_stats.data_ptr() % 256 == 0
            self.ctx.pql_obs_norm_attach(self.obs_stats, w.obs_norm_eps)
            self.ctx.pql_obs_norm_reset()

    def fold_followups(self, on: bool = True):
        """Lets the optimiser kernels carry what follows them in the plain call sequence: the Polyak step of
        the target critics, the hard copy into the lagged policy and the transposed weights of the next
        backward pass (pql_track_attach, pql_weight_cache_*).  soft_update_targets() and
        sync_lagged_policy() then have nothing left to do."""
        torch = self.torch
        self.folded = bool(on)
        if not on:
            self.ctx.pql_track_attach(0, None, 0.0)
            self.ctx.pql_track_attach(1, None, 0.0)
            self.ctx.pql_weight_cache_attach(None)
            return
        self.weight_cache = torch.zeros(self.ctx.weight_cache_bytes() // 4 + 64, dtype=torch.float32, device=self.device)
        assert self.weight_cache.data_ptr() % 256 == 0
        self.ctx.pql_weight_cache_attach(self.weight_cache)
        self.ctx.pql_weight_cache_refresh(self.critic, self.actor)
        self.ctx.pql_track_attach(0, self.critic_target, self.w.tau)
        self.ctx.pql_track_attach(1, self.actor_lag, 1.0)

    def obs_statistics(self):
        """(count, mean[o], m2[o]) in float64 and (mean32[o], rstd32[o]) as stored on the device."""
        o = self.w.obs_dim
        d = self.obs_stats.cpu().numpy()
        f = d[2 + 2 * o: 2 + 3 * o].view(np.float32)
        return d[0], d[2:2 + o].copy(), d[2 + o:2 + 2 * o].copy(), f[:o].copy(), f[o:2 * o].copy()

    # ---- steps, one C call each ----------------------------------------------------------
    def to_device(self, row):
        t = self.torch
        return {k: (v if isinstance(v, t.Tensor) else t.from_numpy(np.ascontiguousarray(v))).to(self.device)
                for k, v in row.items()}

    def push(self, row, stream=None):
        r = self.to_device(row)
        self.ctx.pql_replay_push(self.storage, r["obs"], r["act"], r["rew"], r["next_obs"], r["done"], stream)

    def sample(self, batch_size: Optional[int] = None, stream=None):
        self.ctx.pql_sample_nstep(self.storage, int(batch_size or self.w.batch), self.batch, stream)

    def gather(self, idx, stream=None):
        self.ctx.pql_gather_nstep(self.storage, idx, int(idx.numel()), self.batch, stream)

    def critic_update(self, batch_size: Optional[int] = None, stream=None):
        self.ctx.pql_critic_update(self.critic, self.critic_target, self.actor_lag, self.c_m, self.c_v, self.c_g,
                                   self.batch, int(batch_size or self.w.batch), self.opt, self.critic_loss,
                                   self.workspace, stream)

    def soft_update_targets(self, stream=None):
        if self.folded:
            return                          # done by pql_critic_update's optimiser kernel
        self.ctx.pql_soft_update(self.critic, self.critic_target, self.critic.numel(), self.w.tau, stream)

    def actor_update(self, obs=None, batch_size: Optional[int] = None, stream=None):
        obs = self.batch.obs if obs is None else obs
        self.ctx.pql_actor_update(self.actor, self.critic, self.a_m, self.a_v, self.a_g, obs,
                                  int(batch_size or self.w.batch), self.opt, self.actor_loss, self.workspace, stream)

    def sync_lagged_policy(self, stream=None):
        if self.folded:
            return                          # done by pql_actor_update's optimiser kernel
        self.ctx.pql_soft_update(self.actor, self.actor_lag, self.actor.numel(), 1.0, stream)

    def act(self, obs, sigma_min=None, sigma_max=None, stream=None):
        n = int(obs.shape[0])
        self.ctx.pql_actor_act(self.actor, obs, n, self.w.sigma_min if sigma_min is None else sigma_min,
                               self.w.sigma_max if sigma_max is None else sigma_max, self.act_out, self.workspace,
                               stream)
        return self.act_out[:n]
