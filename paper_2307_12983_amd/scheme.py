"""The three concurrent parts of PQL (Section 3.1: Actor, V-learner, P-learner) on one GPU: three
HIP streams in one process, ordered by events instead of the paper's sleeps (Section 3.2).

Only plumbing lives here: which C entry point is enqueued on which stream, on which buffers, after
which event.  Every step of the arithmetic is one of the library's calls.

Schedule.  One *period* is one Actor iteration (Algorithm 1): `horizon` environment steps,
`v_updates` critic updates (Algorithm 3) and `p_updates` policy updates (Algorithm 2); the defaults
1 / 8 / 4 are the ratios beta_a:v = 1:8 and beta_p:v = 1:2 of Section 3.2, kept exactly.  Inside a
period each part reads and writes only its own copies, so the three streams need no ordering among
themselves; at the period boundary data and networks change hands as in Algorithms 1-3:

    V-learner  <- the Actor's transitions of the period (pushed into the ring) and the P-learner's
                  policy (pi^v, the lagged target policy)
    P-learner  <- the states (it samples them from the ring once they are there) and the
                  V-learner's critics (Q^p)
    Actor      <- the P-learner's policy (pi^a)

Network transfers are snapshot copies into one of two alternating buffers, written by the producer
at the end of its period and read in place by the consumers during the next one, so nobody waits for
a copy.  The events (one per part and period, plus one after the V-learner's push) express exactly
these hand-overs; a part that is ahead waits there, which is the ratio control of Section 3.2.

`concurrent=False` enqueues the same calls in the same logical order on a single stream; both modes
compute bit-identical results.
"""
from __future__ import annotations

from typing import List, Optional

from . import binding as B
from .session import LearnerSession


class ParallelSchemeSession:
    def __init__(self, sess: LearnerSession, env_rows: List[dict], horizon: int = 1, v_updates: int = 8,
                 p_updates: int = 4, concurrent: bool = True):
        import torch
        self.torch, self.s, self.w = torch, sess, sess.w
        self.env = env_rows                       # device-resident synthetic simulator output, cycled
        self.horizon, self.v_updates, self.p_updates = int(horizon), int(v_updates), int(p_updates)
        self.concurrent = concurrent
        # With the follow-ups folded into the optimiser kernels (LearnerSession.fold_followups) the Polyak step
        # of Q' rides on every critic update; the lagged policy, however, follows pi only at the period
        # boundaries here, through the snapshots below, so its per-update tracking is switched off.
        self.folded = bool(getattr(sess, "folded", False))
        if self.folded:
            sess.ctx.pql_track_attach(1, None, 0.0)
        dev = sess.device
        w = self.w
        self.pi_snap = [sess.actor.clone(), sess.actor.clone()]       # pi^a = pi^v: the P-learner's last hand-over
        self.q_snap = [sess.critic.clone(), sess.critic.clone()]      # Q^p: the V-learner's last hand-over
        # SAC variant: the temperature is learned by the P-learner and handed to the V-learner like the policy
        self.alpha_snap = None if sess.temperature is None else [sess.temperature.clone(), sess.temperature.clone()]
        nws = sess.workspace.numel()
        self.ws_p = torch.zeros(nws, dtype=torch.float32, device=dev)
        self.ws_a = torch.zeros(nws, dtype=torch.float32, device=dev)
        assert self.ws_p.data_ptr() % 256 == 0 and self.ws_a.data_ptr() % 256 == 0
        self.p_idx = torch.zeros(sess.max_batch, dtype=torch.int64, device=dev)
        self.p_obs = torch.zeros((sess.max_batch, w.obs_dim), dtype=torch.float32, device=dev)
        self.staged_act = [[torch.zeros((w.num_envs, w.act_dim), dtype=torch.float32, device=dev)
                            for _ in range(self.horizon)] for _ in range(2)]
        if concurrent:
            self.st_a, self.st_v, self.st_p = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        else:
            self.st_a = self.st_v = self.st_p = torch.cuda.current_stream()
        self.period = 0
        self.tick = 0                             # environment rows consumed so far
        self.staged_rows: List[List[dict]] = [[], []]
        self.ev_a: Optional[object] = None        # events of the previous period
        self.ev_p: Optional[object] = None
        start = torch.cuda.Event()
        start.record(torch.cuda.current_stream())
        for st in {self.st_a, self.st_v, self.st_p}:
            st.wait_event(start)

    def _event(self, stream):
        ev = self.torch.cuda.Event()
        ev.record(stream)
        return ev

    def run_period(self):
        s, w, c = self.s, self.w, self.s.ctx
        p = self.period
        cur, prev = p % 2, (p - 1) % 2
        st_a, st_v, st_p = self.st_a, self.st_v, self.st_p
        pi_lag, q_p = self.pi_snap[prev], self.q_snap[prev]

        # ---- boundary, V-learner's stream: receive the Actor's transitions of the last period
        if self.ev_p is not None:
            st_v.wait_event(self.ev_p)            # pi snapshot ready; the P-learner is done with the old Q snapshot
            st_v.wait_event(self.ev_a)            # staged actions ready; the Actor is done with the old pi snapshot
        for row, act in zip(self.staged_rows[prev], self.staged_act[prev]):
            c.pql_replay_push(s.storage, row["obs"], act, row["rew"], row["next_obs"], row["done"], st_v)
        ev_pushed = self._event(st_v)

        # ---- Actor (Algorithm 1): roll out pi^a
        if self.ev_p is not None:
            st_a.wait_event(self.ev_p)
        st_a.wait_event(ev_pushed)                # observation statistics; staging buffers free again
        rows = []
        for t in range(self.horizon):
            row = self.env[self.tick % len(self.env)]
            self.tick += 1
            c.pql_actor_act(pi_lag, row["obs"], w.num_envs, w.sigma_min, w.sigma_max, self.staged_act[cur][t],
                            self.ws_a, st_a)
            rows.append(row)
        self.staged_rows[cur] = rows
        ev_a = self._event(st_a)

        # ---- V-learner (Algorithm 3) and P-learner (Algorithm 2), enqueued interleaved so that
        #      neither stream runs dry while the host is busy with the other
        st_p.wait_event(ev_pushed)                # ring holds the new states; Q snapshot of the last period is complete
        if self.alpha_snap is not None:
            c.pql_sac_attach_lagged(self.alpha_snap[prev])
        done_p = 0
        for k in range(self.v_updates):
            c.pql_sample_nstep(s.storage, w.batch, s.batch, st_v)
            c.pql_critic_update(s.critic, s.critic_target, pi_lag, s.c_m, s.c_v, s.c_g, s.batch, w.batch, s.opt,
                                s.critic_out, s.workspace, st_v)
            if not self.folded:
                c.pql_soft_update(s.critic, s.critic_target, s.critic.numel(), w.tau, st_v)
            want_p = (self.p_updates * (k + 1)) // self.v_updates
            while done_p < want_p:
                self._policy_update(q_p, st_p)
                done_p += 1
        while done_p < self.p_updates:
            self._policy_update(q_p, st_p)
            done_p += 1
        # ---- hand-overs for the next period
        c.pql_soft_update(s.critic, self.q_snap[cur], s.critic.numel(), 1.0, st_v)
        c.pql_soft_update(s.actor, self.pi_snap[cur], s.actor.numel(), 1.0, st_p)
        if self.alpha_snap is not None:
            c.pql_soft_update(s.temperature, self.alpha_snap[cur], 4, 1.0, st_p)
        self.ev_a, self.ev_p = ev_a, self._event(st_p)
        self.period += 1

    def _policy_update(self, q_p, st_p):
        s, w, c = self.s, self.w, self.s.ctx
        c.pql_sample_states(s.storage, w.batch, self.p_idx, self.p_obs, st_p)
        c.pql_actor_update(s.actor, q_p, s.a_m, s.a_v, s.a_g, self.p_obs, w.batch, s.opt, s.actor_out, self.ws_p, st_p)

    def finish(self):
        """Makes the current stream wait for everything enqueued so far."""
        cur = self.torch.cuda.current_stream()
        for st in {self.st_a, self.st_v, self.st_p}:
            if st is not cur:
                cur.wait_event(self._event(st))
