#!/usr/bin/env python3
"""Throughput of the PQL learner hot path on one MI355X.

One "step" is one V-learner critic update together with everything else on the hot path at
the paper's default rates (Table B.1 / Section 4: 8 critic updates per Actor step, one policy
update per 2 critic updates):

    every 8th step : pql_actor_act on N environments + pql_replay_push of that Actor step
    every step     : pql_sample_nstep + pql_critic_update + Polyak update of Q'
    every 2nd step : pql_actor_update + hard copy of the policy into the lagged policy pi^v

By default the Polyak update and the policy copy are performed by the optimiser kernel of the update they
follow (pql_track_attach) and the transposed weights of the backward pass are kept between calls
(pql_weight_cache_*); --plain-calls makes them the separate pql_soft_update calls / launches instead.

All inputs are synthetic and resident in HBM before the timed region starts.  Prints ONE JSON
line.  `value` = critic updates per second of that whole schedule.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2307_12983_amd import workloads as W  # noqa: E402
from paper_2307_12983_amd import profile_tools  # noqa: E402

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0
ACTOR_EVERY = 8                   # critic updates per Actor step (beta_a:v = 1:8)
POLICY_EVERY = 2                  # critic updates per policy update (beta_p:v = 1:2)


def flops_per_sample(w: W.Workload):
    """Algorithmic FLOPs (2 per multiply-add on weight matrices only)."""
    pc = sum(i * o for i, o in w.critic_dims())
    pa = sum(i * o for i, o in w.actor_dims())
    pc_first = w.critic_dims()[0][0] * w.critic_dims()[0][1]
    pa_first = w.actor_dims()[0][0] * w.actor_dims()[0][1]
    act_cols = w.act_dim * w.critic_dims()[0][1]
    target = 2 * pa + 2 * 2 * pc
    fwd = 2 * 2 * pc
    bwd = 2 * (2 * pc + 2 * (pc - pc_first))            # dW for all layers + dX for all but the first
    critic_update = target + fwd + bwd
    # policy update: policy fwd, twin critic fwd, critic dX down to the action columns, policy bwd
    actor_update = 2 * pa + 2 * 2 * pc + 2 * 2 * (pc - pc_first + act_cols) + 2 * pa + 2 * (pa - pa_first)
    return dict(critic_update=critic_update, actor_update=actor_update, act=2 * pa)


class Schedule:
    """Issues the hot-path calls of step i; device-side synthetic environment data is cycled."""

    def __init__(self, sess, env_rows):
        self.s, self.env, self.tick = sess, env_rows, 0

    def step(self, i):
        s, w = self.s, self.s.w
        if i % ACTOR_EVERY == 0:
            row = self.env[self.tick % len(self.env)]
            self.tick += 1
            act = s.act(row["obs"])
            s.ctx.pql_replay_push(s.storage, row["obs"], act, row["rew"], row["next_obs"], row["done"])
        s.sample(w.batch)
        s.critic_update(w.batch)
        s.soft_update_targets()
        if i % POLICY_EVERY == POLICY_EVERY - 1:
            s.actor_update(None, w.batch)
            s.sync_lagged_policy()


def cpu_baseline(w: W.Workload, fill_rows, env_rows_host, budget_s=20.0, parallel=False):
    """The float64 oracle on the host, same schedule, on a bounded number of steps."""
    from oracle import pql_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    ring = O.ReplayRing(w.rows, w.num_envs, w.obs_dim, w.act_dim)
    nz = O.ObsNormalizer(w.obs_dim, w.obs_norm_eps) if w.obs_norm else None
    for row in fill_rows:
        ring.push(row["obs"], row["act"], row["rew"], row["next_obs"], row["done"])
        if nz is not None:
            nz.update(row["obs"])
    actor, critic = W.init_networks(w)
    L = O.Learner(w.actor_dims(), w.critic_dims(), actor, critic, w.lr, w.gamma, w.tau, w.beta1, w.beta2, w.eps,
                  max_grad_norm=(w.max_grad_norm if w.max_grad_norm > 0 else None),
                  v_min=(w.v_min if w.num_atoms >= 2 else None), v_max=(w.v_max if w.num_atoms >= 2 else None),
                  sac=w.sac, log_alpha=float(np.log(np.float64(w.init_alpha))), target_entropy=w.target_entropy,
                  seed=w.rng_seed)
    done_steps, tick, acts = 0, 0, 0
    t0 = time.perf_counter()
    if parallel:
        S = O.ParallelScheme(L, ring, w.nstep, w.batch, w.rng_seed, w.sigma_min, w.sigma_max, normalizer=nz)
        while True:
            row = env_rows_host[S.period % len(env_rows_host)]
            S.run_period(lambda period, t, a: row, [row["obs"]])
            done_steps += S.v_updates
            el = time.perf_counter() - t0
            if el >= budget_s or done_steps >= 64:
                break
        return dict(value=done_steps / el, unit="updates/s", cores=int(threads), kind="oracle",
                    sample="%d periods of the same schedule at batch %d (numpy float64, %.1f s)" % (S.period, w.batch, el))
    while True:
        i = done_steps
        if i % ACTOR_EVERY == 0:
            row = env_rows_host[tick % len(env_rows_host)]
            tick += 1
            seen = row["obs"] if nz is None else nz.normalize(row["obs"])
            if w.sac:
                a = O.sac_actor_act(L.actor, w.actor_dims(), seen, w.rng_seed, acts)
            else:
                a = O.actor_act(L.actor, w.actor_dims(), seen, w.sigma_min, w.sigma_max, w.rng_seed, acts)
            acts += 1
            ring.push(row["obs"], a.astype(np.float32), row["rew"], row["next_obs"], row["done"])
            if nz is not None:
                nz.update(row["obs"])
        batch = O.gather_nstep(ring, O.sample_indices(ring, w.nstep, w.batch, w.rng_seed, i), w.nstep, w.gamma)
        if nz is not None:
            batch = O.normalize_batch(batch, nz)
        L.critic_update(batch)
        L.soft_update_targets()
        if i % POLICY_EVERY == POLICY_EVERY - 1:
            L.actor_update(batch["obs"])
            L.sync_lagged_policy()
        done_steps += 1
        el = time.perf_counter() - t0
        if done_steps % ACTOR_EVERY == 0 and (el >= budget_s or done_steps >= 64):
            break
    return dict(value=done_steps / el, unit="updates/s", cores=int(threads), kind="oracle",
                sample="%d steps of the same schedule at batch %d (numpy float64, %.1f s)" % (done_steps, w.batch, el))


def host_info():
    """What the CPU baseline ran on: model name, logical CPUs, the CPUs this process may use, BLAS threads."""
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    blas, threads = "unknown", 1
    try:
        from threadpoolctl import threadpool_info
        for p in threadpool_info():
            if p.get("user_api") == "blas":
                blas, threads = "%s %s" % (p.get("internal_api", "?"), p.get("version", "")), int(p.get("num_threads", 1))
    except Exception:
        pass
    return dict(cpu_model=model, os_cpu_count=os.cpu_count(), sched_affinity=len(os.sched_getaffinity(0)),
                blas=blas.strip(), blas_threads=threads)


def cpu_actions_per_s(w: W.Workload, obs, budget_s=3.0):
    """The oracle's Actor step (Section 3.3) on one row of N observations."""
    from oracle import pql_oracle as O
    actor, _ = W.init_networks(w)
    n, t0 = 0, time.perf_counter()
    while True:
        if w.sac:
            O.sac_actor_act(actor, w.actor_dims(), obs, w.rng_seed, n)
        else:
            O.actor_act(actor, w.actor_dims(), obs, w.sigma_min, w.sigma_max, w.rng_seed, n)
        n += 1
        el = time.perf_counter() - t0
        if el >= budget_s or n >= 50:
            return w.num_envs * n / el


def run_workload(w, args, steps, warmup, profile_steps, isolated, keep_rows, schedule="serial", variant=False):
    """Fills the ring, times `steps` steps of the schedule and one per-kernel event pass.  Returns the
    fields of the JSON line for this workload, plus the host copies the CPU baseline needs."""
    import torch
    from paper_2307_12983_amd.session import LearnerSession
    sess = LearnerSession(w)
    if not args.plain_calls:
        # the Polyak step of Q', the hard copy pi -> pi^v and the transposed weights of the next backward pass
        # are produced by the optimiser kernels of the updates (pql_track_attach, pql_weight_cache_*): same
        # results bit for bit, three small launches fewer per critic update and two per policy update
        sess.fold_followups()
    rng = W.data_rng(w)
    n_fill = args.fill_rows or w.rows
    keep = []                                   # host copy of the filled rows for the CPU baseline
    for r in range(n_fill):
        row = W.transition_rows(w, rng, 1)[0]
        sess.push(row)
        if keep_rows:
            keep.append(row)
    env_host = W.transition_rows(w, rng, 8)
    env_dev = [sess.to_device(r) for r in env_host]
    torch.cuda.synchronize()

    # One plain copy of known size (tau = 1 is a copy): the yardstick that scales the HBM byte
    # counters when this command runs under a counter-collecting profiler.  Outside the timed region.
    cal_src = torch.ones(profile_tools.CAL_COPY_FLOATS, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    sess.ctx.pql_soft_update(cal_src, cal_dst, cal_src.numel(), 1.0)
    torch.cuda.synchronize()
    # The same copy timed: the rate the memory system sustains for a plain stream (read + write), the
    # achievable ceiling next to the nominal HBM peak for the bandwidth-bound kernels.
    copy_ms = []
    for _ in range(3):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        sess.ctx.pql_soft_update(cal_src, cal_dst, cal_src.numel(), 1.0)
        ev1.record()
        torch.cuda.synchronize()
        copy_ms.append(ev0.elapsed_time(ev1))
    hbm_copy_gbs = 2.0 * 4.0 * cal_src.numel() / (min(copy_ms) * 1e-3) / 1e9
    del cal_src, cal_dst

    # The matrix cores' sustained rate on register operands (no memory): the achievable ceiling next
    # to the nominal peak.  Outside the timed region.
    probe_blocks, probe_iters = 256 * 8, 4096
    probe_out = torch.empty(probe_blocks * 256, dtype=torch.float32, device="cuda")
    sess.ctx.pql_probe_mfma(probe_out, probe_blocks, 64)
    torch.cuda.synchronize()
    probe_ms = []
    for _ in range(4):        # the best of a few launches: the first ones after an idle phase can run at a lower clock
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        sess.ctx.pql_probe_mfma(probe_out, probe_blocks, probe_iters)
        ev1.record()
        torch.cuda.synchronize()
        probe_ms.append(ev0.elapsed_time(ev1))
    mfma_ceiling = probe_blocks * 4 * 4 * probe_iters * 4096.0 / (min(probe_ms) * 1e-3) / 1e12
    del probe_out

    sched = Schedule(sess, env_dev)
    if schedule == "serial":
        for i in range(warmup):
            sched.step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(warmup, warmup + steps):
            sched.step(i)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # four more regions of the same length, untouched by `value`: the spread of the measurement
        rates = [steps / dt]
        nxt = warmup + steps
        for _ in range(max(1, args.repeats) - 1):
            nxt += (-nxt) % ACTOR_EVERY
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for i in range(nxt, nxt + steps):
                sched.step(i)
            torch.cuda.synchronize()
            rates.append(steps / (time.perf_counter() - t1))
            nxt += steps
    else:
        rates = None
        from paper_2307_12983_amd.scheme import ParallelSchemeSession
        ps = ParallelSchemeSession(sess, env_dev, horizon=1, v_updates=ACTOR_EVERY, p_updates=ACTOR_EVERY // POLICY_EVERY,
                                   concurrent=schedule == "parallel")
        for _ in range(warmup // ACTOR_EVERY):
            ps.run_period()
        ps.finish()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps // ACTOR_EVERY):
            ps.run_period()
        ps.finish()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / steps
    value = steps / dt

    # ---- isolated rates (same buffers): critic-only loop and the Actor step
    def timed(fn, reps):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / reps

    def critic_only():
        sess.sample(w.batch); sess.critic_update(w.batch); sess.soft_update_targets()
    t_act = timed(lambda: sess.act(env_dev[0]["obs"]), 100)
    t_critic = timed(critic_only, max(50, steps // 4)) if isolated else None
    t_actor_upd = timed(lambda: sess.actor_update(None, w.batch), max(50, steps // 8)) if isolated else None

    # ---- per-kernel durations from HIP events on the launch stream, same schedule
    sess.ctx.pql_profile_begin(4096 * 4)
    base = nxt if rates is not None else warmup + steps
    base += (-base) % ACTOR_EVERY
    for i in range(base, base + profile_steps):
        sched.step(i)
    torch.cuda.synchronize()
    stats = sess.ctx.pql_profile_end()
    gemm = [k for k in stats if k["flops"] > 0]            # the MFMA kernels (grouped GEMMs and fused row-tile kernels)
    tot_gemm_ms = sum(k["total_ms"] for k in gemm)
    tot_gemm_flops = sum(k["flops"] for k in gemm)
    dom = max(gemm, key=lambda k: k["total_ms"])
    achieved = dom["flops"] / (dom["total_ms"] * 1e-3) / 1e12
    # HBM bytes per launch of the dominant kernel: NOT measured in this run.  It is the figure stored by the
    # two counter passes whose commands the file names (profiles/), and is dropped (null) once a kernel source
    # has changed since, or for a variant (clipping and normalisation, distributional or stochastic networks,
    # another schedule), which runs other kernels.
    traffic_file = os.path.join(ROOT, "profiles", "bench_%s_traffic.txt" % w.name)
    traffic = None if variant else profile_tools.stored_traffic(traffic_file, dom["name"])
    fl = flops_per_sample(w)
    flops_step = w.batch * (fl["critic_update"] + fl["actor_update"] / POLICY_EVERY) + w.num_envs * fl["act"] / ACTOR_EVERY
    kernels = []
    for k in stats:
        e = dict(name=k["name"], launches=k["launches"], avg_us=1e3 * k["total_ms"] / k["launches"])
        if k["flops"] > 0:
            e["tflops"] = k["flops"] / (k["total_ms"] * 1e-3) / 1e12
        if k["bytes"] > 0:
            e["gbs"] = k["bytes"] / (k["total_ms"] * 1e-3) / 1e9
            e["hbm_frac"] = e["gbs"] / PEAK_HBM_GBS
        kernels.append(e)
    out = {
        "value": value, "unit": "updates/s", "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "config": {"workload": "%s-shaped: obs %d, act %d, %d envs, replay %d, batch %d, n=%d, MLP %s ELU fp32; "
                               "per critic update: sample + update + Polyak, policy update every %d, "
                               "Actor step + push every %d%s" % (w.name, w.obs_dim, w.act_dim, w.num_envs, w.capacity, w.batch,
                                                                w.nstep, list(w.hidden), POLICY_EVERY, ACTOR_EVERY,
                                                                "; observation standardisation and gradient clipping 0.5 on"
                                                                if args.paper_defaults else "")
                               + ("; distributional critics, %d atoms on (%g, %g)" % (w.num_atoms, w.v_min, w.v_max)
                                  if w.num_atoms >= 2 else "")
                               + ("; SAC variant (stochastic policy, learnable temperature)" if w.sac else ""),
                   "rows_filled": n_fill, "ring_bytes": n_fill * w.num_envs * (2 * w.obs_dim + w.act_dim + 2) * 4,
                   "schedule": schedule,
                   "followups": "separate launches" if args.plain_calls else "folded into the optimiser kernels"},
        "roofline": {"bound": "mfma", "kernel": dom["name"], "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS, "traffic": traffic,
                     "traffic_source": (None if traffic is None else
                                        "stored: profiles/%s (two rocprofv3 --pmc passes, not this run)" % os.path.basename(traffic_file)),
                     "avg_launch_us": 1e3 * dom["total_ms"] / dom["launches"], "launches": dom["launches"],
                     "achievable_peak": mfma_ceiling, "frac_of_achievable": achieved / mfma_ceiling,
                     "all_gemm_tflops": tot_gemm_flops / (tot_gemm_ms * 1e-3) / 1e12},
        "hbm": {"peak_gbs": PEAK_HBM_GBS, "copy_gbs": hbm_copy_gbs, "copy_frac": hbm_copy_gbs / PEAK_HBM_GBS,
                "copy_bytes": 8 * profile_tools.CAL_COPY_FLOATS},
        "mfma_util_pct": 100.0 * flops_step * value / (PEAK_FP32_MFMA_TFLOPS * 1e12),
        "actor_actions_per_s": w.num_envs / t_act,
        "actor_act_us": 1e6 * t_act,
        "kernels": kernels,
    }
    if rates is not None:
        # `value` is the first region (exactly `steps` steps after the warm-up); the others follow it directly
        out["repeats"] = {"n": len(rates), "values": rates, "median": sorted(rates)[len(rates) // 2],
                          "min": min(rates), "max": max(rates)}
    if isolated:
        out["critic_only_updates_per_s"] = 1.0 / t_critic
        out["critic_only_mfma_util_pct"] = 100.0 * w.batch * fl["critic_update"] / t_critic / (PEAK_FP32_MFMA_TFLOPS * 1e12)
        out["actor_update_per_s"] = 1.0 / t_actor_upd
    del sess, env_dev
    torch.cuda.empty_cache()
    return out, keep, env_host


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=800)
    ap.add_argument("--warmup", type=int, default=80)
    ap.add_argument("--workload", default="ant", choices=list(W.WORKLOADS))
    ap.add_argument("--fill-rows", type=int, default=0, help="ring rows to fill before timing (0 = all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=48)
    ap.add_argument("--paper-defaults", action="store_true",
                    help="switch on the two Table B.1 defaults that the five workloads leave off: observation "
                         "standardisation and gradient clipping at 0.5")
    ap.add_argument("--atoms", type=int, default=0,
                    help="distributional critics (PQL-D) with this many atoms on (-10, 10); the paper uses 51")
    ap.add_argument("--sac", action="store_true",
                    help="PQL + SAC: tanh-Gaussian policy, soft target, learnable temperature")
    ap.add_argument("--schedule", default="serial", choices=["serial", "parallel", "parallel-1stream"],
                    help="serial: every call on one stream, networks shared by all parts (default).  parallel: the "
                         "Actor, V-learner and P-learner on three streams with local network copies exchanged once "
                         "per Actor step (Section 3.1 / 3.2), same 1 : 8 : 4 rates.  parallel-1stream: that schedule "
                         "enqueued on one stream")
    ap.add_argument("--repeats", type=int, default=5,
                    help="timed regions of the serial schedule: the first one is `value`, the others (same length, "
                         "run directly after it) are reported as `repeats` to show the spread")
    ap.add_argument("--no-isolated", dest="isolated", action="store_false",
                    help="skip the extra loops that time the V-learner alone (sample + critic update + Polyak) and "
                         "the policy update alone")
    ap.add_argument("--plain-calls", action="store_true",
                    help="make the Polyak update, the policy copy and the weight transposes separate launches "
                         "(pql_soft_update after every update, transposes inside it) instead of folding them into "
                         "the optimiser kernels")
    ap.add_argument("--no-secondary", dest="secondary", action="store_false",
                    help="skip the second batch-8192 workload (humanoid-shaped) that the default run reports in "
                         "the `secondary` block")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if args.schedule != "serial" and (args.steps % ACTOR_EVERY or args.warmup % ACTOR_EVERY):
        print("--steps and --warmup must be multiples of %d for the parallel schedule" % ACTOR_EVERY, file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)

    w = W.WORKLOADS[args.workload]
    if args.paper_defaults:
        w = w.replace(max_grad_norm=0.5, obs_norm=True)
    if args.atoms >= 2:
        w = w.replace(num_atoms=args.atoms)
    if args.sac:
        w = w.replace(sac=True)
    variant = bool(args.paper_defaults or args.atoms or args.sac or args.schedule != "serial")
    res, keep, env_host = run_workload(w, args, args.steps, args.warmup, args.profile_steps, args.isolated,
                                       keep_rows=not args.no_cpu_baseline, schedule=args.schedule, variant=variant)
    out = {"metric": "V-learner critic updates/s at batch %d" % w.batch, "value": res.pop("value"), "unit": res.pop("unit"),
           "n_gpus": 1, "steps": res.pop("steps"), "warmup": res.pop("warmup"), "ms_per_step": res.pop("ms_per_step"),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic"}
    out.update(res)
    if args.secondary and args.workload == "ant" and not variant:
        # the other workload the metric's batch size names (humanoid-shaped, batch 8192), full ring, fewer steps
        w2 = W.WORKLOADS["humanoid"]
        r2, _, _ = run_workload(w2, args, 160, 16, 16, False, keep_rows=False)
        out["secondary"] = {"metric": "V-learner critic updates/s at batch %d" % w2.batch, "value": r2["value"],
                            "unit": r2["unit"], "steps": r2["steps"], "warmup": r2["warmup"], "ms_per_step": r2["ms_per_step"],
                            "config": r2["config"], "roofline": r2["roofline"], "mfma_util_pct": r2["mfma_util_pct"],
                            "actor_actions_per_s": r2["actor_actions_per_s"], "kernels": r2["kernels"],
                            "repeats": r2.get("repeats")}
    if not args.no_cpu_baseline:
        cb = cpu_baseline(w, keep, env_host, parallel=args.schedule != "serial")
        cb.update(host_info())
        cb["cores"] = cb["blas_threads"] if cb["blas_threads"] > 1 else cb["cores"]
        cb["actions_per_s"] = cpu_actions_per_s(w, env_host[0]["obs"])
        if w.name in ("tiny", "ant") and args.schedule == "serial":
            try:
                from threadpoolctl import threadpool_limits
                with threadpool_limits(limits=1):
                    one = cpu_baseline(w, keep, env_host, budget_s=8.0)
                cb["single_thread"] = {"value": one["value"], "unit": one["unit"], "cores": 1, "sample": one["sample"]}
            except ImportError:
                cb["single_thread"] = None
        out["cpu_baseline"] = cb
    print(json.dumps(out))


if __name__ == "__main__":
    main()
