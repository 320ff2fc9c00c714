"""Thin ctypes binding over ``libpql.so`` (declared in ``include/pql.h``).

Argument marshalling only: every function here forwards device pointers
(``torch.Tensor.data_ptr()``) and sizes to the C entry point of the same name.  PyTorch is
used for device memory and streams, nothing else.  There is no CPU fallback: if the HIP
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpql.so")

PQL_MAX_HIDDEN = 8
ERRORS = {0: "PQL_OK", -1: "PQL_ERR_INVALID_ARG", -2: "PQL_ERR_NULL", -3: "PQL_ERR_NOT_ENOUGH_DATA",
          -4: "PQL_ERR_BATCH_TOO_LARGE", -5: "PQL_ERR_HIP", -6: "PQL_ERR_ALIGNMENT", -7: "PQL_ERR_SCRATCH_TOO_SMALL"}

# every symbol include/pql.h declares
EXPORTS = ["pql_create", "pql_destroy", "pql_replay_rows", "pql_actor_param_count", "pql_critic_param_count",
           "pql_workspace_bytes", "pql_last_error", "pql_get_state", "pql_set_state", "pql_replay_push",
           "pql_sample_nstep", "pql_gather_nstep", "pql_actor_act", "pql_critic_update", "pql_actor_update",
           "pql_soft_update", "pql_adam_step", "pql_profile_begin", "pql_profile_end",
           "pql_obs_norm_bytes", "pql_obs_norm_attach", "pql_obs_norm_reset", "pql_sample_states", "pql_sac_attach",
           "pql_sac_attach_lagged", "pql_probe_mfma", "pql_static_scratch_bytes", "pql_critic_update_static",
           "pql_workspace_view", "pql_track_attach", "pql_weight_cache_bytes", "pql_weight_cache_attach",
           "pql_weight_cache_refresh"]


class PqlConfig(C.Structure):
    _fields_ = [("obs_dim", C.c_int32), ("act_dim", C.c_int32), ("num_envs", C.c_int32), ("capacity", C.c_int64),
                ("nstep", C.c_int32), ("gamma", C.c_float), ("n_hidden", C.c_int32),
                ("hidden", C.c_int32 * PQL_MAX_HIDDEN), ("max_batch", C.c_int32), ("seed", C.c_uint64),
                ("num_atoms", C.c_int32), ("v_min", C.c_float), ("v_max", C.c_float), ("stochastic_policy", C.c_int32)]


class PqlStorage(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("obs", "act", "rew", "next_obs", "done")]


class PqlBatch(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("idx", "obs", "act", "ret", "next_obs", "boot")]


class PqlAdam(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("max_grad_norm", C.c_float)]


class PqlKernelStat(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("launches", C.c_int64), ("total_ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


class PqlError(RuntimeError):
    def __init__(self, code: int, msg: str = ""):
        self.code = code
        super().__init__("%s (%d) %s" % (ERRORS.get(code, "?"), code, msg))


_lib = None


def load_library() -> C.CDLL:
    """Loads libpql.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libpql.so is missing: build it with `python -m paper_2307_12983_amd.build` "
                           "(the HIP library is the only implementation)")
    # torch first: libpql.so must bind to the HIP runtime that torch has loaded (both carry the
    # soname libamdhip64.so.7); two runtimes in one process do not see each other's device state.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    P, I32, I64, F = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    cfgp = C.POINTER(PqlConfig)
    sig = {
        "pql_create": (I32, [cfgp, C.POINTER(P)]),
        "pql_destroy": (I32, [P]),
        "pql_replay_rows": (I64, [cfgp]),
        "pql_actor_param_count": (I64, [cfgp]),
        "pql_critic_param_count": (I64, [cfgp]),
        "pql_workspace_bytes": (I64, [cfgp]),
        "pql_workspace_view": (I32, [cfgp, I32, C.POINTER(I64)]),
        "pql_last_error": (C.c_char_p, [P]),
        "pql_get_state": (I32, [P, C.POINTER(I64)]),
        "pql_set_state": (I32, [P, C.POINTER(I64)]),
        "pql_replay_push": (I32, [P, PqlStorage, P, P, P, P, P, P]),
        "pql_sample_nstep": (I32, [P, PqlStorage, I32, PqlBatch, P]),
        "pql_gather_nstep": (I32, [P, PqlStorage, P, I32, PqlBatch, P]),
        "pql_sample_states": (I32, [P, PqlStorage, I32, P, P, P]),
        "pql_actor_act": (I32, [P, P, P, I32, F, F, P, P, P]),
        "pql_critic_update": (I32, [P, P, P, P, P, P, P, PqlBatch, I32, PqlAdam, P, P, P]),
        "pql_critic_update_static": (I32, [P, P, P, P, P, P, P, PqlBatch, I32, PqlAdam, P, P]),
        "pql_static_scratch_bytes": (I64, []),
        "pql_actor_update": (I32, [P, P, P, P, P, P, P, I32, PqlAdam, P, P, P]),
        "pql_soft_update": (I32, [P, P, P, I64, F, P]),
        "pql_adam_step": (I32, [P, P, P, P, P, I64, PqlAdam, I64, P]),
        "pql_profile_begin": (I32, [P, I32]),
        "pql_profile_end": (I32, [P, C.POINTER(PqlKernelStat), I32, C.POINTER(I32)]),
        "pql_obs_norm_bytes": (I64, [cfgp]),
        "pql_obs_norm_attach": (I32, [P, P, F]),
        "pql_obs_norm_reset": (I32, [P, P]),
        "pql_track_attach": (I32, [P, I32, P, F]),
        "pql_weight_cache_bytes": (I64, [cfgp]),
        "pql_weight_cache_attach": (I32, [P, P]),
        "pql_weight_cache_refresh": (I32, [P, P, P, P]),
        "pql_sac_attach": (I32, [P, P, F]),
        "pql_sac_attach_lagged": (I32, [P, P]),
        "pql_probe_mfma": (I32, [P, P, I32, I32, P]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def make_config(obs_dim, act_dim, num_envs, capacity, nstep, gamma, hidden: Sequence[int], max_batch, seed,
                num_atoms=0, v_min=0.0, v_max=0.0, stochastic_policy=0) -> PqlConfig:
    cfg = PqlConfig()
    cfg.obs_dim, cfg.act_dim, cfg.num_envs, cfg.capacity = obs_dim, act_dim, num_envs, capacity
    cfg.nstep, cfg.gamma, cfg.n_hidden, cfg.max_batch, cfg.seed = nstep, gamma, len(hidden), max_batch, seed
    for i, h in enumerate(hidden[:PQL_MAX_HIDDEN]):
        cfg.hidden[i] = int(h)
    cfg.num_atoms, cfg.v_min, cfg.v_max = int(num_atoms), float(v_min), float(v_max)
    cfg.stochastic_policy = int(stochastic_policy)
    return cfg


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    s = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    return s or None


class Storage:
    """Device tensors of the replay ring (caller-owned memory, allocated with torch)."""

    def __init__(self, rows, num_envs, obs_dim, act_dim, device="cuda"):
        import torch
        n = rows * num_envs
        self.obs = torch.zeros((n, obs_dim), dtype=torch.float32, device=device)
        self.act = torch.zeros((n, act_dim), dtype=torch.float32, device=device)
        self.rew = torch.zeros((n,), dtype=torch.float32, device=device)
        self.next_obs = torch.zeros((n, obs_dim), dtype=torch.float32, device=device)
        self.done = torch.zeros((n,), dtype=torch.float32, device=device)

    def c(self) -> PqlStorage:
        return PqlStorage(self.obs.data_ptr(), self.act.data_ptr(), self.rew.data_ptr(),
                          self.next_obs.data_ptr(), self.done.data_ptr())


class Batch:
    """Device tensors receiving one sampled n-step batch."""

    def __init__(self, batch, obs_dim, act_dim, device="cuda"):
        import torch
        self.idx = torch.zeros((batch,), dtype=torch.int64, device=device)
        self.obs = torch.zeros((batch, obs_dim), dtype=torch.float32, device=device)
        self.act = torch.zeros((batch, act_dim), dtype=torch.float32, device=device)
        self.ret = torch.zeros((batch,), dtype=torch.float32, device=device)
        self.next_obs = torch.zeros((batch, obs_dim), dtype=torch.float32, device=device)
        self.boot = torch.zeros((batch,), dtype=torch.float32, device=device)

    def c(self) -> PqlBatch:
        return PqlBatch(self.idx.data_ptr(), self.obs.data_ptr(), self.act.data_ptr(), self.ret.data_ptr(),
                        self.next_obs.data_ptr(), self.boot.data_ptr())


class Context:
    """Owns a ``pql_ctx`` and exposes the C entry points under their own names."""

    def __init__(self, cfg: PqlConfig):
        self.lib = load_library()
        self.cfg = cfg
        h = C.c_void_p()
        rc = self.lib.pql_create(C.byref(cfg), C.byref(h))
        if rc != 0:
            raise PqlError(rc, "pql_create")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.pql_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != 0:
            raise PqlError(rc, (self.lib.pql_last_error(self.h) or b"").decode())

    # ---- host queries
    def replay_rows(self) -> int:
        return self.lib.pql_replay_rows(C.byref(self.cfg))

    def actor_param_count(self) -> int:
        return self.lib.pql_actor_param_count(C.byref(self.cfg))

    def critic_param_count(self) -> int:
        return self.lib.pql_critic_param_count(C.byref(self.cfg))

    def workspace_bytes(self) -> int:
        return self.lib.pql_workspace_bytes(C.byref(self.cfg))

    def workspace_view(self, what: int) -> int:
        """Byte offset inside the workspace of y (0), Q_1 (1) or Q_2 (2) of the last update."""
        off = C.c_int64(0)
        self._check(self.lib.pql_workspace_view(C.byref(self.cfg), what, C.byref(off)))
        return off.value

    def obs_norm_bytes(self) -> int:
        return self.lib.pql_obs_norm_bytes(C.byref(self.cfg))

    def last_error(self) -> str:
        return (self.lib.pql_last_error(self.h) or b"").decode()

    def get_state(self):
        arr = (C.c_int64 * 8)()
        self._check(self.lib.pql_get_state(self.h, arr))
        return list(arr)

    def set_state(self, state):
        arr = (C.c_int64 * 8)(*state)
        self._check(self.lib.pql_set_state(self.h, arr))

    # ---- device calls
    def pql_replay_push(self, storage, obs, act, rew, next_obs, done, stream=None):
        self._check(self.lib.pql_replay_push(self.h, storage.c(), _ptr(obs), _ptr(act), _ptr(rew), _ptr(next_obs),
                                             _ptr(done), _stream(stream)))

    def pql_sample_nstep(self, storage, batch_size, out, stream=None):
        self._check(self.lib.pql_sample_nstep(self.h, storage.c(), batch_size, out.c(), _stream(stream)))

    def pql_sample_states(self, storage, batch_size, idx_out, obs_out, stream=None):
        self._check(self.lib.pql_sample_states(self.h, storage.c(), batch_size, _ptr(idx_out), _ptr(obs_out),
                                               _stream(stream)))

    def pql_gather_nstep(self, storage, idx, batch_size, out, stream=None):
        self._check(self.lib.pql_gather_nstep(self.h, storage.c(), _ptr(idx), batch_size, out.c(), _stream(stream)))

    def pql_actor_act(self, actor_params, obs, num, sigma_min, sigma_max, act_out, workspace, stream=None):
        self._check(self.lib.pql_actor_act(self.h, _ptr(actor_params), _ptr(obs), num, sigma_min, sigma_max,
                                           _ptr(act_out), _ptr(workspace), _stream(stream)))

    def pql_critic_update(self, critic_params, critic_target_params, actor_target_params, adam_m, adam_v, grads_out,
                          batch, batch_size, opt: PqlAdam, loss_out, workspace, stream=None):
        self._check(self.lib.pql_critic_update(self.h, _ptr(critic_params), _ptr(critic_target_params),
                                               _ptr(actor_target_params), _ptr(adam_m), _ptr(adam_v), _ptr(grads_out),
                                               batch.c(), batch_size, opt, _ptr(loss_out), _ptr(workspace),
                                               _stream(stream)))

    def pql_critic_update_static(self, critic_params, critic_target_params, actor_target_params, adam_m, adam_v,
                                 grads_out, batch, batch_size, opt: PqlAdam, loss_out, stream=None):
        self._check(self.lib.pql_critic_update_static(self.h, _ptr(critic_params), _ptr(critic_target_params),
                                                      _ptr(actor_target_params), _ptr(adam_m), _ptr(adam_v),
                                                      _ptr(grads_out), batch.c(), batch_size, opt, _ptr(loss_out),
                                                      _stream(stream)))

    def static_scratch_bytes(self) -> int:
        return self.lib.pql_static_scratch_bytes()

    def pql_actor_update(self, actor_params, critic_params, adam_m, adam_v, grads_out, obs, batch_size, opt: PqlAdam,
                         loss_out, workspace, stream=None):
        self._check(self.lib.pql_actor_update(self.h, _ptr(actor_params), _ptr(critic_params), _ptr(adam_m),
                                              _ptr(adam_v), _ptr(grads_out), _ptr(obs), batch_size, opt,
                                              _ptr(loss_out), _ptr(workspace), _stream(stream)))

    def pql_adam_step(self, params, grads, adam_m, adam_v, count, opt: PqlAdam, t, stream=None):
        self._check(self.lib.pql_adam_step(self.h, _ptr(params), _ptr(grads), _ptr(adam_m), _ptr(adam_v), count, opt, t,
                                           _stream(stream)))

    def pql_profile_begin(self, max_launches):
        self._check(self.lib.pql_profile_begin(self.h, max_launches))

    def pql_profile_end(self):
        arr = (PqlKernelStat * 64)()
        n = C.c_int32(0)
        self._check(self.lib.pql_profile_end(self.h, arr, 64, C.byref(n)))
        return [dict(name=arr[i].name.decode(), launches=arr[i].launches, total_ms=arr[i].total_ms,
                     flops=arr[i].flops, bytes=arr[i].bytes) for i in range(min(n.value, 64))]

    def pql_soft_update(self, src, dst, count, tau, stream=None):
        self._check(self.lib.pql_soft_update(self.h, _ptr(src), _ptr(dst), count, tau, _stream(stream)))

    def pql_obs_norm_attach(self, stats, eps):
        self._check(self.lib.pql_obs_norm_attach(self.h, _ptr(stats), eps))

    def pql_obs_norm_reset(self, stream=None):
        self._check(self.lib.pql_obs_norm_reset(self.h, _stream(stream)))

    def pql_track_attach(self, which, dst, tau):
        self._check(self.lib.pql_track_attach(self.h, which, _ptr(dst), tau))

    def weight_cache_bytes(self) -> int:
        return self.lib.pql_weight_cache_bytes(C.byref(self.cfg))

    def pql_weight_cache_attach(self, cache):
        self._check(self.lib.pql_weight_cache_attach(self.h, _ptr(cache)))

    def pql_weight_cache_refresh(self, critic_params, actor_params, stream=None):
        self._check(self.lib.pql_weight_cache_refresh(self.h, _ptr(critic_params), _ptr(actor_params), _stream(stream)))

    def pql_sac_attach(self, temperature, target_entropy):
        self._check(self.lib.pql_sac_attach(self.h, _ptr(temperature), target_entropy))

    def pql_sac_attach_lagged(self, log_alpha):
        self._check(self.lib.pql_sac_attach_lagged(self.h, _ptr(log_alpha)))

    def pql_probe_mfma(self, out, blocks, iters, stream=None):
        self._check(self.lib.pql_probe_mfma(self.h, _ptr(out), blocks, iters, _stream(stream)))
