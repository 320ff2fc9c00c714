"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, answers the size queries and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2307_12983_amd import binding as B
from paper_2307_12983_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "pql.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pql_[a-z_]+)\s*\(", text)))


def cfg_of(w, max_batch=None):
    return B.make_config(w.obs_dim, w.act_dim, w.num_envs, w.capacity, w.nstep, w.gamma, w.hidden,
                         max_batch or max(w.batch, w.num_envs), w.rng_seed)


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    names = header_functions()
    assert len(names) == 33 and sorted(B.EXPORTS) == names
    for n in names:
        assert getattr(lib, n) is not None


@pytest.mark.parametrize("name", list(W.WORKLOADS))
def test_size_queries(name):
    w = W.WORKLOADS[name]
    ctx = B.Context(cfg_of(w))
    assert ctx.replay_rows() == w.capacity // w.num_envs
    assert ctx.actor_param_count() == W.param_count(w.actor_dims())
    assert ctx.critic_param_count() == W.param_count(w.critic_dims())
    ws = ctx.workspace_bytes()
    assert ws > 0 and ws % 256 == 0
    # workspace grows with the batch bound
    assert B.Context(cfg_of(w, 2 * max(w.batch, w.num_envs))).workspace_bytes() > ws
    assert ctx.get_state() == [0] * 8
    ctx.close()


def test_create_rejects_bad_configs():
    lib = B.load_library()
    w = W.WORKLOADS["tiny"]
    h = C.c_void_p()
    assert lib.pql_create(None, C.byref(h)) == -2
    assert lib.pql_create(C.byref(cfg_of(w)), None) == -2
    for field, value in [("obs_dim", 0), ("act_dim", 0), ("num_envs", 0), ("nstep", 0), ("n_hidden", 0),
                         ("n_hidden", 9), ("gamma", 0.0), ("gamma", 1.5), ("max_batch", 0), ("capacity", 64 * 2)]:
        cfg = cfg_of(w)
        setattr(cfg, field, value)
        assert lib.pql_create(C.byref(cfg), C.byref(h)) == -1, field
        assert lib.pql_workspace_bytes(C.byref(cfg)) == -1, field
    cfg = cfg_of(w)
    cfg.hidden[1] = 2048                       # last hidden layer wider than the head kernel supports
    assert lib.pql_create(C.byref(cfg), C.byref(h)) == -1
    # a first hidden layer of 65536 columns is fine at a small batch bound, but not at 32768 rows: a quarter
    # of the batch times that row length leaves the 32-bit offsets of the weight-gradient kernel
    cfg = cfg_of(w)
    cfg.hidden[0] = 65536
    assert lib.pql_create(C.byref(cfg), C.byref(h)) == 0
    lib.pql_destroy(h)
    cfg.max_batch = 32768
    assert lib.pql_create(C.byref(cfg), C.byref(h)) == -1
    assert lib.pql_workspace_bytes(C.byref(cfg)) == -1


def test_argument_errors_are_caught_on_the_host_and_leave_state_unchanged():
    """Null pointers, oversize batches and bad scalars return before any kernel launch, so
    these calls are safe without a GPU."""
    w = W.WORKLOADS["tiny"]
    ctx = B.Context(cfg_of(w))
    lib = ctx.lib
    fake = 0x1000                               # never dereferenced: validation fails first
    st_null = B.PqlStorage(None, None, None, None, None)
    st = B.PqlStorage(fake, fake, fake, fake, fake)
    bt = B.PqlBatch(fake, fake, fake, fake, fake, fake)
    opt = B.PqlAdam(1e-3, 0.9, 0.999, 1e-8)
    assert lib.pql_replay_push(ctx.h, st_null, fake, fake, fake, fake, fake, None) == -2
    assert lib.pql_replay_push(ctx.h, st, fake, None, fake, fake, fake, None) == -2
    assert lib.pql_sample_nstep(ctx.h, st, 16, bt, None) == -3            # nothing pushed yet
    assert lib.pql_sample_nstep(ctx.h, st, w.batch + 1, bt, None) == -4
    assert lib.pql_sample_nstep(ctx.h, st, -1, bt, None) == -1
    assert lib.pql_gather_nstep(ctx.h, st, None, 4, bt, None) == -2
    assert lib.pql_actor_act(ctx.h, fake, fake, 0, 0.1, 0.1, fake, 0x1000, None) == -1
    assert lib.pql_actor_act(ctx.h, fake, fake, w.batch + 1, 0.1, 0.1, fake, 0x1000, None) == -4
    assert lib.pql_actor_act(ctx.h, fake, fake, 8, 0.1, 0.1, fake, 0x1010, None) == -6
    assert lib.pql_actor_act(ctx.h, None, fake, 8, 0.1, 0.1, fake, 0x1000, None) == -2
    assert lib.pql_critic_update(ctx.h, fake, fake, fake, fake, fake, fake, bt, w.batch + 1, opt, fake, 0x1000, None) == -4
    assert lib.pql_critic_update(ctx.h, fake, fake, fake, fake, fake, fake, bt, 0, opt, fake, 0x1000, None) == -1
    assert lib.pql_critic_update(ctx.h, fake, fake, None, fake, fake, fake, bt, 8, opt, fake, 0x1000, None) == -2
    bad = B.PqlAdam(1e-3, 1.0, 0.999, 1e-8)
    assert lib.pql_critic_update(ctx.h, fake, fake, fake, fake, fake, fake, bt, 8, bad, fake, 0x1000, None) == -1
    assert lib.pql_actor_update(ctx.h, fake, fake, fake, fake, fake, fake, 8, bad, fake, 0x1000, None) == -1
    assert lib.pql_actor_update(ctx.h, fake, fake, fake, fake, fake, None, 8, opt, fake, 0x1000, None) == -2
    assert lib.pql_actor_update(ctx.h, fake, fake, fake, fake, fake, fake, 8, opt, fake, 0x1008, None) == -6
    assert lib.pql_adam_step(ctx.h, fake, fake, fake, fake, 10, opt, 0, None) == -1
    assert lib.pql_adam_step(ctx.h, fake, None, fake, fake, 10, opt, 1, None) == -2
    assert lib.pql_adam_step(ctx.h, fake, fake, fake, fake, 10, bad, 1, None) == -1
    assert lib.pql_soft_update(ctx.h, fake, fake, 10, 1.5, None) == -1
    assert lib.pql_soft_update(ctx.h, fake, fake, -1, 0.5, None) == -1
    assert lib.pql_soft_update(ctx.h, None, fake, 10, 0.5, None) == -2
    assert lib.pql_soft_update(ctx.h, fake, fake, 10, 0.0, None) == 0      # tau = 0: nothing to do
    assert ctx.get_state() == [0] * 8
    assert "pql_" in ctx.last_error()


def test_state_roundtrip_and_validation():
    w = W.WORKLOADS["tiny"]
    ctx = B.Context(cfg_of(w))
    ctx.set_state([3, 10, 99, 7, 5, 4, 2, 0])
    assert ctx.get_state() == [3, 10, 99, 7, 5, 4, 2, 0]
    with pytest.raises(B.PqlError):
        ctx.set_state([w.rows, 0, 0, 0, 0, 0, 0, 0])
    with pytest.raises(B.PqlError):
        ctx.set_state([0, 0, -1, 0, 0, 0, 0, 0])
    assert ctx.get_state() == [3, 10, 99, 7, 5, 4, 2, 0]


def test_obs_norm_host_side():
    lib = B.load_library()
    w = W.WORKLOADS["tiny"]
    ctx = B.Context(cfg_of(w))
    n = ctx.obs_norm_bytes()
    # count, reserved, mean, m2 in double; mean32, rstd32 in float; one (mean, m2) pair per 64-row chunk
    assert n >= 8 * (2 * w.obs_dim + 2) + 8 * w.obs_dim + 16 * w.obs_dim * ((w.num_envs + 63) // 64)
    bad = cfg_of(w)
    bad.obs_dim = 0
    assert lib.pql_obs_norm_bytes(C.byref(bad)) == -1
    assert lib.pql_obs_norm_attach(ctx.h, C.c_void_p(0x1000 + 8), 1e-5) == -6         # misaligned
    assert lib.pql_obs_norm_attach(ctx.h, C.c_void_p(0x1000), -1.0) == -1             # negative eps
    assert lib.pql_obs_norm_reset(ctx.h, None) == -2                                   # nothing attached
    assert "no statistics block" in ctx.last_error()
    assert lib.pql_obs_norm_attach(ctx.h, None, 0.0) == 0                              # detach is always fine
    ctx.close()


def test_clipping_bound_is_validated_on_the_host():
    lib = B.load_library()
    w = W.WORKLOADS["tiny"]
    ctx = B.Context(cfg_of(w))
    p = C.c_void_p(0x1000)
    bad = B.PqlAdam(1e-3, 0.9, 0.999, 1e-8, -0.5)
    batch = B.PqlBatch(p, p, p, p, p, p)
    assert lib.pql_critic_update(ctx.h, p, p, p, p, p, p, batch, 8, bad, p, p, None) == -1
    assert lib.pql_actor_update(ctx.h, p, p, p, p, p, p, 8, bad, p, p, None) == -1
    clip = B.PqlAdam(1e-3, 0.9, 0.999, 1e-8, 0.5)
    assert lib.pql_adam_step(ctx.h, p, p, p, p, 16, clip, 1, None) == -1               # no scratch for the norm here
    assert ctx.get_state() == [0] * 8
    ctx.close()


def test_variant_switches_are_validated_on_the_host():
    lib = B.load_library()
    w = W.WORKLOADS["tiny"]
    h = C.c_void_p()

    def cfg(**kw):
        return B.make_config(w.obs_dim, w.act_dim, w.num_envs, w.capacity, w.nstep, w.gamma, w.hidden, 256, w.rng_seed, **kw)

    for bad in (dict(num_atoms=-1), dict(num_atoms=65), dict(num_atoms=51, v_min=1.0, v_max=1.0),
                dict(stochastic_policy=2), dict(stochastic_policy=1, num_atoms=51, v_min=-10.0, v_max=10.0)):
        assert lib.pql_create(C.byref(cfg(**bad)), C.byref(h)) == -1, bad
    # output widths follow the switches
    base = B.Context(cfg())
    dist = B.Context(cfg(num_atoms=51, v_min=-10.0, v_max=10.0))
    sac = B.Context(cfg(stochastic_policy=1))
    hl = w.hidden[-1]
    assert dist.critic_param_count() - base.critic_param_count() == 50 * (hl + 1)
    assert sac.actor_param_count() - base.actor_param_count() == w.act_dim * (hl + 1)
    assert dist.actor_param_count() == base.actor_param_count() and sac.critic_param_count() == base.critic_param_count()
    # the temperature belongs to the stochastic policy only, and updates refuse to run without it
    p = C.c_void_p(0x1000)
    assert lib.pql_sac_attach(base.h, p, -2.0) == -1
    assert lib.pql_sac_attach(sac.h, C.c_void_p(0x1004), -2.0) == -6
    opt = B.PqlAdam(1e-3, 0.9, 0.999, 1e-8, 0.0)
    batch = B.PqlBatch(p, p, p, p, p, p)
    assert lib.pql_critic_update(sac.h, p, p, p, p, p, p, batch, 8, opt, p, p, None) == -2
    assert lib.pql_actor_update(sac.h, p, p, p, p, p, p, 8, opt, p, p, None) == -2
    assert "temperature" in sac.last_error()
    for c in (base, dist, sac):
        c.close()


def test_state_sampling_and_probe_argument_errors():
    lib = B.load_library()
    w = W.WORKLOADS["tiny"]
    ctx = B.Context(cfg_of(w))
    p = C.c_void_p(0x1000)
    st = B.PqlStorage(p, p, p, p, p)
    assert lib.pql_sample_states(ctx.h, st, 16, p, p, None) == -3            # nothing pushed yet
    assert lib.pql_sample_states(ctx.h, st, 16, None, p, None) == -2
    assert lib.pql_sample_states(ctx.h, st, -1, p, p, None) == -1
    assert lib.pql_sample_states(ctx.h, st, max(w.batch, w.num_envs) + 1, p, p, None) == -4
    assert lib.pql_probe_mfma(ctx.h, None, 8, 8, None) == -2
    assert lib.pql_probe_mfma(ctx.h, p, 0, 8, None) == -1
    assert ctx.get_state() == [0] * 8
    ctx.close()


def test_static_scratch_variant_checks_arguments_and_size_on_the_host():
    """pql_critic_update_static: argument errors as pql_critic_update's, and a configuration whose
    workspace exceeds the library's fixed scratch array is refused before any device call."""
    lib = B.load_library()
    limit = lib.pql_static_scratch_bytes()
    assert limit == 64 << 20
    p = C.c_void_p(0x1000)
    batch = B.PqlBatch(p, p, p, p, p, p)
    opt = B.PqlAdam(1e-3, 0.9, 0.999, 1e-8, 0.0)
    small = B.Context(cfg_of(W.WORKLOADS["tiny"]))
    assert small.workspace_bytes() <= limit
    assert lib.pql_critic_update_static(small.h, p, p, None, p, p, p, batch, 8, opt, p, None) == -2
    assert lib.pql_critic_update_static(small.h, p, p, p, p, p, p, batch, 0, opt, p, None) == -1
    assert lib.pql_critic_update_static(small.h, p, p, p, p, p, p, batch, W.WORKLOADS["tiny"].batch + 1, opt, p, None) == -4
    assert small.get_state() == [0] * 8
    big = B.Context(cfg_of(W.WORKLOADS["humanoid"]))
    assert big.workspace_bytes() > limit
    assert lib.pql_critic_update_static(big.h, p, p, p, p, p, p, batch, 8, opt, p, None) == -7
    assert "static" in big.last_error() and str(limit) in big.last_error()
    assert big.get_state() == [0] * 8
    # the largest ant-shaped batch bound the header names
    w = W.WORKLOADS["ant"]
    assert B.Context(cfg_of(w, 3416)).workspace_bytes() <= limit < B.Context(cfg_of(w, 3417 + 31)).workspace_bytes()
    small.close(); big.close()


def test_workspace_view_offsets():
    lib = B.load_library()
    ctx = B.Context(cfg_of(W.WORKLOADS["ant"]))
    offs = [ctx.workspace_view(k) for k in range(3)]
    assert len(set(offs)) == 3 and all(o % 256 == 0 and 0 <= o < ctx.workspace_bytes() for o in offs)
    off = C.c_int64(0)
    assert lib.pql_workspace_view(C.byref(ctx.cfg), 3, C.byref(off)) == -1
    assert lib.pql_workspace_view(C.byref(ctx.cfg), 0, None) == -2
    ctx.close()


def test_followup_attachments_are_validated_on_the_host():
    lib = B.load_library()
    w = W.WORKLOADS["ant"]
    ctx = B.Context(cfg_of(w))
    p = C.c_void_p(0x1000)
    assert lib.pql_track_attach(ctx.h, 2, p, 0.5) == -1                       # unknown vector
    assert lib.pql_track_attach(ctx.h, 0, p, 1.5) == -1
    assert lib.pql_track_attach(ctx.h, 0, p, -0.1) == -1
    assert lib.pql_track_attach(ctx.h, 0, p, 0.05) == 0 and lib.pql_track_attach(ctx.h, 1, p, 1.0) == 0
    assert lib.pql_track_attach(ctx.h, 0, None, 7.0) == 0                     # detaching ignores tau
    n = ctx.weight_cache_bytes()
    # per critic: W_2^T (256 x 256), the action rows of W_1 (8 x 256), W_out (256 x 1); the policy's W_2^T, W_out^T
    assert n == 4 * (2 * (256 * 256 + 8 * 256 + 256) + 256 * 256 + 256 * 8)
    assert lib.pql_weight_cache_refresh(ctx.h, p, p, None) == -2              # nothing attached
    assert lib.pql_weight_cache_attach(ctx.h, C.c_void_p(0x1010)) == -6
    assert lib.pql_weight_cache_attach(ctx.h, None) == 0
    bad = cfg_of(w)
    bad.n_hidden = 0
    assert lib.pql_weight_cache_bytes(C.byref(bad)) == -1
    ctx.close()


def test_header_is_plain_c_and_the_ctypes_structures_have_its_layout(tmp_path):
    """include/pql.h must compile as C99 and as C++ on its own, and the binding's ctypes mirrors must have
    the header's sizes and field offsets (a program compiled against the header prints them)."""
    import shutil
    import subprocess
    gcc, gxx = shutil.which("gcc"), shutil.which("g++")
    if not gcc or not gxx:
        pytest.skip("no host C compiler")
    header = os.path.join(ROOT, "include", "pql.h")
    for cc, std, lang in ((gcc, "-std=c99", "c"), (gxx, "-std=c++11", "c++")):
        r = subprocess.run([cc, std, "-x", lang, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", header],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
    mirrors = {"pql_config": B.PqlConfig, "pql_replay_storage": B.PqlStorage, "pql_batch": B.PqlBatch,
               "pql_adam": B.PqlAdam, "pql_kernel_stat": B.PqlKernelStat}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "pql.h"', 'int main(void) {']
    for cname, cls in mirrors.items():
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (cname, cname))
        for field, _ in cls._fields_:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (cname, field, cname, field))
    lines.append('printf("PQL_MAX_HIDDEN %d\\n", PQL_MAX_HIDDEN); return 0; }')
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    r = subprocess.run([gcc, "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    got = dict(l.split() for l in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.splitlines())
    assert int(got["PQL_MAX_HIDDEN"]) == B.PQL_MAX_HIDDEN
    for cname, cls in mirrors.items():
        assert int(got[cname]) == C.sizeof(cls), cname
        for field, _ in cls._fields_:
            assert int(got["%s.%s" % (cname, field)]) == getattr(cls, field).offset, "%s.%s" % (cname, field)


def test_ctypes_prototypes_match_the_header():
    """Every prototype of include/pql.h against the binding's restype / argtypes: same number of parameters,
    scalars of the same width, structures by value of the mirrored class, pointers where the header has pointers."""
    text = open(os.path.join(ROOT, "include", "pql.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    protos = re.findall(r"\b(int32_t|int64_t|const\s+char\s*\*)\s*(pql_[a-z_]+)\s*\(([^)]*)\)\s*;", text)
    assert sorted(n for _, n, _ in protos) == sorted(B.EXPORTS)
    scalars = {"int32_t": C.c_int32, "int64_t": C.c_int64, "float": C.c_float}
    by_value = {"pql_replay_storage": B.PqlStorage, "pql_batch": B.PqlBatch, "pql_adam": B.PqlAdam}
    lib = B.load_library()

    def is_pointer(t):
        return t in (C.c_void_p, C.c_char_p) or isinstance(t, type) and issubclass(t, C._Pointer)

    for ret, name, params in protos:
        fn = getattr(lib, name)
        want_ret = C.c_char_p if "char" in ret else scalars[ret]
        assert fn.restype is want_ret, name
        plist = [p.strip() for p in params.split(",")] if params.strip() not in ("", "void") else []
        assert len(plist) == len(fn.argtypes), "%s: %d parameters in the header, %d in the binding" % (name, len(plist), len(fn.argtypes))
        for k, (p, t) in enumerate(zip(plist, fn.argtypes)):
            where = "%s parameter %d (%s)" % (name, k, p)
            if "*" in p or "[" in p:
                assert is_pointer(t), where
                continue
            base = [tok for tok in p.split() if tok != "const"][0]
            if base in by_value:
                assert t is by_value[base], where
            else:
                assert t is scalars[base], where


def test_a_plain_c_program_links_against_the_library(tmp_path):
    """The boundary from C itself (no Python, no torch): a C99 program includes the header, links libpql.so and
    calls the host-side queries; its answers must be those the binding gets."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if not gcc:
        pytest.skip("no host C compiler")
    w = W.WORKLOADS["tiny"]
    src = tmp_path / "client.c"
    src.write_text('''
#include <stdio.h>
#include <string.h>
#include "pql.h"
int main(void) {
    pql_config c;
    pql_ctx *ctx = NULL, *none = NULL;
    int64_t st[8];
    memset(&c, 0, sizeof(c));
    c.obs_dim = %d; c.act_dim = %d; c.num_envs = %d; c.capacity = %d; c.nstep = %d; c.gamma = 0.99f;
    c.n_hidden = 2; c.hidden[0] = %d; c.hidden[1] = %d; c.max_batch = %d; c.seed = 7;
    printf("%%d\\n", (int)pql_create(&c, &ctx));
    printf("%%lld %%lld %%lld %%lld\\n", (long long)pql_replay_rows(&c), (long long)pql_actor_param_count(&c),
           (long long)pql_critic_param_count(&c), (long long)pql_workspace_bytes(&c));
    printf("%%d %%lld\\n", (int)pql_get_state(ctx, st), (long long)st[1]);
    c.obs_dim = 0;
    printf("%%d %%d\\n", (int)pql_create(&c, &none), none == NULL);
    printf("%%s\\n", pql_last_error(NULL));
    return pql_destroy(ctx) == PQL_OK ? 0 : 1;
}
''' % (w.obs_dim, w.act_dim, w.num_envs, w.capacity, w.nstep, w.hidden[0], w.hidden[1], max(w.batch, w.num_envs)))
    libdir = os.path.dirname(B.LIB_PATH)
    exe = tmp_path / "client"
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                        "-L", libdir, "-l:libpql.so", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    run = subprocess.run([str(exe)], capture_output=True, text=True)
    assert run.returncode == 0, run.stderr
    out = run.stdout.splitlines()
    ctx = B.Context(cfg_of(w))
    assert out[0] == "0"
    assert [int(x) for x in out[1].split()] == [ctx.replay_rows(), ctx.actor_param_count(), ctx.critic_param_count(),
                                                ctx.workspace_bytes()]
    assert out[2] == "0 0" and out[3] == "-1 1" and out[4] == "null context"
    ctx.close()
