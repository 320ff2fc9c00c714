"""Pins for the oracle's integer parts: generator, ring, index sampling, n-step fold.

None of these checks re-type the oracle's formulas: they use published known answers,
a list-of-rows model of the ring, closed forms on hand-built episodes and brute force.
"""
import os

import numpy as np
import pytest

from oracle import pql_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = O.philox4x32_10([np.array([c]) for c in v[0:4]], (v[4], v[5]))
        assert [int(o[0]) for o in out] == v[6:10]


def test_philox_vectorised_equals_elementwise():
    rng = np.random.default_rng(0)
    ctr = rng.integers(0, 2**32, size=(4, 257), dtype=np.uint64)
    out = O.philox4x32_10(list(ctr), (123, 456))
    for i in (0, 1, 100, 256):
        one = O.philox4x32_10([np.array([c[i]]) for c in ctr], (123, 456))
        assert [int(o[0]) for o in one] == [int(o[i]) for o in out]


def test_rng_words_streams_and_calls_differ():
    k = np.arange(16)
    a = O.rng_words(7, O.STREAM_SAMPLE, 0, k)
    b = O.rng_words(7, O.STREAM_ACT, 0, k)
    c = O.rng_words(7, O.STREAM_SAMPLE, 1, k)
    d = O.rng_words(7, O.STREAM_SAMPLE, 0, k)
    assert not np.array_equal(a[0], b[0]) and not np.array_equal(a[0], c[0])
    assert all(np.array_equal(x, y) for x, y in zip(a, d))
    # counter layout: word0 = k, word1 = stream, word2/3 = call; key = seed halves
    ref = O.philox4x32_10([np.array([5]), np.array([1]), np.array([9]), np.array([2])], (0xAABBCCDD, 0x11))
    got = O.rng_words((0x11 << 32) | 0xAABBCCDD, 1, (2 << 32) | 9, np.array([5]))
    assert [int(x[0]) for x in ref] == [int(x[0]) for x in got]


# ---------------------------------------------------------------- ring vs list-of-rows
def _coded_row(push_no, N, o, a):
    """Values that encode (push number, env, field, column) so any misplaced element shows."""
    env = np.arange(N, dtype=np.float32)[:, None]
    obs = push_no * 1000 + env * 10 + np.arange(o, dtype=np.float32)[None, :] * 0.01 + 0.1
    act = push_no * 1000 + env * 10 + np.arange(a, dtype=np.float32)[None, :] * 0.01 + 0.2
    nxt = push_no * 1000 + env * 10 + np.arange(o, dtype=np.float32)[None, :] * 0.01 + 0.3
    rew = (push_no * 1000 + env[:, 0] * 10 + 0.4).astype(np.float32)
    done = ((push_no + np.arange(N)) % 7 == 0).astype(np.float32)
    return obs.astype(np.float32), act.astype(np.float32), rew, nxt.astype(np.float32), done


@pytest.mark.parametrize("T,N", [(5, 3), (7, 4), (1, 2)])
def test_ring_push_matches_list_model(T, N):
    o, a = 3, 2
    ring = O.ReplayRing(T, N, o, a)
    model = []                                   # chronological list of rows, newest last
    for p in range(int(2.5 * T) + 2):
        row = _coded_row(p, N, o, a)
        ring.push(*row)
        model.append(row)
        model = model[-T:]
        assert ring.count == len(model)
        for j, (mo, ma, mr, mn, md) in enumerate(model):
            pr = ring.physical_row(j)
            sl = slice(pr * N, (pr + 1) * N)
            assert np.array_equal(ring.obs[sl], mo) and np.array_equal(ring.act[sl], ma)
            assert np.array_equal(ring.rew[sl], mr) and np.array_equal(ring.next_obs[sl], mn)
            assert np.array_equal(ring.done[sl], md)


# ---------------------------------------------------------------- index sampling
def _filled_ring(T, N, pushes, o=2, a=1):
    ring = O.ReplayRing(T, N, o, a)
    for p in range(pushes):
        ring.push(*_coded_row(p, N, o, a))
    return ring


@pytest.mark.parametrize("T,N,pushes,n", [(7, 4, 3, 3), (7, 4, 7, 3), (7, 4, 18, 3), (10, 5, 23, 5), (6, 3, 40, 1)])
def test_sampled_windows_are_valid_and_never_cross_the_write_head(T, N, pushes, n):
    ring = _filled_ring(T, N, pushes)
    idx = O.sample_indices(ring, n, 4000, seed=11, call=3)
    assert idx.dtype == np.int64 and idx.min() >= 0 and idx.max() < T * N
    row0, env = idx // N, idx % N
    # chronological position of the start row
    j = (row0 - (ring.head - ring.count)) % T
    assert j.max() <= ring.count - n and j.min() >= 0
    # the push number is encoded in the stored reward: windows must be n consecutive pushes
    first = pushes - ring.count
    for k in range(n):
        slot = ((row0 + k) % T) * N + env
        push_no = np.floor(ring.rew[slot] / 1000.0)
        assert np.array_equal(push_no, first + j + k)
    # every valid start is reachable
    assert len(np.unique(j * N + env)) == (ring.count - n + 1) * N


def test_sampling_is_uniform_chi_square():
    ring = _filled_ring(6, 4, 6)
    n = 3
    V = (6 - n + 1) * 4
    idx = np.concatenate([O.sample_indices(ring, n, 4096, seed=5, call=c) for c in range(8)])
    j = ((idx // 4) - (ring.head - ring.count)) % 6
    cnt = np.bincount(j * 4 + idx % 4, minlength=V).astype(np.float64)
    exp = idx.size / V
    chi2 = ((cnt - exp) ** 2 / exp).sum()
    assert chi2 < 45.0                            # 15 dof: P(chi2 > 45) ~ 8e-5


def test_sampling_degenerate_single_window_and_errors():
    ring = _filled_ring(5, 1, 3)
    idx = O.sample_indices(ring, 3, 50, seed=1, call=0)
    assert np.all(idx == idx[0]) and idx[0] == ring.physical_row(0)
    with pytest.raises(ValueError):
        O.sample_indices(_filled_ring(5, 2, 2), 3, 4, seed=1, call=0)


def test_sampling_scaling_matches_big_integer_definition():
    """floor(u * V / 2^64) recomputed from the raw generator words with exact fractions."""
    from fractions import Fraction
    ring = _filled_ring(9, 7, 9)
    n, B = 2, 64
    idx = O.sample_indices(ring, n, B, seed=99, call=4)
    w = O.rng_words(99, O.STREAM_SAMPLE, 4, np.arange(B))
    V = (9 - n + 1) * 7
    for k in range(B):
        u = Fraction(int(w[1][k]) * 2**32 + int(w[0][k]), 2**64)     # uniform in [0,1)
        p = int(u * V)
        assert idx[k] == ring.physical_row(p // 7) * 7 + p % 7


# ---------------------------------------------------------------- n-step fold
def _episode_ring(T, rewards, dones, pushes_before=0):
    """One environment; obs value = push number so gathered rows identify themselves."""
    ring = O.ReplayRing(T, 1, 1, 1)
    for p in range(pushes_before):
        ring.push(np.full((1, 1), -1.0), np.zeros((1, 1)), np.zeros(1), np.zeros((1, 1)), np.zeros(1))
    for p, (r, d) in enumerate(zip(rewards, dones)):
        ring.push(np.full((1, 1), float(p)), np.full((1, 1), p + 0.5), np.array([r]),
                  np.full((1, 1), p + 0.25), np.array([d]))
    return ring


@pytest.mark.parametrize("gamma", [0.99, 0.5])
@pytest.mark.parametrize("n", [1, 3, 5])
def test_nstep_closed_forms(n, gamma):
    L = 8
    # no terminations, unit rewards: geometric sum and gamma^n
    ring = _episode_ring(L, [1.0] * L, [0.0] * L)
    out = O.gather_nstep(ring, np.array([0, 2]), n, gamma)
    assert np.allclose(out["ret"], (1 - gamma**n) / (1 - gamma), rtol=1e-13)
    assert np.allclose(out["boot"], gamma**n, rtol=1e-13)
    assert out["obs"][:, 0].tolist() == [0.0, 2.0]
    assert out["act"][:, 0].tolist() == [0.5, 2.5]
    assert out["next_obs"][:, 0].tolist() == [n - 1 + 0.25, n + 1 + 0.25]
    # termination at window step k: rewards up to and including k count, nothing after
    for k in range(n):
        dones = [0.0] * L
        dones[1 + k] = 1.0
        ring = _episode_ring(L, [1.0] * L, dones)
        out = O.gather_nstep(ring, np.array([1]), n, gamma)
        assert np.allclose(out["ret"], (1 - gamma**(k + 1)) / (1 - gamma), rtol=1e-13)
        assert out["boot"][0] == 0.0


def test_nstep_one_step_td_and_distinct_rewards():
    ring = _episode_ring(6, [3.0, -2.0, 5.0, 7.0, 11.0, 13.0], [0, 1, 0, 0, 0, 0])
    out = O.gather_nstep(ring, np.array([0, 1, 2]), 1, 0.9)
    assert np.allclose(out["ret"], [3.0, -2.0, 5.0]) and np.allclose(out["boot"], [0.9, 0.0, 0.9])
    out = O.gather_nstep(ring, np.array([2]), 3, 0.9)
    assert np.isclose(out["ret"][0], 5.0 + 0.9 * 7.0 + 0.81 * 11.0, rtol=1e-14)
    out = O.gather_nstep(ring, np.array([0]), 3, 0.9)       # done at the 2nd step masks the 3rd
    assert np.isclose(out["ret"][0], 3.0 + 0.9 * -2.0, rtol=1e-14) and out["boot"][0] == 0.0


def test_nstep_window_wraps_around_the_ring_end():
    # 4-row ring, 6 pushes: chronological rows are pushes 2..5, physical rows 2,3,0,1
    ring = _episode_ring(4, [1, 2, 3, 4, 5, 6], [0] * 6)
    assert ring.head == 2 and ring.count == 4
    start = ring.physical_row(1)                  # push 3 lives in physical row 3
    out = O.gather_nstep(ring, np.array([start]), 3, 0.5)
    assert out["obs"][0, 0] == 3.0 and out["next_obs"][0, 0] == 5.25
    assert np.isclose(out["ret"][0], 4 + 0.5 * 5 + 0.25 * 6)


def test_nstep_env_column_is_respected():
    ring = O.ReplayRing(4, 3, 1, 1)
    for p in range(4):
        ring.push(np.arange(3, dtype=np.float32)[:, None] + 10 * p, np.zeros((3, 1)),
                  np.array([1.0, 10.0, 100.0]) * (p + 1), np.zeros((3, 1)), np.zeros(3))
    out = O.gather_nstep(ring, np.array([0 * 3 + 1, 1 * 3 + 2]), 2, 1.0)
    assert np.allclose(out["ret"], [10 + 20, 200 + 300])
    assert out["obs"][:, 0].tolist() == [1.0, 12.0]
