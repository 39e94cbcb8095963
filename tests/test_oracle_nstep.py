"""Pins for the oracle's n-step priorities: hand-worked episodes, closed forms, special cases.

None of these call the oracle to produce the expected value.
"""
import numpy as np
import pytest

import oracle
from conftest import read_golden

F32 = np.float32


def run(qo, qt, ac, rw, dc, n, alpha=0.6, eps=1e-6, F=24):
    return oracle.nstep_priorities(qo, qt, ac, rw, dc, n, alpha, eps, F)


def test_hand_episode_dpg_form():
    g = read_golden("nstep_hand_episode.txt")
    n, T = int(g["n"][0]), int(g["T"][0])
    rw = np.array(g["reward"], F32)[None]
    dc = np.array(g["discount"], F32)[None]
    qo = np.array(g["dpg_q_online"], F32)[None, :, None]
    qt = np.array(g["dpg_q_target"], F32)[None, :, None]
    ac = np.zeros((1, T + n), np.int32)
    prio, ret, gacc, _ = run(qo, qt, ac, rw, dc, n)
    assert ret[0].tolist() == [float(v) for v in g["dpg_ret"]]
    assert gacc[0].tolist() == [float(v) for v in g["dpg_gacc"]]
    assert prio[0].tolist() == [float(v) for v in g["dpg_prio"]]


def test_hand_episode_dqn_form_with_argmax_ties():
    g = read_golden("nstep_hand_episode.txt")
    n, T = int(g["n"][0]), int(g["T"][0])
    rw = np.array(g["reward"], F32)[None]
    dc = np.array(g["discount"], F32)[None]
    qo = np.array([g["dqn_q_online_%d" % u] for u in range(T + n)], F32)[None]
    qt = np.array([g["dqn_q_target_%d" % u] for u in range(T + n)], F32)[None]
    ac = np.array(g["dqn_action"], np.int32)[None]
    prio, ret, gacc, _ = run(qo, qt, ac, rw, dc, n)
    assert prio[0].tolist() == [float(v) for v in g["dqn_prio"]]
    assert ret[0].tolist() == [float(v) for v in g["dpg_ret"]]      # same rewards/discounts


@pytest.mark.parametrize("n", [1, 3, 5, 8])
def test_constant_reward_geometric_series(n):
    # r = c, no termination: R = c (1 - gamma^n) / (1 - gamma), Gamma = gamma^n
    gamma, c, T, A = 0.99, 0.7, 20, 3
    L = T + n
    qo = np.zeros((2, L, A), F32)
    prio, ret, gacc, _ = run(qo, qo, np.zeros((2, L), np.int32), np.full((2, L), c, F32),
                             np.full((2, L), gamma, F32), n)
    np.testing.assert_allclose(ret, c * (1 - gamma ** n) / (1 - gamma), rtol=1e-6)
    np.testing.assert_allclose(gacc, gamma ** n, rtol=1e-6)
    np.testing.assert_allclose(prio, ret, rtol=0, atol=0)           # Q == 0 -> |delta| = R


def test_constant_value_no_reward():
    # q == v everywhere, r == 0: delta = (gamma^n - 1) v
    gamma, v, n, T, A = 0.9, 2.5, 4, 10, 5
    L = T + n
    qo = np.full((1, L, A), v, F32)
    prio, _, _, _ = run(qo, qo, np.ones((1, L), np.int32), np.zeros((1, L), F32), np.full((1, L), gamma, F32), n)
    np.testing.assert_allclose(prio, abs((gamma ** n - 1) * v), rtol=1e-6)


def test_one_step_is_textbook_double_q():
    # n = 1: delta = r + gamma * q_target(s', argmax_a q_online(s', a)) - q_online(s, a)
    rng = np.random.default_rng(3)
    S, T, A, gamma = 4, 30, 6, 0.97
    L = T + 1
    qo = rng.standard_normal((S, L, A)).astype(F32)
    qt = rng.standard_normal((S, L, A)).astype(F32)
    ac = rng.integers(0, A, (S, L)).astype(np.int32)
    rw = rng.standard_normal((S, L)).astype(F32)
    dc = np.where(rng.random((S, L)) < 0.2, 0.0, gamma).astype(F32)
    prio, ret, gacc, _ = run(qo, qt, ac, rw, dc, 1)
    exp = np.empty((S, T))
    for s in range(S):
        for t in range(T):
            a_star = int(np.argmax(qo[s, t + 1]))
            exp[s, t] = abs(float(rw[s, t]) + float(dc[s, t]) * float(qt[s, t + 1, a_star]) - float(qo[s, t, ac[s, t]]))
    np.testing.assert_allclose(prio, exp, rtol=1e-5, atol=1e-6)
    assert np.array_equal(ret, rw[:, :T]) and np.array_equal(gacc, dc[:, :T])


def test_same_network_bootstraps_with_the_max():
    # an actor holds one copy of the network: q_target is q_online, and the bootstrap is max_a q
    rng = np.random.default_rng(4)
    S, T, A, n = 3, 12, 7, 3
    L = T + n
    qo = rng.standard_normal((S, L, A)).astype(F32)
    rw = np.zeros((S, L), F32)
    dc = np.ones((S, L), F32)
    ac = np.zeros((S, L), np.int32)
    prio, _, _, _ = run(qo, qo, ac, rw, dc, n)
    exp = np.abs(qo[:, n:, :].max(-1) - qo[:, :T, 0])
    np.testing.assert_allclose(prio, exp, rtol=1e-6, atol=1e-7)


def test_truncation_ignores_everything_after_the_episode_end():
    # terminate at offset j < n: R = sum_{i<=j} gamma^i r, Gamma = 0, and rows after the end cannot matter
    gamma, n, T, A = 0.9, 5, 1, 2
    for j in range(n):
        L = T + n
        rw = np.arange(1, L + 1, dtype=F32)[None]
        dc = np.full((1, L), gamma, F32)
        dc[0, j] = 0.0
        qo = np.zeros((1, L, A), F32)
        qt = np.zeros((1, L, A), F32)
        ac = np.zeros((1, L), np.int32)
        base = run(qo, qt, ac, rw, dc, n)
        rw2, qo2, qt2 = rw.copy(), qo.copy(), qt.copy()
        rw2[0, j + 1:] = 1e30
        qo2[0, j + 1:] = 1e30
        qt2[0, j + 1:] = -1e30
        poisoned = run(qo2, qt2, ac, rw2, dc, n)
        exp_R = sum(gamma ** i * (i + 1) for i in range(j + 1))
        assert base[2][0, 0] == 0.0 and poisoned[2][0, 0] == 0.0
        np.testing.assert_allclose(base[1][0, 0], exp_R, rtol=1e-6)
        for a, b in zip(base[:3], poisoned[:3]):
            assert np.array_equal(a, b)


def test_random_against_the_written_out_sum():
    # the definition with explicit powers and products, in float64
    rng = np.random.default_rng(5)
    S, T, A, n, gamma = 5, 50, 18, 3, 0.99
    L = T + n
    qo = rng.standard_normal((S, L, A)).astype(F32)
    qt = rng.standard_normal((S, L, A)).astype(F32)
    ac = rng.integers(0, A, (S, L)).astype(np.int32)
    rw = rng.standard_normal((S, L)).astype(F32)
    dc = np.where(rng.random((S, L)) < 0.05, 0.0, gamma).astype(F32)
    prio, ret, gacc, fx = run(qo, qt, ac, rw, dc, n)
    d64, r64 = dc.astype(np.float64), rw.astype(np.float64)
    for s in range(S):
        for t in range(T):
            R = sum(np.prod(d64[s, t:t + j]) * r64[s, t + j] for j in range(n))
            G = np.prod(d64[s, t:t + n])
            a_star = int(np.argmax(qo[s, t + n]))
            delta = R + G * float(qt[s, t + n, a_star]) - float(qo[s, t, ac[s, t]])
            assert abs(ret[s, t] - R) <= 1e-5 * abs(R) + 1e-6
            assert abs(gacc[s, t] - G) <= 1e-6
            assert abs(prio[s, t] - abs(delta)) <= 1e-5 * abs(delta) + 1e-6
    # the fixed-point column is the quantiser applied to the fp32 priority
    qm = oracle.qmax(0)
    for s in range(S):
        for t in range(0, T, 7):
            assert int(fx[s, t]) == oracle.quantise(prio[s, t], 0.6, 1e-6, 24, qm)[0]


def test_streams_are_independent():
    rng = np.random.default_rng(6)
    S, T, A, n = 4, 9, 3, 3
    L = T + n
    args = [rng.standard_normal((S, L, A)).astype(F32), rng.standard_normal((S, L, A)).astype(F32),
            rng.integers(0, A, (S, L)).astype(np.int32), rng.standard_normal((S, L)).astype(F32),
            np.full((S, L), 0.99, F32)]
    full = run(*args, n)
    for s in range(S):
        one = run(*[a[s:s + 1] for a in args], n)
        for a, b in zip(full, one):
            assert np.array_equal(a[s:s + 1], b)
