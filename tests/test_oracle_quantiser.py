"""Pins for the oracle's p^alpha fixed-point quantiser: double-precision pow, exact special
cases, monotonicity, clamping.  Expected values come from Python's own arithmetic."""
import math

import numpy as np
import pytest

import oracle

F32 = np.float32
ALPHAS = [0.6, 0.0, 1.0, 0.3, 0.7, 0.5, -0.4]


def test_pow_spec_tracks_double_pow_over_the_whole_input_range():
    rng = np.random.default_rng(0)
    xs = np.exp2(rng.uniform(-100, 100, 20000)).astype(F32)
    xs = np.concatenate([xs, rng.lognormal(0, 2, 20000).astype(F32), (1 + rng.uniform(-1e-3, 1e-3, 2000)).astype(F32)])
    for alpha in ALPHAS:
        a32 = float(F32(alpha))
        worst = 0.0
        for x in xs:
            exact = math.pow(float(x), a32)
            worst = max(worst, abs(oracle.pow_spec(x, alpha) - exact) / exact)
        assert worst < 2e-7, (alpha, worst)     # under two fp32 ulps; the parity tolerance is 1e-5


def test_pow_spec_exact_cases():
    for alpha in ALPHAS:
        assert oracle.pow_spec(1.0, alpha) == 1.0
    for x in (1e-30, 0.3, 1.0, 7.0, 1e30):
        assert oracle.pow_spec(x, 0.0) == 1.0                       # alpha = 0: uniform replay
    for e in range(-100, 101):
        assert oracle.pow_spec(2.0 ** e, 1.0) == 2.0 ** e           # powers of two are exact
        if e % 2 == 0:
            assert oracle.pow_spec(2.0 ** e, 0.5) == 2.0 ** (e // 2)
            assert oracle.pow_spec(2.0 ** e, -0.5) == 2.0 ** (-e // 2)


def test_pow_spec_is_monotone_on_a_grid():
    for alpha in (0.3, 0.6, 1.0):
        xs = np.exp2(np.linspace(-40, 40, 40001)).astype(F32)
        ys = [oracle.pow_spec(x, alpha) for x in xs]
        assert all(b >= a for a, b in zip(ys, ys[1:]))
    ys = [oracle.pow_spec(x, -0.4) for x in np.exp2(np.linspace(-40, 40, 4001)).astype(F32)]
    assert all(b <= a for a, b in zip(ys, ys[1:]))


@pytest.mark.parametrize("alpha", [0.6, 0.3, 1.0])
def test_quantise_is_floor_of_scaled_power(alpha):
    rng = np.random.default_rng(1)
    eps, F = 1e-6, 24
    qm = oracle.qmax(1 << 21)
    for p in np.concatenate([rng.lognormal(0, 1, 3000), np.abs(rng.standard_normal(3000)), [0.0, 1e-9, 1e3]]):
        p = F32(p)
        q, clamped = oracle.quantise(p, alpha, eps, F, qm)
        x = float(F32(p) + F32(eps))
        exact = math.pow(x, float(F32(alpha)))
        assert not clamped
        assert abs(q / 2.0 ** F - exact) <= 1e-5 * exact + 2.0 ** -F
        assert oracle.quantise(-p, alpha, eps, F, qm)[0] == q        # priority is |delta|


def test_quantise_values_fixed_by_hand():
    # alpha = 1, eps = 0, powers of two: mass = p * 2^F exactly
    for e in range(-20, 10):
        assert oracle.quantise(2.0 ** e, 1.0, 0.0, 24, 1 << 41) == (1 << (24 + e), False)
    # alpha = 0: every transition weighs exactly 2^F
    for p in (0.0, 1e-3, 5.0, 1e20):
        assert oracle.quantise(p, 0.0, 1e-6, 24, 1 << 41) == (1 << 24, False)
    # zero TD error with the usual eps: (1e-6)^0.6 * 2^24 = 4214.2...
    q, c = oracle.quantise(0.0, 0.6, 1e-6, 24, 1 << 41)
    assert not c and q == math.floor(math.pow(float(F32(1e-6)), float(F32(0.6))) * 2 ** 24) == 4214


def test_quantise_truncates_toward_zero():
    # small masses, where the fp32 error of the power (1e-7 relative) cannot move the integer part
    alpha, eps, F = 0.6, 1e-6, 24
    seen = 0
    for i in range(1, 4000):
        p = F32(i * 1e-7)
        exact = math.pow(float(F32(p) + F32(eps)), float(F32(alpha))) * 2 ** F
        if 0.55 < exact - math.floor(exact) < 0.95:
            assert oracle.quantise(p, alpha, eps, F, 1 << 41)[0] == math.floor(exact)
            seen += 1
    assert seen > 500


def test_quantise_clamps_and_counts():
    qm = oracle.qmax(1 << 24)
    assert qm == 1 << 38 and oracle.qmax((1 << 24) + 1) == 1 << 37 and oracle.qmax(0) == 1 << 62
    assert oracle.quantise(1e30, 1.0, 0.0, 24, qm) == (qm, True)
    assert oracle.quantise(float("inf"), 0.6, 1e-6, 24, qm) == (qm, True)
    assert oracle.quantise(float("nan"), 0.6, 1e-6, 24, qm) == (1, True)
    assert oracle.quantise(1e-30, 1.0, 0.0, 24, qm) == (1, True)
    assert oracle.quantise(2.0 ** 14, 1.0, 0.0, 24, qm) == (qm, False)      # lands exactly on the bound
    assert oracle.quantise(2.0 ** 14 * 1.5, 1.0, 0.0, 24, qm) == (qm, True)
    # the bound keeps any full tree below 2^63
    for P in (8192, 1 << 21, (1 << 24) + (1 << 20)):
        assert P * oracle.qmax(P) < 1 << 63
