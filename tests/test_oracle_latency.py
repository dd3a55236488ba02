"""Pins for oracle/latency.py: the numbers and identities the paper prints, the
agreement of the closed forms with a simulation of the model, brute force on two
workers, and a known-answer vector of the random number generator."""
import itertools
import math

import numpy as np
import pytest

from oracle import latency as ol

FIG = dict(lam=0.5, rho=0.5, eps=0.1, gamma=0.0, pe=0.05)      # parameters of Figs. 1-2, n = 8


def test_uncoded_limit_is_point_66():
    """Sec. III: for n = 8, p_e = 0.05 the sigma = 0 curve tends to (1-p_e)^n ~ 0.66."""
    v = ol.gc_cdf(1e4, 8, 0, **FIG)
    assert abs(v - 0.95 ** 8) < 1e-12 and abs(v - 0.66) < 0.005
    assert abs(ol.ngc_cdf(1e4, 8, 0, **FIG) - 0.95 ** 8) < 1e-12


def test_limits_grow_with_tolerance():
    """lim P(T<=t) = P(at most sigma failures)."""
    for s in range(0, 7):
        expect = sum(math.comb(8, k) * 0.05 ** k * 0.95 ** (8 - k) for k in range(s + 1))
        assert abs(ol.gc_cdf(1e4, 8, s, **FIG) - expect) < 1e-12
        assert abs(ol.ngc_cdf(1e4, 8, s, **FIG) - expect) < 1e-10


def test_erlang_cdf_against_scipy_and_poisson_identity():
    from scipy import stats
    for u in range(1, 9):
        for t in (0.3, 2.0, 7.5, 20.0):
            F = ol.layer_cdf(u, t, 0.5, 0.5, 0.1, 0.2)
            tau = t - (0.2 + 0.1 + u * 0.5)
            ref = stats.gamma.cdf(tau, a=u, scale=2.0) if tau > 0 else 0.0
            assert abs(F - ref) < 1e-12
    # Corollary 1's proof: at rho = 0, F_u - F_{u+1} = e^{-lam t} (lam t)^u / u!
    lam, t = 0.7, 3.1
    for u in range(1, 8):
        diff = ol.layer_cdf(u, t, lam, 0.0, 0.0, 0.0) - ol.layer_cdf(u + 1, t, lam, 0.0, 0.0, 0.0)
        assert abs(diff - math.exp(-lam * t) * (lam * t) ** u / math.factorial(u)) < 1e-14


def test_nested_code_with_one_layer_is_the_uncoded_scheme():
    for t in (1.0, 3.0, 9.0):
        assert abs(ol.ngc_cdf(t, 8, 0, **FIG) - ol.gc_cdf(t, 8, 0, **FIG)) < 1e-13


def test_corollary_matches_theorem_at_rho_zero():
    for kappa in range(0, 4):
        for t in (0.5, 2.0, 6.0):
            a = ol.ngc_conditional_cdf(t, 8, 3, kappa, 0.5, 0.0, 0.1, 0.0)
            b = ol.ngc_conditional_cdf_rho0(t, 8, 3, kappa, 0.5, 0.1, 0.0)
            assert abs(a - b) < 1e-12


def test_nested_code_is_never_slower_than_any_of_its_component_codes():
    for t in np.linspace(2, 18, 9):
        ngc = ol.ngc_cdf(t, 8, 3, **FIG)
        for sigma in range(4):
            assert ngc >= ol.gc_cdf(t, 8, sigma, **FIG) - 1e-12
    # Fig. 2's remark: s_max = 4 and s_max = 6 have almost equal characteristics
    assert max(abs(ol.ngc_cdf(t, 8, 4, **FIG) - ol.ngc_cdf(t, 8, 6, **FIG)) for t in np.linspace(2, 18, 9)) < 0.01


def test_two_workers_by_brute_force():
    """n = 2, s_max = 1: decodable iff both finished one task or one finished two."""
    lam, rho, eps, gamma, pe, t = 0.8, 0.3, 0.05, 0.1, 0.2, 2.5
    F1 = ol.layer_cdf(1, t, lam, rho, eps, gamma)
    F2 = ol.layer_cdf(2, t, lam, rho, eps, gamma)
    # states of one alive worker: 0, exactly 1, >= 2 tasks finished
    p = {0: 1 - F1, 1: F1 - F2, 2: F2}
    both = sum(p[a] * p[b] for a, b in itertools.product(p, repeat=2) if (a >= 1 and b >= 1) or a == 2 or b == 2)
    one = p[2]
    expect = (1 - pe) ** 2 * both + 2 * pe * (1 - pe) * one
    assert abs(ol.ngc_cdf(t, 2, 1, lam, rho, eps, gamma, pe) - expect) < 1e-14


def test_philox_known_answer():
    """Counter 0, key 0 -> 6627e8d5 e169c58d bc57ac4c 9b00dbd8 (Random123 test vector)."""
    out = ol.philox4x32([0], [0], [0], [0], 0, 0)
    assert [int(x[0]) for x in out] == [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]
    out = ol.philox4x32([0xFFFFFFFF], [0xFFFFFFFF], [0xFFFFFFFF], [0xFFFFFFFF], 0xFFFFFFFF, 0xFFFFFFFF)
    assert [int(x[0]) for x in out] == [0x408F276D, 0x41C83B0E, 0xA20BC7C6, 0x6D5451FD]


@pytest.mark.parametrize("smax", [0, 2, 3])
def test_simulation_agrees_with_closed_forms(smax):
    trials = 200000
    L = ol.simulate(trials, 8, smax, seed=11, **FIG)
    T_ngc = L.min(axis=1)
    for t in (3.0, 5.0, 8.0, 14.0):
        se = 3.5 * math.sqrt(0.25 / trials) + 1e-4
        assert abs(ol.empirical_cdf(T_ngc, t) - ol.ngc_cdf(t, 8, smax, **FIG)) < se
        for sigma in range(smax + 1):
            assert abs(ol.empirical_cdf(L[:, sigma], t) - ol.gc_cdf(t, 8, sigma, **FIG)) < se


def test_printed_summation_limit_disagrees_with_the_model():
    """The limit as printed in Theorem 1 lets configurations through in which a layer
    already has its finishers; the simulation sides with the proof's condition."""
    trials = 200000
    L = ol.simulate(trials, 8, 3, seed=5, **FIG)
    t = 6.0
    emp = ol.empirical_cdf(L.min(axis=1), t)
    good = ol.ngc_cdf(t, 8, 3, **FIG)
    printed = ol.ngc_cdf(t, 8, 3, printed_limits=True, **FIG)
    assert abs(emp - good) < 0.005
    assert abs(emp - printed) > 0.02
