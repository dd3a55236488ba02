"""Property pins for the oracle on randomly drawn small codes (hypothesis): Def. 1 by brute
force over every tolerated straggler set, Def. 2, exact recovery of the sum of the partial
gradients from every sufficient layer, agreement of the library's host-side selection with the
oracle's on the same code, and the latency model's closed forms on random parameters."""
import itertools

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import codes, coding


@st.composite
def small_nested_code(draw):
    n = draw(st.integers(min_value=2, max_value=8))
    extra = draw(st.sets(st.integers(min_value=1, max_value=n - 1), max_size=3))
    layers = [0] + sorted(extra)
    seed = draw(st.integers(min_value=0, max_value=2 ** 16))
    return n, layers, seed


@settings(max_examples=30, deadline=None)
@given(small_nested_code())
def test_every_tolerated_straggler_set_decodes_to_the_plain_sum(case):
    n, layers, seed = case
    Bs = codes.nested_code(n, layers, "cyclic", seed=seed, draws=2)
    rng = np.random.default_rng(seed)
    G = rng.standard_normal((n, 5))
    full = G.sum(axis=0)
    for u, (B, sigma) in enumerate(zip(Bs, layers)):
        assert np.count_nonzero(B, axis=1).tolist() == [sigma + 1] * n          # load (k/n)(sigma+1)
        if u:
            assert np.all((Bs[u - 1] != 0) <= (B != 0))                         # Def. 2
        C = coding.encode(B, G)
        for s in range(sigma + 1):
            for out in itertools.combinations(range(n), s):
                mask = np.zeros(n, np.uint8)
                mask[list(out)] = 1
                a, resid = coding.decode_vector(B, mask)
                assert resid < 1e-8 and np.all(a[mask == 1] == 0.0)
                assert np.allclose(coding.decode(a, C), full, rtol=0, atol=1e-7 * (1 + np.abs(a).sum()))
    # the layer rule picks the cheapest sufficient layer
    for s in range(n + 1):
        mask = np.zeros(n, np.uint8)
        mask[:s] = 1
        if s > layers[-1]:
            try:
                coding.select_layer(layers, mask)
                raise AssertionError("more stragglers than the code tolerates must not decode")
            except coding.Undecodable:
                pass
        else:
            u = coding.select_layer(layers, mask)
            assert layers[u] >= s and (u == 0 or layers[u - 1] < s)


@settings(max_examples=20, deadline=None)
@given(small_nested_code(), st.integers(min_value=0, max_value=2 ** 16))
def test_library_selection_agrees_with_the_oracle_on_the_same_code(ngc, case, mask_seed):
    n, layers, seed = case
    Bs = codes.nested_code(n, layers, "cyclic", seed=seed, draws=2)
    ctx = ngc.ngc_create(n, n, layers, 8)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        rng = np.random.default_rng(mask_seed)
        for _ in range(6):
            mask = (rng.random(n) < 0.3).astype(np.uint8)
            try:
                u_o = coding.select_layer(layers, mask)
            except coding.Undecodable:
                try:
                    ngc.ngc_select_decode_vec(ctx, mask, n)
                    raise AssertionError("the library decoded what the oracle calls undecodable")
                except ngc.NgcError as e:
                    assert e.code == ngc.NGC_ERR_UNDECODABLE
                continue
            a_o, _ = coding.decode_vector(Bs[u_o], mask)
            u, a, resid = ngc.ngc_select_decode_vec(ctx, mask, n)
            assert u == u_o and resid < 1e-8
            assert np.array_equal(a != 0, a_o != 0)
            assert np.allclose(a, a_o, rtol=0, atol=1e-8 * (1 + np.abs(a_o).max()))
    finally:
        ngc.ngc_destroy(ctx)


# ---- latency model: the library's dynamic programme against the oracle's nested sum, and the
# ---- properties any latency distribution of Sec. IV must have -----------------------------------
@settings(max_examples=60, deadline=None)
@given(st.integers(2, 7), st.data())
def test_latency_closed_forms_on_random_parameters(ngc, n, data):
    from oracle import latency as ol
    smax = data.draw(st.integers(0, n - 1))
    lam = data.draw(st.floats(0.2, 3.0))
    rho = data.draw(st.floats(0.0, 1.0))
    eps = data.draw(st.floats(0.0, 0.5))
    gamma = data.draw(st.floats(0.0, 0.5))
    pe = data.draw(st.floats(0.0, 0.4))
    ts = np.linspace(gamma + eps, gamma + eps + (smax + 1) * (rho + 6.0 / lam), 9)
    nested = ngc.ngc_latency_cdf_ngc(n, smax, lam, rho, eps, gamma, pe, ts)
    nested_o = np.array([ol.ngc_cdf(t, n, smax, lam, rho, eps, gamma, pe) for t in ts])
    assert np.allclose(nested, nested_o, rtol=1e-9, atol=1e-12)
    assert np.all(np.diff(nested) >= -1e-12) and nested[0] <= 1e-12 and nested[-1] <= 1.0 + 1e-12
    for sigma in range(smax + 1):
        fixed = ngc.ngc_latency_cdf_gc(n, sigma, lam, rho, eps, gamma, pe, ts)
        fixed_o = np.array([ol.gc_cdf(t, n, sigma, lam, rho, eps, gamma, pe) for t in ts])
        assert np.allclose(fixed, fixed_o, rtol=1e-9, atol=1e-12)
        # the nested code stops no later than any of its component codes (Sec. IV)
        assert np.all(nested >= fixed - 1e-9)
    # a code with a single layer sigma = 0 is the uncoded scheme: every worker must finish one task
    uncoded = ngc.ngc_latency_cdf_gc(n, 0, lam, rho, eps, gamma, pe, ts)
    F1 = np.array([ol.layer_cdf(1, t, lam, rho, eps, gamma) for t in ts])
    assert np.allclose(uncoded, (1.0 - pe) ** n * F1 ** n, rtol=1e-9, atol=1e-12)
