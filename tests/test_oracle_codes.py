"""Pins for oracle/codes.py and oracle/coding.py: Def. 1 by brute force, Def. 2,
Alg. 1's first layer, the fractional-repetition worked case, and the coding
invariant decode == sum of partial gradients for every straggler set."""
import itertools
import os

import numpy as np
import pytest

from oracle import codes, coding, gradients as og

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _masks(n, max_s):
    for s in range(max_s + 1):
        for out in itertools.combinations(range(n), s):
            m = np.zeros(n, np.uint8)
            m[list(out)] = 1
            yield m


@pytest.mark.parametrize("n,layers", [(6, [0, 1, 2, 3]), (8, [0, 1, 2, 3]), (8, [0, 1, 3, 7]),
                                      (7, [0, 2, 5])])
def test_cyclic_nested_code_satisfies_def1_and_def2(n, layers):
    Bs = codes.nested_code(n, layers, "cyclic", seed=3, draws=4)
    assert np.array_equal(Bs[0], np.eye(n))                       # Alg. 1: B_0 = I
    prev = None
    for B, sigma in zip(Bs, layers):
        supp = [set(np.flatnonzero(B[i])) for i in range(n)]
        for i in range(n):
            assert supp[i] == {(i + t) % n for t in range(sigma + 1)}   # Lemma 2: i and its sigma successors
            assert len(supp[i]) == sigma + 1                           # load (k/n)(sigma+1)
            if prev is not None:
                assert prev[i] <= supp[i]                              # Def. 2 nesting
        prev = supp
        # Def. 1: any n-sigma rows span an (n-sigma)-dim space containing 1.  The rank is counted
        # with an absolute threshold of 1e-9 on the singular values: the rows are solutions of
        # linear systems, accurate to about 1e-13 relative to entries of order 1..100, so a
        # singular value that should vanish comes out near 1e-12, while matrix_rank's default
        # threshold (largest singular value x dimension x 2.2e-16, here about 1e-13) sits right
        # at that noise level; the smallest singular value that should not vanish is above 1e-4
        # for these sizes, far from either threshold (the pins pass with the default as well).
        for out in itertools.combinations(range(n), sigma):
            S = [i for i in range(n) if i not in out]
            assert np.linalg.matrix_rank(B[S], tol=1e-9) == n - sigma
            assert np.linalg.matrix_rank(np.vstack([B[S], np.ones(n)]), tol=1e-9) == n - sigma
        # every straggler set of size <= sigma decodes: a B = 1, supp(a) in responders
        for m in _masks(n, sigma):
            a, resid = coding.decode_vector(B, m)
            assert resid < 1e-9
            assert np.all(a[m == 1] == 0.0)
            assert np.allclose(a @ B, 1.0, atol=1e-9)


def test_decoding_matrix_rows_times_B_is_all_ones():
    B = codes.nested_code(7, [0, 2], seed=1, draws=2)[1]
    A = codes.decoding_matrix(B, 2)
    assert A.shape == (21, 7)
    assert np.allclose(A @ B, 1.0, atol=1e-9)                       # Def. 1: A B = 1
    assert np.all((A != 0).sum(axis=1) <= 5)


def test_min_norm_equals_unique_solution_when_exactly_n_minus_sigma_respond():
    n, sigma = 9, 3
    B = codes.nested_code(n, [0, sigma], seed=5, draws=2)[1]
    for out in itertools.combinations(range(n), sigma):
        m = np.zeros(n, np.uint8)
        m[list(out)] = 1
        S = np.flatnonzero(m == 0)
        a, _ = coding.decode_vector(B, m)
        # independent route: normal equations of the consistent system B_S^T x = 1
        x = np.linalg.solve(B[S] @ B[S].T, B[S] @ np.ones(n))
        assert np.allclose(a[S], x, rtol=1e-6, atol=1e-8)
        a1, r1 = coding.decode_vector_first(B, sigma, m)
        assert np.allclose(a1, a, rtol=1e-6, atol=1e-8) and r1 < 1e-9


def test_first_responders_rule_is_supported_on_lowest_indices():
    n, sigma = 8, 3
    B = codes.nested_code(n, [0, sigma], seed=2, draws=2)[1]
    m = np.zeros(n, np.uint8)
    m[2] = 1                                  # one straggler, tolerance 3: 7 respond, 5 are used
    a, r = coding.decode_vector_first(B, sigma, m)
    assert r < 1e-9
    assert set(np.flatnonzero(a)) <= {0, 1, 3, 4, 5}


def test_fracrep_worked_case_matches_golden():
    Bs = codes.nested_code(4, [0, 1], "fracrep")
    assert np.array_equal(Bs[1], np.array([[1, 1, 0, 0], [1, 1, 0, 0],
                                           [0, 0, 1, 1], [0, 0, 1, 1.0]]))
    seen = 0
    with open(os.path.join(GOLD, "fracrep_n4.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            tok = line.split()
            mask = np.array([int(c) for c in tok[0]], np.uint8)
            u = coding.select_layer([0, 1], mask)
            assert u == int(tok[1])
            a, r = coding.decode_vector(Bs[u], mask)
            assert np.allclose(a, [float(t) for t in tok[2:6]], atol=1e-12) and r < 1e-12
            seen += 1
    assert seen == 5


def test_fracrep_weights_are_one_over_responders_in_block():
    n, sigma = 12, 3
    B = codes.fracrep_code(n, sigma)
    rng = np.random.default_rng(0)
    for _ in range(50):
        m = np.zeros(n, np.uint8)
        m[rng.choice(n, size=rng.integers(0, sigma + 1), replace=False)] = 1
        a, r = coding.decode_vector(B, m)
        for i in range(n):
            blk = codes.fracrep_support(n, sigma, i)
            alive = sum(1 for j in blk if m[j] == 0)
            assert np.isclose(a[i], 0.0 if m[i] else 1.0 / alive, atol=1e-12)


def test_fracrep_nesting_rule():
    codes.nested_code(8, [0, 1, 3, 7], "fracrep")
    with pytest.raises(ValueError):
        codes.nested_code(20, [0, 1, 4], "fracrep")       # 2 does not divide 5


def test_select_layer_table():
    layers = [0, 1, 3, 7]
    expect = {0: 0, 1: 1, 2: 2, 3: 2, 4: 3, 5: 3, 6: 3, 7: 3}
    for s in range(17):
        m = np.zeros(16, np.uint8)
        m[:s] = 1
        if s in expect:
            assert coding.select_layer(layers, m) == expect[s]
        else:
            with pytest.raises(coding.Undecodable):
                coding.select_layer(layers, m)


def _c1_like(n=4, rows=16, d=5, seed=0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, rows, d))
    th_star = rng.standard_normal(d)
    Y = X @ th_star + 0.01 * rng.standard_normal((n, rows))
    return X, Y, rng.standard_normal(d)


def test_decode_equals_sum_of_partial_gradients_for_all_16_subsets_of_n4():
    X, Y, th = _c1_like()
    G = og.partial_gradients(0, X, Y, th)
    full = og.lsq_gradient(X.reshape(-1, 5), Y.reshape(-1), th)
    layers = [0, 1]
    for kind in ("fracrep", "cyclic"):
        Bs = codes.nested_code(4, layers, kind, seed=0, draws=2)
        ok = bad = 0
        for bits in range(16):
            m = np.array([(bits >> i) & 1 for i in range(4)], np.uint8)
            try:
                u, a, g = coding.coded_gradient(Bs, layers, G, m)
            except coding.Undecodable:
                bad += 1
                continue
            ok += 1
            assert np.all(a[m == 1] == 0)
            assert np.allclose(g, full, rtol=1e-10, atol=1e-10)
        assert (ok, bad) == (5, 11)


def test_layer_zero_without_stragglers_is_plain_row_sum():
    G = np.random.default_rng(1).standard_normal((6, 11))
    Bs = codes.nested_code(6, [0, 2], seed=0, draws=2)
    u, a, g = coding.coded_gradient(Bs, [0, 2], G, np.zeros(6, np.uint8))
    assert u == 0 and np.array_equal(a, np.ones(6))
    assert np.allclose(g, G.sum(axis=0), rtol=1e-14)
    assert np.array_equal(coding.encode(Bs[0], G), G)


def test_decode_is_the_same_from_every_sufficient_layer():
    n, layers = 8, [0, 1, 3]
    G = np.random.default_rng(2).standard_normal((n, 13))
    Bs = codes.nested_code(n, layers, seed=4, draws=2)
    m = np.zeros(n, np.uint8)
    m[5] = 1
    outs = []
    for u in (1, 2):
        a, r = coding.decode_vector(Bs[u], m)
        outs.append(coding.decode(a, coding.encode(Bs[u], G)))
    assert np.allclose(outs[0], outs[1], rtol=1e-9, atol=1e-9)
    assert np.allclose(outs[0], G.sum(axis=0), rtol=1e-9, atol=1e-9)


def test_encode_row_is_the_sparse_combination_written_out():
    n, sigma = 7, 2
    B = codes.nested_code(n, [0, sigma], seed=9, draws=2)[1]
    G = np.random.default_rng(3).standard_normal((n, 4))
    C = coding.encode(B, G)
    for i in range(n):
        acc = np.zeros(4)
        for j in codes.cyclic_support(n, sigma, i):
            acc += B[i, j] * G[j]
        assert np.allclose(C[i], acc, rtol=1e-13, atol=1e-13)
    assert coding.encode_layers([np.eye(n), B], G).shape == (2, n, 4)


def test_coded_descent_follows_uncoded_descent_whatever_the_stragglers():
    """Exact recovery (Sec. I): the trajectory does not depend on who straggles,
    and converges to the least-squares solution."""
    n, layers = 4, [0, 1]
    X, Y, _ = _c1_like(rows=32)
    m_total = n * 32
    Bs = codes.nested_code(n, layers, "cyclic", seed=0, draws=2)
    rng = np.random.default_rng(11)
    th_c = np.zeros(5)
    th_u = np.zeros(5)
    for it in range(300):
        mask = np.zeros(n, np.uint8)
        if rng.random() < 0.7:
            mask[rng.integers(n)] = 1
        G = og.partial_gradients(0, X, Y, th_c)
        _, _, g = coding.coded_gradient(Bs, layers, G, mask)
        th_c = og.gd_update(th_c, g, 0.5, m_total)
        th_u = og.gd_update(th_u, og.lsq_gradient(X.reshape(-1, 5), Y.reshape(-1), th_u),
                            0.5, m_total)
    assert np.allclose(th_c, th_u, rtol=1e-9, atol=1e-10)
    th_ls = np.linalg.lstsq(X.reshape(-1, 5), Y.reshape(-1), rcond=None)[0]
    assert np.allclose(th_c, th_ls, rtol=1e-6, atol=1e-8)


def test_fp32_messages_stay_within_the_forward_error_bound():
    n, layers = 16, [0, 1, 3, 7]
    G = np.random.default_rng(5).standard_normal((n, 64))
    Bs = codes.nested_code(n, layers, seed=0, draws=4)
    rng = np.random.default_rng(6)
    for _ in range(30):
        m = (rng.random(n) < 0.2).astype(np.uint8)
        if m.sum() > 7:
            continue
        u, a, g32 = coding.coded_gradient(Bs, layers, G, m, np.float32)
        full = G.sum(axis=0)
        kap = coding.conditioning(a, coding.encode(Bs[u], G), full)
        err = np.linalg.norm(g32 - full) / np.linalg.norm(full)
        assert err <= 2.0 ** -24 * kap * 4


@pytest.mark.parametrize("n,c,layers,kind", [(4, 2, [0, 1], "fracrep"), (6, 3, [0, 1, 3], "cyclic"),
                                              (5, 2, [0, 2], "cyclic")])
def test_codes_for_k_equal_c_times_n_partitions(n, c, layers, kind):
    """Sec. II-C: with k = c n partitions an atomic task is k/n partial gradients;
    Def. 1 then asks for row weight >= (k/n)(sigma+1) and for the all-ones row of
    length k in the span of any n - sigma rows."""
    k = c * n
    Bs = codes.expand_partitions(codes.nested_code(n, layers, kind, seed=1, draws=2), c)
    G = np.random.default_rng(0).standard_normal((k, 7))
    full = G.sum(axis=0)
    for B, sigma in zip(Bs, layers):
        assert B.shape == (n, k)
        assert np.all((B != 0).sum(axis=1) == c * (sigma + 1))
        for out in itertools.combinations(range(n), sigma):
            S = [i for i in range(n) if i not in out]
            assert np.linalg.matrix_rank(np.vstack([B[S], np.ones(k)]), tol=1e-9) == \
                np.linalg.matrix_rank(B[S], tol=1e-9)
            m = np.zeros(n, np.uint8)
            m[list(out)] = 1
            a, resid = coding.decode_vector(B, m)
            assert resid < 1e-9 and np.all(a[m == 1] == 0)
            assert np.allclose(coding.decode(a, coding.encode(B, G)), full, rtol=1e-9, atol=1e-9)
    for i in range(n):
        for u in range(len(layers) - 1):
            assert set(np.flatnonzero(Bs[u][i])) <= set(np.flatnonzero(Bs[u + 1][i]))


def test_zero_padded_rows_do_not_change_the_gradient():
    """Sec. II-C footnote: if k does not divide m the data can be zero-padded."""
    rng = np.random.default_rng(2)
    X = rng.standard_normal((10, 4))
    y = rng.standard_normal(10)
    th = rng.standard_normal(4)
    Xp = np.vstack([X, np.zeros((2, 4))])
    yp = np.concatenate([y, np.zeros(2)])
    assert np.allclose(og.lsq_gradient(Xp, yp, th), og.lsq_gradient(X, y, th), rtol=1e-14)
    ypm = np.concatenate([np.sign(y), np.ones(2)])
    assert np.allclose(og.logistic_gradient(Xp, ypm, th), og.logistic_gradient(X, np.sign(y), th), rtol=1e-14)


# ---- guarded layer choice (an option on top of the Observation after Def. 2) ---------------
def _kappa_hat_by_hand(B, mask):
    """kappa_hat of the least-norm decode vector, written out with library routines only."""
    S = np.flatnonzero(mask == 0)
    aS = np.linalg.lstsq(B[S].T, np.ones(B.shape[1]), rcond=None)[0]
    return float(np.abs(aS) @ np.sqrt((B[S] ** 2).sum(axis=1)) / np.sqrt(B.shape[1])), S, aS


def test_guarded_choice_fracrep_closed_form():
    # n = 4, layers (0, 1), block code 1100/1100/0011/0011, worker 0 straggles: the layer-1
    # vector is (0, 1, 1/2, 1/2), every row has norm sqrt 2, k = 4:
    # kappa_hat = (1 + 1/2 + 1/2) sqrt 2 / 2 = sqrt 2
    Bs = codes.nested_code(4, [0, 1], "fracrep")
    m = np.array([1, 0, 0, 0], np.uint8)
    a, _ = coding.decode_vector(Bs[1], m)
    assert np.isclose(coding.amplification(Bs[1], a), np.sqrt(2.0), atol=1e-12)
    # no stragglers, layer 0 = identity: a = 1, rows of norm 1: kappa_hat = 4 / 2
    assert np.isclose(coding.amplification(Bs[0], np.ones(4)), 2.0, atol=1e-12)
    # a limit nobody meets: the layer of smallest kappa_hat among the sufficient ones;
    # without stragglers layer 1 gives a = 1/2 each, kappa_hat = 4 (1/2) sqrt 2 / 2 = sqrt 2 < 2
    u, a = coding.select_guarded(Bs, [0, 1], np.zeros(4, np.uint8), 0.1)
    assert u == 1 and np.allclose(a, 0.5)
    u, a = coding.select_guarded(Bs, [0, 1], np.zeros(4, np.uint8), 2.0)      # layer 0 meets the limit
    assert u == 0 and np.allclose(a, 1.0)
    with pytest.raises(coding.Undecodable):
        coding.select_guarded(Bs, [0, 1], np.array([1, 1, 0, 0], np.uint8), 1e9)


def test_guarded_choice_without_a_limit_is_the_plain_rule():
    layers = [0, 1, 3]
    Bs = codes.nested_code(8, layers, "cyclic", seed=2, draws=2)
    for m in _masks(8, 3):
        u, a = coding.select_guarded(Bs, layers, m, np.inf)
        assert u == coding.select_layer(layers, m)
        assert np.array_equal(a, coding.decode_vector(Bs[u], m)[0])


@pytest.mark.parametrize("limit", [0.5, 1.5, 3.0, 10.0])
def test_guarded_choice_rule_by_brute_force(limit):
    """Every mask of a small nested code: the result decodes (Def. 1), lies at or above the
    smallest sufficient layer, and is the first layer within the limit, else the best one."""
    layers = [0, 1, 2, 4]
    n = 7
    Bs = codes.nested_code(n, layers, "cyclic", seed=5, draws=2)
    moved = 0
    for m in _masks(n, 4):
        u, a = coding.select_guarded(Bs, layers, m, limit)
        u0 = min(v for v, s in enumerate(layers) if s >= int(m.sum()))
        assert u >= u0
        assert np.all(a[m == 1] == 0.0) and np.allclose(a @ Bs[u], 1.0, atol=1e-9)
        kh = [_kappa_hat_by_hand(Bs[v], m)[0] for v in range(u0, len(layers))]
        within = [v for v, x in zip(range(u0, len(layers)), kh) if x <= limit]
        want = within[0] if within else u0 + int(np.argmin(kh))
        assert u == want
        _, S, aS = _kappa_hat_by_hand(Bs[u], m)
        assert np.allclose(a[S], aS, atol=1e-9)
        moved += u != u0
    assert limit >= 10.0 or moved > 0          # tight limits do move rounds up


def test_guarded_choice_tames_the_tail_of_a_random_code():
    """n = 16, sigma = 7, exactly 7 stragglers: the worst sets of a random real-valued code
    amplify rounding by orders of magnitude more than the same sets one layer up."""
    layers = [0, 1, 3, 7, 11]
    Bs = codes.nested_code(16, layers, "cyclic", seed=0, draws=2)
    rng = np.random.default_rng(1)
    plain, guarded = [], []
    for _ in range(300):
        m = np.zeros(16, np.uint8)
        m[rng.choice(16, size=7, replace=False)] = 1
        a0, _ = coding.decode_vector(Bs[3], m)
        plain.append(coding.amplification(Bs[3], a0))
        u, a = coding.select_guarded(Bs, layers, m, 50.0)
        guarded.append(coding.amplification(Bs[u], a))
        assert np.allclose(a @ Bs[u], 1.0, atol=1e-8)
    assert max(plain) > 20 * max(guarded)
    assert max(guarded) <= 50.0


def test_full_replication_layer_gives_equal_weights():
    """sigma = n - 1: the rows of the component code span one dimension (Def. 1, second bullet:
    rank n - sigma = 1) and contain 1, so every row is the all-ones vector and the least-norm
    decode vector over r responders is 1/r on each of them, however the construction rounds."""
    for seed in (0, 149):
        B = codes.nested_code(6, [0, 5], "cyclic", seed=seed, draws=2)[1]
        assert np.allclose(B, 1.0, atol=1e-12)
        for m in _masks(6, 5):
            a, resid = coding.decode_vector(B, m)
            r = 6 - int(m.sum())
            assert resid < 1e-12
            assert np.allclose(a, np.where(m == 0, 1.0 / r, 0.0), atol=1e-12)
