"""Host-side behaviour of libngc that needs no GPU: the library loads and
exports the declared symbols, argument checks, code construction (checked
against Defs. 1-2 of the paper, not against the oracle's numbers), layer choice
and decode-vector selection (checked against the oracle)."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

from oracle import codes, coding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol(ngc):
    header = open(os.path.join(ROOT, "include", "ngc.h")).read()
    declared = set(re.findall(r"\b(ngc_[a-z0-9_]+)\s*\(", header))
    declared -= {"ngc_ctx"}
    assert declared == set(ngc.EXPORTS)
    lib = ctypes.CDLL(ngc.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_shape_query_returns_what_the_context_was_created_with(ngc):
    d = 8 * 6 + 6 + 6 * 3 + 3
    ctx = ngc.ngc_create(6, 12, [0, 2, 5], d)
    try:
        assert ngc.ngc_get_shape(ctx) == (6, 12, 3, d, 0)
        ngc.ngc_set_mlp2_shape(ctx, 8, 6, 3)
        assert ngc.ngc_get_shape(ctx) == (6, 12, 3, d, 8)
        with pytest.raises(ValueError):
            ngc.ngc_set_code(ctx, 1, np.eye(6))                  # B must be n x k
        with pytest.raises(ValueError):
            ngc.ngc_select_decode_vec(ctx, np.zeros(5, np.uint8), 5)   # mask of the wrong length
    finally:
        ngc.ngc_destroy(ctx)


def test_create_rejects_bad_arguments(ngc):
    bad = [
        dict(n=4, k=5, layers=[0, 1], d=8),          # k != n (Sec. II-C)
        dict(n=4, k=4, layers=[1, 2], d=8),          # first layer must be sigma = 0
        dict(n=4, k=4, layers=[0, 2, 2], d=8),       # not strictly ascending
        dict(n=4, k=4, layers=[0, 4], d=8),          # tolerance >= n
        dict(n=0, k=0, layers=[0], d=8),
        dict(n=65, k=65, layers=[0], d=8),
        dict(n=4, k=4, layers=[0, 1], d=0),
        dict(n=4, k=4, layers=[0, 1], d=2 ** 33 + 1),   # column-tile counts would not fit a grid
    ]
    for kw in bad:
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_create(kw["n"], kw["k"], kw["layers"], kw["d"])
        assert e.value.code == ngc.NGC_ERR_INVALID
    ngc.ngc_destroy(ngc.ngc_create(4, 4, [0, 1], 2 ** 33))    # the largest d (no memory is touched)
    ngc.ngc_destroy(None)


def test_layer_zero_is_identity_and_set_code_checks_nesting(ngc):
    ctx = ngc.ngc_create(4, 4, [0, 1, 3], 8)
    try:
        assert np.array_equal(ngc.ngc_get_code(ctx, 0, 4), np.eye(4))      # Alg. 1: B_0 = I
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_get_code(ctx, 1, 4)
        assert e.value.code == ngc.NGC_ERR_STATE
        B1 = codes.fracrep_code(4, 1)
        ngc.ngc_set_code(ctx, 1, B1)
        assert np.array_equal(ngc.ngc_get_code(ctx, 1, 4), B1)
        # layer 2 must contain layer 1's supports (Def. 2)
        bad = np.eye(4)
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_set_code(ctx, 2, bad)
        assert e.value.code == ngc.NGC_ERR_INVALID
        # a worker must hold its own partition
        bad = np.ones((4, 4))
        bad[2, 2] = 0.0
        with pytest.raises(ngc.NgcError):
            ngc.ngc_set_code(ctx, 2, bad)
        with pytest.raises(ngc.NgcError):
            ngc.ngc_set_code(ctx, 3, np.ones((4, 4)))
        nan = np.ones((4, 4))
        nan[0, 1] = np.nan
        with pytest.raises(ngc.NgcError):
            ngc.ngc_set_code(ctx, 2, nan)
        ngc.ngc_set_code(ctx, 2, np.ones((4, 4)))
    finally:
        ngc.ngc_destroy(ctx)


@pytest.mark.parametrize("n,layers", [(6, [0, 1, 2, 3]), (8, [0, 1, 3, 7]), (9, [0, 2, 4])])
def test_built_cyclic_code_satisfies_def1_and_def2(ngc, n, layers):
    ctx = ngc.ngc_create(n, n, layers, 4)
    try:
        ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC, 7)
        prev = None
        for u, sigma in enumerate(layers):
            B = ngc.ngc_get_code(ctx, u, n)
            if sigma == 0:
                assert np.array_equal(B, np.eye(n))
            supp = [set(np.flatnonzero(B[i])) for i in range(n)]
            for i in range(n):
                assert supp[i] == {(i + t) % n for t in range(sigma + 1)}
                if prev is not None:
                    assert prev[i] <= supp[i]
            prev = supp
            for out in itertools.combinations(range(n), sigma):
                S = [i for i in range(n) if i not in out]
                assert np.linalg.matrix_rank(B[S], tol=1e-9) == n - sigma
                assert np.linalg.matrix_rank(np.vstack([B[S], np.ones(n)]), tol=1e-9) == n - sigma
    finally:
        ngc.ngc_destroy(ctx)


def test_build_code_is_deterministic_in_the_seed(ngc):
    def built(seed):
        ctx = ngc.ngc_create(12, 12, [0, 1, 3], 4)
        ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC, seed)
        B = [ngc.ngc_get_code(ctx, u, 12) for u in range(3)]
        ngc.ngc_destroy(ctx)
        return B
    a, b, c = built(5), built(5), built(6)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert not np.array_equal(a[2], c[2])


def test_built_fracrep_code(ngc):
    ctx = ngc.ngc_create(8, 8, [0, 1, 3, 7], 4)
    try:
        ngc.ngc_build_code(ctx, ngc.NGC_CODE_FRACREP, 0)
        for u, sigma in enumerate([0, 1, 3, 7]):
            assert np.array_equal(ngc.ngc_get_code(ctx, u, 8), codes.fracrep_code(8, sigma))
    finally:
        ngc.ngc_destroy(ctx)
    ctx = ngc.ngc_create(20, 20, [0, 1, 4], 4)
    try:
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_build_code(ctx, ngc.NGC_CODE_FRACREP, 0)       # 2 does not divide 5
        assert e.value.code == ngc.NGC_ERR_INVALID
        with pytest.raises(ngc.NgcError):
            ngc.ngc_build_code(ctx, 9, 0)
    finally:
        ngc.ngc_destroy(ctx)


def test_select_matches_golden_fracrep_case_for_all_16_masks(ngc):
    ctx = ngc.ngc_create(4, 4, [0, 1], 4)
    try:
        ngc.ngc_build_code(ctx, ngc.NGC_CODE_FRACREP, 0)
        gold = {}
        with open(os.path.join(ROOT, "tests", "golden", "fracrep_n4.txt")) as f:
            for line in f:
                if line.startswith("#") or not line.strip():
                    continue
                tok = line.split()
                gold[tok[0]] = (int(tok[1]), [float(t) for t in tok[2:6]])
        ok = bad = 0
        for bits in range(16):
            m = np.array([(bits >> i) & 1 for i in range(4)], np.uint8)
            key = "".join(str(int(b)) for b in m)
            if key in gold:
                u, a, r = ngc.ngc_select_decode_vec(ctx, m, 4)
                assert u == gold[key][0]
                assert np.allclose(a, gold[key][1], atol=1e-12)
                assert r < 1e-12
                ok += 1
            else:
                with pytest.raises(ngc.NgcError) as e:
                    ngc.ngc_select_decode_vec(ctx, m, 4)
                assert e.value.code == ngc.NGC_ERR_UNDECODABLE
                bad += 1
        assert (ok, bad) == (5, 11)
    finally:
        ngc.ngc_destroy(ctx)


@pytest.mark.parametrize("n,layers,kind", [(16, [0, 1, 3, 7], "cyclic"), (32, [0, 1, 3, 7, 15], "cyclic"),
                                           (64, [0, 1, 3, 7, 15, 31], "cyclic"),
                                           (64, [0, 1, 3, 7, 15, 31], "fracrep"), (20, [0, 1, 4, 9], "cyclic")])
def test_select_agrees_with_oracle_on_random_masks(ngc, n, layers, kind):
    Bs = codes.nested_code(n, layers, kind, seed=0, draws=2)
    ctx = ngc.ngc_create(n, n, layers, 4)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        rng = np.random.default_rng(n)
        for t in range(60):
            s = int(rng.integers(0, layers[-1] + 3))
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=min(s, n), replace=False)] = 1
            try:
                u_o = coding.select_layer(layers, m)
            except coding.Undecodable:
                with pytest.raises(ngc.NgcError) as e:
                    ngc.ngc_select_decode_vec(ctx, m, n)
                assert e.value.code == ngc.NGC_ERR_UNDECODABLE
                continue
            u, a, r = ngc.ngc_select_decode_vec(ctx, m, n)
            a_o, r_o = coding.decode_vector(Bs[u_o], m)
            assert u == u_o
            assert np.array_equal(a != 0, a_o != 0)                    # support: exact
            assert np.all(a[m == 1] == 0)
            assert r < 1e-8
            scale = max(1.0, np.abs(a_o).max())
            assert np.abs(a - a_o).max() <= 1e-7 * scale
            # first-responders rule
            u1, a1, r1 = ngc.ngc_select_decode_vec_first(ctx, m, n)
            if kind == "cyclic":
                a1_o, _ = coding.decode_vector_first(Bs[u_o], layers[u_o], m)
                assert u1 == u_o and r1 < 1e-8
                assert np.abs(a1 - a1_o).max() <= 1e-7 * max(1.0, np.abs(a1_o).max())
                assert np.count_nonzero(a1) <= n - layers[u_o]
    finally:
        ngc.ngc_destroy(ctx)


@pytest.mark.parametrize("n,layers,kind,limits", [
    (16, [0, 1, 3, 7], "cyclic", (2.0, 10.0, 100.0)), (32, [0, 1, 3, 7, 15], "cyclic", (20.0, 300.0)),
    (64, [0, 1, 3, 7, 15, 31], "cyclic", (100.0, 1000.0)), (8, [0, 1, 3, 7], "fracrep", (0.5, 1.5, 4.0)),
    (12, [0, 1, 2, 3, 4, 5], "cyclic", (1.0, 5.0, 30.0))])
def test_guarded_choice_agrees_with_oracle(ngc, n, layers, kind, limits):
    """ngc_set_decode_guard: the layer and the vector of the guarded rule are the oracle's for
    masks that stress it (as many stragglers as a layer tolerates) and for random ones; with
    the guard off the plain rule is back; the first-responders variant is never guarded."""
    Bs = codes.nested_code(n, layers, kind, seed=0, draws=2)
    ctx = ngc.ngc_create(n, n, layers, 4)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        rng = np.random.default_rng(3 * n)
        masks = []
        for t in range(80):
            s = layers[1 + t % (len(layers) - 1)] if t % 2 else int(rng.integers(0, layers[-1] + 1))
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=s, replace=False)] = 1
            masks.append(m)
        moved = 0
        for limit in limits:
            ngc.ngc_set_decode_guard(ctx, limit)
            for m in masks:
                u_o, a_o = coding.select_guarded(Bs, layers, m, limit)
                u, a, r = ngc.ngc_select_decode_vec(ctx, m, n)
                assert u == u_o
                assert np.array_equal(a != 0, a_o != 0) and np.all(a[m == 1] == 0) and r < 1e-8
                assert np.abs(a - a_o).max() <= 1e-7 * max(1.0, np.abs(a_o).max())
                moved += u != coding.select_layer(layers, m)
                u1, _, _ = ngc.ngc_select_decode_vec_first(ctx, m, n)
                assert u1 == coding.select_layer(layers, m)
        assert moved > 0
        for off in (0.0, float("inf")):
            ngc.ngc_set_decode_guard(ctx, off)
            for m in masks[:20]:
                assert ngc.ngc_select_decode_vec(ctx, m, n)[0] == coding.select_layer(layers, m)
        for bad in (-1.0, float("nan")):
            with pytest.raises(ngc.NgcError) as e:
                ngc.ngc_set_decode_guard(ctx, bad)
            assert e.value.code == ngc.NGC_ERR_INVALID
    finally:
        ngc.ngc_destroy(ctx)


def test_guarded_choice_with_several_partitions_per_worker(ngc):
    """k = c n: the estimate is taken over the k columns of the expanded code on both sides."""
    n, c, layers = 8, 2, [0, 1, 3, 5]
    Bs = codes.expand_partitions(codes.nested_code(n, layers, "cyclic", seed=4, draws=2), c)
    ctx = ngc.ngc_create(n, n * c, layers, 4)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        rng = np.random.default_rng(11)
        moved = 0
        for limit in (1.5, 4.0, 20.0):
            ngc.ngc_set_decode_guard(ctx, limit)
            for _ in range(60):
                m = np.zeros(n, np.uint8)
                m[rng.choice(n, size=int(rng.integers(0, layers[-1] + 1)), replace=False)] = 1
                u_o, a_o = coding.select_guarded(Bs, layers, m, limit)
                u, a, r = ngc.ngc_select_decode_vec(ctx, m, n)
                assert u == u_o and r < 1e-8
                assert np.abs(a - a_o).max() <= 1e-7 * max(1.0, np.abs(a_o).max())
                moved += u != coding.select_layer(layers, m)
        assert moved > 0
    finally:
        ngc.ngc_destroy(ctx)


def test_select_on_the_full_replication_layer(ngc):
    """sigma = n - 1 (every row the all-ones vector up to the rounding of its construction): the
    least-norm vector over r responders is 1/r each, from the oracle's code and the library's own."""
    n, layers = 6, [0, 5]
    for built in (False, True):
        ctx = ngc.ngc_create(n, n, layers, 4)
        try:
            if built:
                ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC, 3)
            else:
                ngc.ngc_set_code(ctx, 1, codes.nested_code(n, layers, "cyclic", seed=149, draws=2)[1])
            for bits in range(1, 2 ** n - 1):
                m = np.array([(bits >> i) & 1 for i in range(n)], np.uint8)
                u, a, resid = ngc.ngc_select_decode_vec(ctx, m, n)
                r = n - int(m.sum())
                assert u == 1 and resid < 1e-9
                assert np.allclose(a, np.where(m == 0, 1.0 / r, 0.0), atol=1e-9)
        finally:
            ngc.ngc_destroy(ctx)


def test_select_reports_singular_for_a_matrix_that_is_no_gradient_code(ngc):
    n = 6
    ctx = ngc.ngc_create(n, n, [0, 2], 4)
    try:
        B = np.eye(n)
        for i in range(n):
            B[i, (i + 1) % n] = 2.0
            B[i, (i + 2) % n] = -1.0 - i      # rows do not span the all-ones row once two are missing
        ngc.ngc_set_code(ctx, 1, B)
        m = np.zeros(n, np.uint8)
        m[[0, 3]] = 1
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_select_decode_vec(ctx, m, n)
        assert e.value.code == ngc.NGC_ERR_SINGULAR
    finally:
        ngc.ngc_destroy(ctx)


def test_select_on_a_degenerate_code_with_dependent_straggler_rows(ngc):
    """B = 1 1^T + u v^T with u = e_2 + e_3: workers 2 and 3 hold the same row, so whatever is
    orthogonal to B's columns has dependent entries on them.  Losing both of them is decodable
    (a = (1/2, 1/2, 0, 0) by symmetry); losing workers 0 and 1 is not."""
    n = 4
    ctx = ngc.ngc_create(n, n, [0, 2], 4)
    try:
        B = np.ones((n, n))
        B[2:, 3] += 1.0
        ngc.ngc_set_code(ctx, 1, B)
        m = np.array([0, 0, 1, 1], np.uint8)
        u, a, r = ngc.ngc_select_decode_vec(ctx, m, n)
        assert u == 1 and r < 1e-12
        assert np.allclose(a, [0.5, 0.5, 0.0, 0.0], atol=1e-14)
        a_o, _ = coding.decode_vector(B, m)
        assert np.allclose(a, a_o, atol=1e-12)
        m = np.array([0, 0, 0, 1], np.uint8)                  # one of the twins still responds
        u, a, r = ngc.ngc_select_decode_vec(ctx, m, n)
        a_o, _ = coding.decode_vector(B, m)
        assert r < 1e-12 and a[3] == 0.0 and np.allclose(a, a_o, atol=1e-12)
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_select_decode_vec(ctx, np.array([1, 1, 0, 0], np.uint8), n)
        assert e.value.code == ngc.NGC_ERR_SINGULAR
    finally:
        ngc.ngc_destroy(ctx)


def test_null_arguments_are_rejected_not_dereferenced(ngc):
    ctx = ngc.ngc_create(4, 4, [0, 1], 8)
    try:
        lib = ngc._lib
        assert lib.ngc_set_code(ctx, 1, None) == ngc.NGC_ERR_INVALID
        assert lib.ngc_select_decode_vec(ctx, None, None, None, None) == ngc.NGC_ERR_INVALID
        assert lib.ngc_partition_grads(ctx, 0, None, None, None, 4, None) == ngc.NGC_ERR_INVALID
        assert lib.ngc_encode(ctx, None, -1, None) == ngc.NGC_ERR_INVALID
        assert lib.ngc_decode(ctx, 0, None, None, None) == ngc.NGC_ERR_INVALID
        assert lib.ngc_update(ctx, None, None, 0.1) == ngc.NGC_ERR_INVALID
        assert "null" in ngc.ngc_last_error(ctx)
        assert ngc.ngc_strerror(-2).startswith("more stragglers")
    finally:
        ngc.ngc_destroy(ctx)


def test_empty_and_misaligned_inputs_are_rejected_before_any_device_work(ngc):
    """No rows, a buffer that is not 16-byte aligned, an unknown loss: the call returns
    INVALID from its argument checks (the addresses below are never dereferenced and no GPU is
    needed to get that far)."""
    import ctypes
    n = 4
    ctx = ngc.ngc_create(n, n, [0, 1], 8)
    try:
        lib = ngc._lib
        ok = ctypes.c_void_p(0x10000)             # stands for an aligned device address
        odd = ctypes.c_void_p(0x10004)
        prog = (ctypes.c_int * n)(*([2] * n))
        mask = (ctypes.c_uint8 * n)()
        a = (ctypes.c_double * n)()
        u = ctypes.c_int(0)
        rows = ctypes.c_int64
        for r in (0, -3):
            assert lib.ngc_partition_grads(ctx, 0, ok, ok, ok, rows(r), ok) == ngc.NGC_ERR_INVALID
            assert "rows" in ngc.ngc_last_error(ctx)
            assert lib.ngc_worker_grads(ctx, 0, ok, ok, ok, rows(r), prog, ok) == ngc.NGC_ERR_INVALID
            assert lib.ngc_iteration(ctx, 0, ok, ok, ok, rows(r), mask, ctypes.c_double(0.1), ok, ok, ok,
                                     ctypes.byref(u), a) == ngc.NGC_ERR_INVALID
        assert lib.ngc_partition_grads(ctx, 0, odd, ok, ok, rows(4), ok) == ngc.NGC_ERR_INVALID
        assert "aligned" in ngc.ngc_last_error(ctx)
        assert lib.ngc_partition_grads(ctx, 0, ok, ok, odd, rows(4), ok) == ngc.NGC_ERR_INVALID
        assert lib.ngc_partition_grads(ctx, 0, ok, ok, ok, rows(4), odd) == ngc.NGC_ERR_INVALID
        assert lib.ngc_worker_grads(ctx, 0, ok, ok, ok, rows(4), prog, odd) == ngc.NGC_ERR_INVALID
        assert lib.ngc_worker_grads(ctx, 9, ok, ok, ok, rows(4), prog, ok) == ngc.NGC_ERR_INVALID
        assert "loss" in ngc.ngc_last_error(ctx)
        assert lib.ngc_iteration(ctx, 9, ok, ok, ok, rows(4), mask, ctypes.c_double(0.1), ok, ok, ok,
                                 ctypes.byref(u), a) == ngc.NGC_ERR_INVALID
        assert lib.ngc_iteration(ctx, 0, ok, ok, ok, rows(4), mask, ctypes.c_double(0.1), ok, odd, ok,
                                 ctypes.byref(u), a) == ngc.NGC_ERR_INVALID
        # the perceptron loss before its shape is known
        assert lib.ngc_worker_grads(ctx, 2, ok, ok, ok, rows(4), prog, ok) == ngc.NGC_ERR_STATE
        # an undecodable round launches nothing: three stragglers against a tolerance of one
        for i in range(3):
            mask[i] = 1
        assert lib.ngc_iteration(ctx, 0, ok, ok, ok, rows(4), mask, ctypes.c_double(0.1), ok, ok, ok,
                                 ctypes.byref(u), a) == ngc.NGC_ERR_UNDECODABLE
    finally:
        ngc.ngc_destroy(ctx)


# ---- redundancy-faithful execution: schedule and termination rule (host only) -----------------
@pytest.mark.parametrize("n,layers,kind", [(8, [0, 1, 3], "cyclic"), (8, [0, 1, 3, 7], "fracrep"),
                                           (6, [0, 2, 3], "cyclic")])
def test_worker_schedule_matches_oracle(ngc, n, layers, kind):
    from oracle import workers as ow
    Bs = codes.nested_code(n, layers, kind, seed=0, draws=2)
    ctx = ngc.ngc_create(n, n, layers, 4)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        assert ngc.ngc_worker_task_count(ctx) == layers[-1] + 1
        for i in range(n):
            assert ngc.ngc_worker_schedule(ctx, i) == ow.task_order(Bs, i)
    finally:
        ngc.ngc_destroy(ctx)


def test_select_from_progress_matches_oracle_rule(ngc):
    from oracle import workers as ow
    n, layers = 6, [0, 1, 3]
    Bs = codes.nested_code(n, layers, "cyclic", seed=1, draws=2)
    ctx = ngc.ngc_create(n, n, layers, 4)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        rng = np.random.default_rng(0)
        seen = set()
        cases = [rng.integers(0, 5, n) for _ in range(300)] + [np.full(n, t) for t in range(5)]
        for progress in cases:
            for min_layer in (0, 2):
                try:
                    u_o, mask_o = ow.terminate(Bs, layers, progress, min_layer)
                except coding.Undecodable:
                    with pytest.raises(ngc.NgcError) as e:
                        ngc.ngc_select_from_progress(ctx, progress, n, min_layer)
                    assert e.value.code == ngc.NGC_ERR_UNDECODABLE
                    seen.add(-1)
                    continue
                u, mask, a, r = ngc.ngc_select_from_progress(ctx, progress, n, min_layer)
                assert u == u_o and np.array_equal(mask, mask_o)
                a_o = codes.min_norm_decode_vector(Bs[u_o], np.flatnonzero(mask_o == 0))
                assert np.array_equal(a != 0, a_o != 0)
                assert np.abs(a - a_o).max() <= 1e-8 * max(1.0, np.abs(a_o).max())
                assert r < 1e-8
                seen.add(u)
        assert seen == {-1, 0, 1, 2}
        with pytest.raises(ngc.NgcError):
            ngc.ngc_select_from_progress(ctx, [1] * n, n, 7)
        with pytest.raises(ngc.NgcError):
            ngc.ngc_select_from_progress(ctx, [-1] * n, n, 0)
    finally:
        ngc.ngc_destroy(ctx)


# ---- latency model: closed forms on the host against the oracle ---------------------------------
def test_latency_closed_forms_match_oracle(ngc):
    from oracle import latency as ol
    t = np.linspace(0.0, 20.0, 41)
    for (n, lam, rho, eps, gamma, pe) in [(8, 0.5, 0.5, 0.1, 0.0, 0.05), (6, 1.3, 0.0, 0.0, 0.2, 0.2),
                                          (12, 0.8, 0.25, 0.05, 0.1, 0.0)]:
        for s in (0, 1, 3, 5):
            gc = ngc.ngc_latency_cdf_gc(n, s, lam, rho, eps, gamma, pe, t)
            nested = ngc.ngc_latency_cdf_ngc(n, s, lam, rho, eps, gamma, pe, t)
            for q, tq in enumerate(t):
                assert abs(gc[q] - ol.gc_cdf(tq, n, s, lam, rho, eps, gamma, pe)) < 1e-12
                if n <= 8:      # the oracle's nested sum is exponential in s
                    assert abs(nested[q] - ol.ngc_cdf(tq, n, s, lam, rho, eps, gamma, pe)) < 1e-12
            assert np.all(np.diff(nested) >= -1e-13) and np.all(nested >= gc - 1e-13)
    # the one number the paper prints: n = 8, p_e = 0.05, sigma = 0 tends to ~0.66
    assert abs(ngc.ngc_latency_cdf_gc(8, 0, 0.5, 0.5, 0.1, 0.0, 0.05, [1e4])[0] - 0.95 ** 8) < 1e-12
    # a size the nested sum could not enumerate
    big = ngc.ngc_latency_cdf_ngc(64, 31, 0.5, 0.5, 0.1, 0.0, 0.05, [5.0, 50.0, 1e4])
    assert 0.0 <= big[0] <= big[1] <= big[2] <= 1.0 and big[2] > 0.999999
    with pytest.raises(ngc.NgcError):
        ngc.ngc_latency_cdf_gc(8, 8, 0.5, 0.5, 0.1, 0.0, 0.05, [1.0])
    with pytest.raises(ngc.NgcError):
        ngc.ngc_latency_cdf_ngc(8, 3, -1.0, 0.5, 0.1, 0.0, 0.05, [1.0])


# ---- explicit decoding matrix A_sigma (Def. 1) --------------------------------------------------
@pytest.mark.parametrize("n,layers,kind", [(8, [0, 1, 3], "cyclic"), (7, [0, 2, 5], "cyclic"),
                                           (8, [0, 1, 3, 7], "fracrep")])
def test_decoding_table_satisfies_def1_and_matches_oracle(ngc, n, layers, kind):
    Bs = codes.nested_code(n, layers, kind, seed=0, draws=2)
    ctx = ngc.ngc_create(n, n, layers, 4)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        for u, sigma in enumerate(layers):
            with pytest.raises(ngc.NgcError) as e:
                ngc.ngc_get_decoding_row(ctx, u, 0, n)
            assert e.value.code == ngc.NGC_ERR_STATE
            rows = ngc.ngc_build_decoding_table(ctx, u)
            assert rows == len(list(itertools.combinations(range(n), sigma)))
            A_o = codes.decoding_matrix(Bs[u], sigma)                 # same (lexicographic) row order
            for r, out in enumerate(itertools.combinations(range(n), sigma)):
                m = np.zeros(n, np.uint8)
                m[list(out)] = 1
                assert ngc.ngc_decoding_row_index(ctx, u, m) == r
                a = ngc.ngc_get_decoding_row(ctx, u, r, n)
                assert np.all(a[list(out)] == 0.0)                    # supported on the responders
                assert np.allclose(a @ Bs[u], 1.0, atol=1e-9)         # A B = 1
                assert np.abs(a - A_o[r]).max() <= 1e-8 * max(1.0, np.abs(A_o[r]).max())
            # fewer stragglers than sigma: the lowest n - sigma responders decode
            if sigma >= 2:
                m = np.zeros(n, np.uint8)
                m[1] = 1
                r = ngc.ngc_decoding_row_index(ctx, u, m)
                a = ngc.ngc_get_decoding_row(ctx, u, r, n)
                a_first, _ = coding.decode_vector_first(Bs[u], sigma, m)
                assert a[1] == 0.0 and np.allclose(a, a_first, atol=1e-8)
            if sigma + 1 < n:
                m = np.zeros(n, np.uint8)
                m[: sigma + 1] = 1
                with pytest.raises(ngc.NgcError) as e:
                    ngc.ngc_decoding_row_index(ctx, u, m)
                assert e.value.code == ngc.NGC_ERR_UNDECODABLE
        # a new matrix for the layer discards its table
        ngc.ngc_set_code(ctx, 1, Bs[1])
        with pytest.raises(ngc.NgcError):
            ngc.ngc_get_decoding_row(ctx, 1, 0, n)
    finally:
        ngc.ngc_destroy(ctx)


def test_decoding_table_size_limit(ngc):
    ctx = ngc.ngc_create(32, 32, [0, 15], 4)
    try:
        ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC, 0)
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_build_decoding_table(ctx, 1)                      # C(32,15) rows
        assert e.value.code == ngc.NGC_ERR_INVALID
    finally:
        ngc.ngc_destroy(ctx)


# ---- k = c*n partitions (an atomic task is k/n partial gradients, Sec. II-C) --------------------
def test_context_with_several_partitions_per_worker(ngc):
    from oracle import workers as ow
    n, c, layers = 6, 2, [0, 1, 3]
    k = n * c
    ctx = ngc.ngc_create(n, k, layers, 4)
    try:
        assert np.array_equal(ngc.ngc_get_code(ctx, 0, n, k), np.kron(np.eye(n), np.ones((1, c))))
        ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC, 3)
        Bs = [ngc.ngc_get_code(ctx, u, n, k) for u in range(3)]
        for B, sigma in zip(Bs, layers):
            assert np.all((B != 0).sum(axis=1) == c * (sigma + 1))            # Def. 1: weight (k/n)(sigma+1)
            assert np.array_equal(B[:, 0::2], B[:, 1::2])
            for out in itertools.combinations(range(n), sigma):
                m = np.zeros(n, np.uint8)
                m[list(out)] = 1
                u, a, r = ngc.ngc_select_decode_vec(ctx, m, n)
                assert r < 1e-8
        # the oracle's widened code through set_code, decode vectors against the oracle
        Bo = codes.expand_partitions(codes.nested_code(n, layers, "cyclic", seed=0, draws=2), c)
        for u, B in enumerate(Bo):
            ngc.ngc_set_code(ctx, u, B)
        rng = np.random.default_rng(0)
        for _ in range(40):
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=int(rng.integers(0, 4)), replace=False)] = 1
            u, a, r = ngc.ngc_select_decode_vec(ctx, m, n)
            u_o = coding.select_layer(layers, m)
            a_o, _ = coding.decode_vector(Bo[u_o], m)
            assert u == u_o and np.abs(a - a_o).max() <= 1e-8 * max(1.0, np.abs(a_o).max())
        assert ngc.ngc_worker_task_count(ctx) == 4
        for i in range(n):
            assert ngc.ngc_worker_schedule(ctx, i) == ow.task_order(Bo, i)
        bad = Bo[1].copy()
        bad[2, 2 * c + 1] = 0.0                                            # worker 2 must hold all of group 2
        with pytest.raises(ngc.NgcError):
            ngc.ngc_set_code(ctx, 1, bad)
    finally:
        ngc.ngc_destroy(ctx)
    for n, k in ((4, 6), (8, 4), (40, 80)):
        with pytest.raises(ngc.NgcError):
            ngc.ngc_create(n, k, [0, 1], 4)


def test_lds_need_of_the_iteration_tail(ngc):
    """Size formula of ngc_iteration's second launch, retyped here from the layout the header
    states: sixteen fp64 partial-sum rows of 16 V + 1, a G tile of k x 16 V floats, the decode
    layer's messages n x 16 V floats, and (if kept in LDS) the compressed code tables
    L n + 1 row pointers + a column index and a coefficient per non-zero."""
    def want(n, k, L, nnz, V, tables):
        b = 16 * (16 * V + 1) * 8 + (k + n) * 16 * V * 4
        return b + (L * n + 1 + 2 * nnz) * 4 if tables else b

    cases = [(4, 4, (0, 1)), (32, 32, (0, 1, 3, 7, 15)), (64, 64, (0, 1, 3, 7, 15, 31)),
             (8, 16, (0, 1, 3)), (64, 64, tuple(range(32)))]
    for n, k, layers in cases:
        ctx = ngc.ngc_create(n, k, layers, 1024)
        try:
            with pytest.raises(ngc.NgcError) as e:
                ngc.ngc_tail_lds_bytes(ctx, 4)                     # a layer without its code
            assert e.value.code == ngc.NGC_ERR_STATE
            ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC, 1)
            nnz = sum(int(np.count_nonzero(ngc.ngc_get_code(ctx, u))) for u in range(len(layers)))
            assert nnz == sum((s + 1) * k for s in layers)          # row weight (k/n)(sigma+1), Def. 1
            for V in (1, 2, 4):
                w, wo = ngc.ngc_tail_lds_bytes(ctx, V)
                assert w == want(n, k, len(layers), nnz, V, True)
                assert wo == want(n, k, len(layers), nnz, V, False)
            with pytest.raises(ngc.NgcError):
                ngc.ngc_tail_lds_bytes(ctx, 3)
        finally:
            ngc.ngc_destroy(ctx)
    # the full layer set of 64 workers: the tables alone exceed the 160 KiB of LDS a CU has,
    # the tiles without them fit easily
    ctx = ngc.ngc_create(64, 64, tuple(range(32)), 1024)
    try:
        ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC, 1)
        w, wo = ngc.ngc_tail_lds_bytes(ctx, 4)
        assert w > 160 * 1024 > 64 * 1024 > wo
    finally:
        ngc.ngc_destroy(ctx)
