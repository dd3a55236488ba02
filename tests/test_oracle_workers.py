"""Pins for oracle/workers.py: the layered schedule, the termination rule and
the fact that messages built from a worker's own partial gradients are the rows
of B G, so that decoding returns the full gradient (Secs. II-C, III, IV)."""
import itertools

import numpy as np
import pytest

from oracle import codes, coding, gradients as og, workers as ow


def _data(n, rows=6, d=5, seed=0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, rows, d))
    Y = rng.standard_normal((n, rows))
    return X, Y, rng.standard_normal(d)


def test_cyclic_schedule_is_own_partition_then_cyclic_successors():
    Bs = codes.nested_code(8, [0, 1, 3], seed=0, draws=2)
    for i in range(8):
        assert ow.task_order(Bs, i) == [(i + t) % 8 for t in range(4)]
        assert [ow.tasks_needed(Bs, i, u) for u in range(3)] == [1, 2, 4]     # load s+1 (Sec. II-C)


def test_fracrep_schedule_starts_with_own_partition_and_stays_in_block():
    Bs = codes.nested_code(8, [0, 1, 3], "fracrep")
    assert ow.task_order(Bs, 5) == [5, 4, 6, 7]
    assert ow.task_order(Bs, 2) == [2, 3, 0, 1]
    for i in range(8):
        order = ow.task_order(Bs, i)
        assert order[0] == i and sorted(order) == codes.fracrep_support(8, 3, i)


def test_termination_rule_table():
    n, layers = 6, [0, 1, 3]
    Bs = codes.nested_code(n, layers, seed=1, draws=2)
    # everybody finished one task: layer 0 decodes
    assert ow.terminate(Bs, layers, [1] * n)[0] == 0
    # one worker has nothing: layer 0 fails; layer 1 needs 5 workers with 2 tasks
    with pytest.raises(coding.Undecodable):
        ow.terminate(Bs, layers, [0, 1, 1, 1, 1, 1])
    u, mask = ow.terminate(Bs, layers, [0, 2, 2, 2, 2, 2])
    assert u == 1 and list(mask) == [1, 0, 0, 0, 0, 0]
    # four of six with two tasks is not enough for sigma = 1, three with four tasks is for sigma = 3
    with pytest.raises(coding.Undecodable):
        ow.terminate(Bs, layers, [0, 0, 2, 2, 2, 2])
    u, mask = ow.terminate(Bs, layers, [0, 0, 2, 4, 4, 4])
    assert u == 2 and list(mask) == [1, 1, 1, 0, 0, 0]
    # a worker ahead of the others is simply used at the lower layer
    assert ow.terminate(Bs, layers, [4, 1, 1, 1, 1, 1])[0] == 0
    # conventional code with fixed sigma = 3: lower layers are not an option
    with pytest.raises(coding.Undecodable):
        ow.terminate(Bs, layers, [2] * n, min_layer=2)
    assert ow.terminate(Bs, layers, [4, 4, 4, 1, 0, 0], min_layer=2)[0] == 2


def test_worker_messages_are_rows_of_BG_and_decode_to_the_full_gradient():
    n, layers = 4, [0, 1]
    X, Y, th = _data(n)
    G = og.partial_gradients(0, X, Y, th)
    full = G.sum(axis=0)
    for kind in ("cyclic", "fracrep"):
        Bs = codes.nested_code(n, layers, kind, seed=2, draws=2)
        decodable = 0
        for progress in itertools.product(range(3), repeat=n):          # all 81 progress vectors
            W = ow.worker_partials(0, X, Y, th, Bs, progress)
            C = ow.worker_messages(Bs, W, progress)
            for u in range(2):
                CB = coding.encode(Bs[u], G)
                for i in range(n):
                    if progress[i] >= ow.tasks_needed(Bs, i, u):
                        assert np.allclose(C[u][i], CB[i], rtol=1e-12, atol=1e-12)
                    else:
                        assert C[u][i] is None
            try:
                u, mask, a, g = ow.decode_from_workers(Bs, layers, W, progress)
            except coding.Undecodable:
                # then really no layer has enough finished workers
                assert sum(p >= 1 for p in progress) < n and sum(p >= 2 for p in progress) < n - 1
                continue
            decodable += 1
            assert np.allclose(g, full, rtol=1e-10, atol=1e-10)
            assert np.all(a[mask == 1] == 0)
            # no smaller layer would have done
            for v in range(u):
                assert sum(progress[i] >= ow.tasks_needed(Bs, i, v) for i in range(n)) < n - layers[v]
        assert decodable == 20          # 16 with everybody past task 1, 4 with one idle worker and three at 2


def test_load_of_nested_code_versus_fixed_sigma_code():
    """With s stragglers a nested code stops after s_u + 1 tasks per worker, a
    conventional code with sigma = s_max after s_max + 1: overhead factor
    (sigma+1)/(s+1) per non-straggler (Sec. III)."""
    n, layers = 8, [0, 1, 3, 7]
    Bs = codes.nested_code(n, layers, seed=3, draws=2)
    smax = layers[-1]
    for s in (0, 1, 3):
        dead = list(range(s))
        # workers advance one task per time step until the main node can decode
        def run(min_layer):
            progress = np.zeros(n, int)
            for step in range(smax + 1):
                progress[[i for i in range(n) if i not in dead]] += 1
                try:
                    u, _ = ow.terminate(Bs, layers, progress, min_layer)
                    return u, ow.tasks_executed(progress)
                except coding.Undecodable:
                    pass
            raise AssertionError("never decodable")
        u_ngc, work_ngc = run(0)
        u_gc, work_gc = run(len(layers) - 1)
        assert layers[u_ngc] == s and u_gc == len(layers) - 1
        assert work_ngc == (n - s) * (s + 1)
        assert work_gc == (n - s) * (smax + 1)
        assert work_gc / work_ngc == (smax + 1) / (s + 1)


def test_schedule_with_several_partitions_per_task():
    """k = 2n: a task is the two partitions of a group; worker i starts with group i."""
    Bs = codes.expand_partitions(codes.nested_code(4, [0, 1], seed=0, draws=2), 2)
    assert ow.task_order(Bs, 1) == [2, 3, 4, 5]
    assert ow.task_order(Bs, 3) == [6, 7, 0, 1]
    assert [ow.tasks_needed(Bs, 0, u) for u in range(2)] == [1, 2]
    X, Y, th = _data(8)
    G = og.partial_gradients(0, X, Y, th)
    progress = [2, 2, 0, 2]
    W = ow.worker_partials(0, X, Y, th, Bs, progress)
    assert [len(w) for w in W] == [4, 4, 0, 4]
    u, mask, a, g = ow.decode_from_workers(Bs, [0, 1], W, progress)
    assert u == 1 and list(mask) == [0, 0, 1, 0]
    assert np.allclose(g, G.sum(axis=0), rtol=1e-10, atol=1e-10)
