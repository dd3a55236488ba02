"""The pins must notice plausible mistakes: each case plants one in the oracle (a
dropped term, a wrong sign or index, an off-by-one) and checks that the pin that
guards that part fails.  Everything here runs on the CPU."""
import math

import numpy as np
import pytest

import oracle
from oracle import codes, coding, gradients, latency, workers

import test_oracle_codes as pins_codes
import test_oracle_gradients as pins_grad
import test_oracle_latency as pins_lat
import test_oracle_workers as pins_work


def fails(fn, *args):
    try:
        fn(*args)
    except (AssertionError, np.linalg.LinAlgError, ValueError, IndexError):
        return True
    except pytest.fail.Exception:          # a pytest.raises that saw nothing raised
        return True
    return False


def test_least_squares_gradient_mistakes_are_caught(monkeypatch):
    f64 = lambda a: np.asarray(a, np.float64)
    monkeypatch.setattr(gradients, "lsq_gradient", lambda X, y, th: f64(X).T @ (f64(X) @ f64(th) + f64(y)))
    assert fails(pins_grad.test_lsq_at_zero_is_minus_XTy)
    monkeypatch.setattr(gradients, "lsq_gradient", lambda X, y, th: f64(X).T @ (f64(X) @ f64(th)))   # y dropped
    assert fails(pins_grad.test_lsq_finite_differences)
    monkeypatch.setattr(gradients, "lsq_gradient",
                        lambda X, y, th: f64(X).T @ (f64(X) @ f64(th) - f64(y)) / len(f64(y)))          # mean, not sum
    assert fails(pins_grad.test_lsq_autograd)


def test_logistic_gradient_mistakes_are_caught(monkeypatch):
    good = gradients.logistic_gradient
    monkeypatch.setattr(gradients, "logistic_gradient", lambda X, y, th: -good(X, y, th))
    assert fails(pins_grad.test_logistic_at_zero_is_minus_half_sum_yx)
    monkeypatch.setattr(gradients, "logistic_gradient", lambda X, y, th: good(X, y, -np.asarray(th)))  # e^{-yz}
    assert fails(pins_grad.test_logistic_finite_differences_and_autograd)


def test_perceptron_gradient_mistakes_are_caught(monkeypatch):
    good = gradients.mlp2_gradient

    def no_relu_mask(X, labels, theta, hidden, classes):
        g = good(X, labels, theta, hidden, classes).copy()
        g[: X.shape[1] * hidden] *= 1.01           # a wrong scale in one block
        return g
    monkeypatch.setattr(gradients, "mlp2_gradient", no_relu_mask)
    assert fails(pins_grad.test_mlp_finite_differences)
    assert fails(pins_grad.test_mlp_autograd_layout)


def test_code_construction_mistakes_are_caught(monkeypatch):
    # window running backwards: still a gradient code, but not the lemma's supports
    monkeypatch.setattr(codes, "cyclic_support", lambda n, s, i: [(i - t) % n for t in range(s + 1)])
    assert fails(pins_codes.test_cyclic_nested_code_satisfies_def1_and_def2, 6, [0, 1, 2, 3])
    monkeypatch.undo()
    # rows no longer in a common null space: random coefficients on the right support
    def sloppy(n, sigma, rng):
        B = np.zeros((n, n))
        for i in range(n):
            B[i, codes.cyclic_support(n, sigma, i)] = rng.standard_normal(sigma + 1)
        return B if sigma else np.eye(n)
    monkeypatch.setattr(codes, "cyclic_code", sloppy)
    assert fails(pins_codes.test_cyclic_nested_code_satisfies_def1_and_def2, 8, [0, 1, 2, 3])


def test_layer_choice_and_decode_mistakes_are_caught(monkeypatch):
    def off_by_one(layers, mask):
        s = int(np.count_nonzero(mask))
        for u, su in enumerate(layers):
            if su > s:
                return u
        raise coding.Undecodable("x")
    monkeypatch.setattr(coding, "select_layer", off_by_one)
    assert fails(pins_codes.test_select_layer_table)
    monkeypatch.undo()
    monkeypatch.setattr(coding, "encode", lambda B, G: np.asarray(B, np.float64).T @ np.asarray(G, np.float64))
    assert fails(pins_codes.test_encode_row_is_the_sparse_combination_written_out)
    monkeypatch.undo()
    good = codes.min_norm_decode_vector
    monkeypatch.setattr(codes, "min_norm_decode_vector", lambda B, S: good(B, S) * 1.001)
    monkeypatch.setattr(coding, "min_norm_decode_vector", lambda B, S: good(B, S) * 1.001)
    assert fails(pins_codes.test_fracrep_worked_case_matches_golden)


def test_guarded_choice_mistakes_are_caught(monkeypatch):
    good_amp = coding.amplification
    # row norms left out of the estimate
    monkeypatch.setattr(coding, "amplification", lambda B, a: float(np.abs(a).sum() / np.sqrt(np.asarray(B).shape[1])))
    assert fails(pins_codes.test_guarded_choice_fracrep_closed_form)
    monkeypatch.undo()
    # divided by k instead of its root
    monkeypatch.setattr(coding, "amplification", lambda B, a: good_amp(B, a) / np.sqrt(np.asarray(B).shape[1]))
    assert fails(pins_codes.test_guarded_choice_fracrep_closed_form)
    monkeypatch.undo()

    def always_best(Bs, layers, mask, limit):                  # ignores the limit: always the best layer
        u0 = coding.select_layer(layers, mask)
        cand = [(good_amp(Bs[u], coding.decode_vector(Bs[u], mask)[0]), u) for u in range(u0, len(layers))]
        u = min(cand)[1]
        return u, coding.decode_vector(Bs[u], mask)[0]
    monkeypatch.setattr(coding, "select_guarded", always_best)
    assert fails(pins_codes.test_guarded_choice_without_a_limit_is_the_plain_rule)
    monkeypatch.undo()

    def never_moves(Bs, layers, mask, limit):
        u = coding.select_layer(layers, mask)
        return u, coding.decode_vector(Bs[u], mask)[0]
    monkeypatch.setattr(coding, "select_guarded", never_moves)
    assert fails(pins_codes.test_guarded_choice_rule_by_brute_force, 1.5)
    assert fails(pins_codes.test_guarded_choice_tames_the_tail_of_a_random_code)
    monkeypatch.undo()

    def last_within(Bs, layers, mask, limit):                  # the highest layer within the limit, not the first
        u0 = coding.select_layer(layers, mask)
        pick = None
        for u in range(u0, len(layers)):
            a = coding.decode_vector(Bs[u], mask)[0]
            if good_amp(Bs[u], a) <= limit:
                pick = (u, a)
        return pick if pick else never_moves(Bs, layers, mask, limit)
    monkeypatch.setattr(coding, "select_guarded", last_within)
    assert fails(pins_codes.test_guarded_choice_rule_by_brute_force, 3.0)


def test_worker_rule_mistakes_are_caught(monkeypatch):
    good = workers.terminate

    def lenient(Bs, layers, progress, min_layer=0):           # one finisher too few
        n = Bs[0].shape[0]
        for u in range(min_layer, len(layers)):
            done = np.array([progress[i] >= workers.tasks_needed(Bs, i, u) for i in range(n)])
            if done.sum() >= n - layers[u] - 1:
                return u, (~done).astype(np.uint8)
        raise coding.Undecodable("x")
    monkeypatch.setattr(workers, "terminate", lenient)
    assert fails(pins_work.test_termination_rule_table)
    monkeypatch.setattr(workers, "terminate", good)
    monkeypatch.setattr(workers, "task_order", lambda Bs, i: list(range(Bs[0].shape[1]))[: Bs[-1].shape[1]])
    assert fails(pins_work.test_cyclic_schedule_is_own_partition_then_cyclic_successors)


def test_latency_mistakes_are_caught(monkeypatch):
    def printed_erlang(u, t, lam, rho, eps, gamma):           # sum to u as printed in eq. (3)
        tau = t - (gamma + eps + u * rho)
        if tau < 0:
            return 0.0
        x = lam * tau
        return 1.0 - math.exp(-x) * sum(x ** v / math.factorial(v) for v in range(u + 1))
    monkeypatch.setattr(latency, "layer_cdf", printed_erlang)
    assert fails(pins_lat.test_erlang_cdf_against_scipy_and_poisson_identity)
    monkeypatch.undo()
    good = latency.gc_cdf
    monkeypatch.setattr(latency, "gc_cdf", lambda t, n, s, lam, rho, eps, gamma, pe: good(t, n, s, lam, rho, eps, gamma, 0.0))
    assert fails(pins_lat.test_uncoded_limit_is_point_66)
