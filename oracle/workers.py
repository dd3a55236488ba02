"""Redundancy-faithful execution of a nested gradient code  (Sec. III).

Each worker computes the partial gradients of its own stored partitions, layer
by layer: first the one of the component code sigma = 0, then the additional
ones of the next larger sigma, and so on (the layered task scheduling after
Def. 2).  The main node watches how many tasks every worker has finished and
stops the iteration as soon as some component code can be decoded: for the code
with tolerance sigma it needs n - sigma workers that have finished all sigma+1
tasks of that layer (Sec. IV, proof of Theorem 1: "n-u+1 workers to finish
layer u", u = sigma+1 tasks).  Those workers send b_sigma^(i) G computed from
their own partial gradients (Sec. II-C).  A conventional gradient code with a
fixed sigma is the same scheme restricted to one layer (Def. 1).

TEST INFRASTRUCTURE ONLY; fp64.
"""
import numpy as np

from . import gradients
from .codes import min_norm_decode_vector
from .coding import Undecodable


def task_order(Bs, i):
    """Partitions worker i works through, in layer order.

    Layer u needs the partitions in supp(b_u^(i)); by nesting (Def. 2) each layer
    only adds partitions to those of the layer below.  Within a layer new
    partitions are taken in cyclic order starting at the worker's own index.
    """
    n, k = Bs[0].shape
    c = k // n
    order = []
    for B in Bs:
        for t in range(k):
            j = (i * c + t) % k
            if B[i, j] != 0.0 and j not in order:
                order.append(j)
    return order


def tasks_needed(Bs, i, u):
    """Number of finished atomic tasks (k/n partial gradients each, Sec. II-C) after
    which worker i can form its layer-u message."""
    n, k = Bs[0].shape
    return int(np.count_nonzero(Bs[u][i])) // (k // n)


def worker_partials(loss, X, Y, theta, Bs, progress, hidden=0, classes=0):
    """W[i] = list of the partial gradients worker i has finished, in task order.
    Every worker computes its own copy (no sharing between workers)."""
    n, k = Bs[0].shape
    out = []
    for i in range(n):
        order = task_order(Bs, i)[: int(progress[i]) * (k // n)]
        out.append([gradients.partial_gradients(loss, X[j:j + 1], Y[j:j + 1], theta,
                                                hidden, classes)[0] for j in order])
    return out


def worker_messages(Bs, W, progress):
    """C[u][i] = sum_t B_u[i][task_t] * W[i][t] for every layer the worker has
    finished; None where it has not."""
    n, k = Bs[0].shape
    C = []
    for u, B in enumerate(Bs):
        row = []
        for i in range(n):
            if progress[i] < tasks_needed(Bs, i, u):
                row.append(None)
                continue
            order = task_order(Bs, i)
            acc = 0.0
            for t, j in enumerate(order[: int(progress[i]) * (k // n)]):
                if B[i, j] != 0.0:
                    acc = acc + B[i, j] * np.asarray(W[i][t], np.float64)
            row.append(acc)
        C.append(row)
    return C


def terminate(Bs, layers, progress, min_layer=0):
    """Termination rule: the smallest layer u >= min_layer for which at least
    n - s_u workers have finished their s_u + 1 tasks.  Returns (u, mask) with
    mask[i] = 1 for workers whose message is not used (they have not finished
    layer u).  min_layer = index of sigma restricts the scheme to a conventional
    gradient code with that fixed sigma."""
    n = Bs[0].shape[0]
    for u in range(min_layer, len(layers)):
        done = np.array([progress[i] >= tasks_needed(Bs, i, u) for i in range(n)])
        if done.sum() >= n - layers[u]:
            return u, (~done).astype(np.uint8)
    raise Undecodable("no component code has enough finished workers yet")


def decode_from_workers(Bs, layers, W, progress, min_layer=0):
    """Main node: choose the layer by the termination rule, take the least-norm
    decode vector over the finished workers, combine their messages."""
    u, mask = terminate(Bs, layers, progress, min_layer)
    S = np.flatnonzero(mask == 0)
    a = min_norm_decode_vector(Bs[u], S)
    C = worker_messages(Bs, W, progress)
    g = 0.0
    for i in S:
        g = g + a[i] * C[u][i]
    return u, mask, a, g


def tasks_executed(progress):
    """Partial-gradient computations actually carried out in the iteration."""
    return int(np.sum(progress))
