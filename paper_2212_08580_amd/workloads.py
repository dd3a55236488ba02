"""Seeded synthetic inputs for the coded-gradient workloads.

This module only draws random data (features, labels, model parameters,
straggler masks).  It holds none of the method's arithmetic: no gradient, no
code construction, no encode/decode.  Both the CPU checker and the GPU library
are fed from here so that they see bit-identical fp32 arrays.

The paper works on a generic data matrix with m rows split into k = n row
blocks (Sec. II-C) and names no data set; every workload below is therefore
synthetic, with the shapes and distributions of the five benchmark
configurations:

  C1  least squares, n=4,  4 x 256 rows,    d=64,   layers s=(0,1), fractional repetition
  C2  logistic,      n=16, 16 x 8192 rows,  d=1024, layers s=(0,1,3,7), cyclic
  C3  least squares, n=32, 32 x 16384 rows, d=4096, layers s=(0,1,3,7,15), cyclic
  C4  2-layer MLP 784-1024-10, n=20, 20 x 3000 rows, layers s=(0,1,4,9), cyclic
  C5  encode/decode stress, n=64, d=16384, layers s=(0,1,3,7,15,31), cyclic

Random streams: numpy PCG64 seeded with SeedSequence([seed, config_id,
stream_id, partition]) so that a partition can be regenerated on its own.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Optional, Sequence, Tuple

import numpy as np

LOSS_LSQ = 0
LOSS_LOGISTIC = 1
LOSS_MLP2 = 2

CODE_CYCLIC = 0
CODE_FRACREP = 1

# stream identifiers inside one configuration
_S_X, _S_NOISE, _S_TRUTH, _S_THETA, _S_MASK, _S_LABEL, _S_G = range(7)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    loss: int                     # LOSS_*; -1 for the encode/decode-only stress case
    n: int                        # workers = partitions (the paper sets k = n)
    rows: int                     # rows per partition, m / k
    d_in: int                     # features per row
    d: int                        # gradient length (the paper's l)
    layers: Tuple[int, ...]       # straggler tolerances s_0 < s_1 < ...
    code: int                     # CODE_*
    p_straggle: float             # per-worker Bernoulli straggler probability
    noise: float                  # label noise standard deviation
    hidden: int = 0               # MLP hidden width
    classes: int = 0              # MLP classes

    @property
    def m(self) -> int:
        return self.n * self.rows

    def scaled(self, rows: Optional[int] = None, d: Optional[int] = None,
               n: Optional[int] = None, layers: Optional[Sequence[int]] = None,
               name: Optional[str] = None) -> "Workload":
        """A shrunken copy with the same distributions (CPU-sized parity cases)."""
        kw = {}
        if rows is not None:
            kw["rows"] = rows
        if d is not None:
            assert self.loss in (LOSS_LSQ, LOSS_LOGISTIC, -1)
            kw["d"] = d
            kw["d_in"] = d
        if n is not None:
            kw["n"] = n
        if layers is not None:
            kw["layers"] = tuple(layers)
        kw["name"] = name or (self.name + "-scaled")
        return dataclasses.replace(self, **kw)


def mlp_param_count(d_in: int, hidden: int, classes: int) -> int:
    return d_in * hidden + hidden + hidden * classes + classes


C1 = Workload("C1-lsq-n4", 1, LOSS_LSQ, 4, 256, 64, 64, (0, 1), CODE_FRACREP, 0.0, 0.01)
C2 = Workload("C2-logistic-n16", 2, LOSS_LOGISTIC, 16, 8192, 1024, 1024, (0, 1, 3, 7),
              CODE_CYCLIC, 0.2, 0.1)
C3 = Workload("C3-lsq-n32-d4096", 3, LOSS_LSQ, 32, 16384, 4096, 4096, (0, 1, 3, 7, 15),
              CODE_CYCLIC, 0.1, 0.01)
C4 = Workload("C4-mlp-n20", 4, LOSS_MLP2, 20, 3000, 784, mlp_param_count(784, 1024, 10),
              (0, 1, 4, 9), CODE_CYCLIC, 0.1, 0.0, hidden=1024, classes=10)
C5 = Workload("C5-codec-n64", 5, -1, 64, 0, 16384, 16384, (0, 1, 3, 7, 15, 31),
              CODE_CYCLIC, 0.2, 0.0)

CONFIGS = {w.name.split("-")[0]: w for w in (C1, C2, C3, C4, C5)}


def _rng(seed: int, w: Workload, stream: int, part: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(
        [int(seed), int(w.config_id), int(stream), int(part)])))


def truth_vector(w: Workload, seed: int = 0) -> np.ndarray:
    """Ground-truth parameter used only to synthesise labels (theta* or w*)."""
    return _rng(seed, w, _S_TRUTH).standard_normal(w.d_in, dtype=np.float32)


def theta(w: Workload, seed: int = 0, scale: Optional[float] = None) -> np.ndarray:
    """Evaluation point of the gradient.

    Regression losses: N(0,1) (a generic point away from the optimum, so the
    gradient is not a difference of nearly equal numbers); pass scale=0.01 for
    the start point of a descent run.  MLP: weights N(0, 1/fan_in), biases 0,
    laid out as [W1 (d_in x hidden) | b1 | W2 (hidden x classes) | b2].
    """
    g = _rng(seed, w, _S_THETA)
    if w.loss == LOSS_MLP2:
        w1 = g.standard_normal((w.d_in, w.hidden), dtype=np.float32) / np.float32(np.sqrt(w.d_in))
        w2 = g.standard_normal((w.hidden, w.classes), dtype=np.float32) / np.float32(np.sqrt(w.hidden))
        return np.concatenate([w1.ravel(), np.zeros(w.hidden, np.float32),
                               w2.ravel(), np.zeros(w.classes, np.float32)])
    t = g.standard_normal(w.d, dtype=np.float32)
    if scale is not None:
        t *= np.float32(scale)
    return t


def partition(w: Workload, j: int, seed: int = 0,
              truth: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Row block j: features [rows, d_in] fp32 and its labels.

    LSQ: y = x.theta* + N(0, noise^2) (fp32).  Logistic: y = sign(x.w* +
    N(0, noise^2)) in {-1,+1} (fp32).  MLP: x ~ U[0,1), y uniform class id
    (int32).
    """
    gx = _rng(seed, w, _S_X, j)
    if w.loss == LOSS_MLP2:
        x = gx.random((w.rows, w.d_in), dtype=np.float32)
        y = _rng(seed, w, _S_LABEL, j).integers(0, w.classes, size=w.rows, dtype=np.int32)
        return x, y
    x = gx.standard_normal((w.rows, w.d_in), dtype=np.float32)
    if truth is None:
        truth = truth_vector(w, seed)
    clean = x.astype(np.float64) @ truth.astype(np.float64)
    noisy = clean + w.noise * _rng(seed, w, _S_NOISE, j).standard_normal(w.rows)
    if w.loss == LOSS_LSQ:
        y = noisy.astype(np.float32)
    else:
        y = np.where(noisy >= 0.0, 1.0, -1.0).astype(np.float32)
    return x, y


def dataset(w: Workload, seed: int = 0, threads: int = 8,
            out_x: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """All partitions stacked: X [n, rows, d_in] fp32 and y [n, rows]."""
    ydt = np.int32 if w.loss == LOSS_MLP2 else np.float32
    X = out_x if out_x is not None else np.empty((w.n, w.rows, w.d_in), np.float32)
    Y = np.empty((w.n, w.rows), ydt)
    truth = None if w.loss == LOSS_MLP2 else truth_vector(w, seed)

    def fill(j: int) -> None:
        X[j], Y[j] = partition(w, j, seed, truth)

    if threads > 1 and w.n > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(w.n)))
    else:
        for j in range(w.n):
            fill(j)
    return X, Y


def partial_gradients(w: Workload, seed: int = 0) -> np.ndarray:
    """Stand-in partition gradients G [n, d] ~ N(0,1) for the encode/decode stress case."""
    return _rng(seed, w, _S_G).standard_normal((w.n, w.d), dtype=np.float32)


def bernoulli_masks(w: Workload, rounds: int, seed: int = 0,
                    p: Optional[float] = None) -> np.ndarray:
    """Straggler masks [rounds, n] uint8 (1 = straggler), each worker i.i.d. Bernoulli(p)."""
    p = w.p_straggle if p is None else p
    return (_rng(seed, w, _S_MASK).random((rounds, w.n)) < p).astype(np.uint8)


def binomial_count_masks(w: Workload, rounds: int, seed: int = 0,
                         p: Optional[float] = None) -> np.ndarray:
    """Masks whose straggler count is Binomial(n, p) and whose members are a
    uniformly random subset of that size."""
    p = w.p_straggle if p is None else p
    g = _rng(seed, w, _S_MASK, 1)
    out = np.zeros((rounds, w.n), np.uint8)
    counts = g.binomial(w.n, p, size=rounds)
    for t in range(rounds):
        out[t, g.choice(w.n, size=int(counts[t]), replace=False)] = 1
    return out
