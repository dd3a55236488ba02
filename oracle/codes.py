"""Construction of nested gradient codes  (Sec. III: Defs. 1-2, Alg. 1, Lemma 2).

An (n,k,sigma) gradient code needs an encoding matrix B_sigma (n x k) such that
any n-sigma rows span a subspace containing the all-ones row, with at least
(k/n)(sigma+1) non-zeros per row (Def. 1).  A nested code is a family of such
matrices whose row supports grow with sigma (Def. 2).  k = n throughout
(Sec. II-C).  TEST INFRASTRUCTURE ONLY; fp64.

Readings of the paper taken here:
* Lemma 2 prints the cyclic support as {i,...,i+sigma+1}; that has sigma+2
  elements, which contradicts B_0 = I (Alg. 1) and the load (k/n)(sigma+1)
  (Sec. II-C).  The support used is {i,...,i+sigma} mod n.
* Alg. 1 obtains the coefficients from a routine of the cited gradient-coding
  paper that is not reproduced.  Any B with that support which satisfies Def. 1
  is a valid outcome; the one built here puts every row into the null space of
  a random sigma x n matrix H with H 1 = 0, so that all rows lie in an
  (n-sigma)-dimensional space that contains 1 and any n-sigma of them are a
  basis of it with probability one.
* Fractional repetition is only named in Sec. I; the block form used here
  (worker i shares the all-ones row of its block of sigma+1 consecutive
  partitions) keeps i in its own support, as Def. 2 with B_0 = I requires.
* Layers may be a subset of sigma = 0..s_max; inclusion of supports is
  transitive so a subset of component codes is still nested.
"""
import itertools

import numpy as np


def cyclic_support(n, sigma, i):
    """Columns {i, ..., i+sigma} mod n of row i (0-based)."""
    return [(i + t) % n for t in range(sigma + 1)]


def fracrep_support(n, sigma, i):
    """Block {w*floor(i/w), ..., +w-1}, w = sigma+1, which must divide n."""
    w = sigma + 1
    if n % w:
        raise ValueError("fractional repetition needs (sigma+1) | n")
    return list(range(w * (i // w), w * (i // w) + w))


def identity_code(n):
    """B_0 = I (Alg. 1, first step)."""
    return np.eye(n)


def cyclic_code(n, sigma, rng):
    """B_sigma with cyclic support and rows in null(H), H random with H 1 = 0.

    Row i has coefficient 1 at column i; the other sigma coefficients solve the
    sigma x sigma system that makes H b_i = 0.
    """
    if sigma == 0:
        return identity_code(n)
    if not 0 < sigma < n:
        raise ValueError("need 0 <= sigma < n")
    H = rng.standard_normal((sigma, n))
    H[:, n - 1] = -H[:, : n - 1].sum(axis=1)
    B = np.zeros((n, n))
    for i in range(n):
        cols = cyclic_support(n, sigma, i)
        rest = cols[1:]
        x = np.linalg.solve(H[:, rest], -H[:, i])
        B[i, i] = 1.0
        B[i, rest] = x
    return B


def fracrep_code(n, sigma):
    """Block fractional-repetition B_sigma: ones on the worker's block."""
    B = np.zeros((n, n))
    for i in range(n):
        B[i, fracrep_support(n, sigma, i)] = 1.0
    return B


def min_norm_decode_vector(B, responders):
    """a with a_S^T B_S = 1^T of least 2-norm, zero outside S (Def. 1, last two bullets).

    The rows of a component code span n - sigma dimensions (Def. 1, second bullet), fewer than
    there are responders whenever more than n - sigma respond; singular values below 1e-10 of
    the largest are the rounding of the construction (for sigma = n - 1 every row is the
    all-ones vector up to 1e-14), not part of the code, and are cut."""
    n = B.shape[0]
    S = np.asarray(responders, dtype=int)
    a = np.zeros(n)
    if S.size:
        sol = np.linalg.lstsq(B[S].T, np.ones(B.shape[1]), rcond=1e-10)[0]
        a[S] = sol
    return a


def amplification_score(B, sigma, rng, samples=32):
    """Mean over random straggler sets of size sigma of sum_i |a_i| ||b_i||_1.

    Measures how much rounding of the worker messages is magnified by decoding;
    used only to choose between equally valid random draws.
    """
    n = B.shape[0]
    l1 = np.abs(B).sum(axis=1)
    tot = 0.0
    for _ in range(samples):
        out = rng.choice(n, size=sigma, replace=False)
        S = np.setdiff1d(np.arange(n), out)
        a = min_norm_decode_vector(B, S)
        tot += float(np.abs(a) @ l1)
    return tot / samples


def nested_code(n, layers, kind="cyclic", seed=0, draws=16):
    """[B^(0), ..., B^(L-1)] for tolerances layers[0] < layers[1] < ...  (Alg. 1).

    kind "cyclic": each layer with sigma > 0 is the best of `draws` random
    cyclic codes by amplification_score.  kind "fracrep": block codes, nested
    iff (s_u + 1) divides (s_{u+1} + 1).
    """
    layers = list(layers)
    if layers != sorted(set(layers)) or layers[0] != 0:
        raise ValueError("layers must be strictly ascending and start at 0")
    out = []
    for u, sigma in enumerate(layers):
        if sigma == 0:
            out.append(identity_code(n))
        elif kind == "fracrep":
            if (sigma + 1) % (layers[u - 1] + 1):
                raise ValueError("fractional-repetition layers are not nested")
            out.append(fracrep_code(n, sigma))
        elif kind == "cyclic":
            best, best_score = None, np.inf
            for t in range(draws):
                ss = np.random.SeedSequence([int(seed), n, sigma, t])
                B = cyclic_code(n, sigma, np.random.Generator(np.random.PCG64(ss)))
                score = amplification_score(
                    B, sigma, np.random.Generator(np.random.PCG64(
                        np.random.SeedSequence([int(seed), n, sigma, 1000]))))
                if score < best_score:
                    best, best_score = B, score
            out.append(best)
        else:
            raise ValueError("unknown code kind %r" % (kind,))
    return out


def expand_partitions(Bs, c):
    """Codes for k = c*n partitions (Sec. II-C: an atomic task is k/n partial
    gradients, assigned jointly): worker i treats the c partitions of group j
    like the single partition j of the k = n code, B = B' (x) 1_{1 x c}.  Row
    weight becomes (k/n)(sigma+1) and a B = 1_k whenever a B' = 1_n."""
    return [np.kron(np.asarray(B, np.float64), np.ones((1, int(c)))) for B in Bs]


def decoding_matrix(B, sigma):
    """A_sigma with one row per straggler set of size sigma (Def. 1): row j is
    supported on the j-th (n-sigma)-subset and satisfies a_j B = 1.
    Only for small n: it has C(n, sigma) rows."""
    n = B.shape[0]
    rows = []
    for out in itertools.combinations(range(n), sigma):
        S = [i for i in range(n) if i not in out]
        rows.append(min_norm_decode_vector(B, S))
    return np.array(rows)
