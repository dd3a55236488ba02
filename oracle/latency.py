"""Latency model of gradient codes and nested gradient codes  (Secs. II-D, IV).

A non-failing worker needs gamma + eps + u*rho + Erlang(u, lambda) to finish u
tasks (eq. (2)); a worker fails for good with probability p_e.  Lemma 1 gives the
latency distribution of a conventional (n,k,sigma) gradient code, Theorem 1 that
of an (n,k,s_max) nested code (component codes sigma = 0..s_max), Corollary 1
its rho = 0 form.  A Monte-Carlo simulation of the same model is the
independent check.  TEST INFRASTRUCTURE ONLY; fp64.

Readings of the paper taken here:
* Eq. (3) prints the sum of the Erlang CDF up to k = u; the CDF of a sum of u
  exponentials stops at u-1.  The proof of Corollary 1 (F_u - F_{u+1} =
  e^{-lambda t}(lambda t)^u/u!) only holds with u-1, which is what is used.
* Theorem 1 prints the summation limit of i_u as min{n-u, n-kappa-sum_{v>u} i_v},
  while its proof states the condition "cannot decode at layer u" as
  i_u <= n-u-sum_{v>u} i_v (fewer than n-u+1 workers have finished u tasks).
  The proof's condition is used: limit = n - max(u, kappa) - sum_{v>u} i_v.  The
  printed limit is available as ngc_cdf(..., printed_limits=True); the simulation
  agrees with the proof's condition, not with the printed limit.
* Corollary 1 prints (e^{lambda t})^{i_0}; the factor for workers that have
  finished nothing is (1 - F_1)^{i_0} = (e^{-lambda t})^{i_0}.
"""
import math

import numpy as np


def layer_cdf(u, t, lam, rho, eps, gamma):
    """F_u(t) = P(gamma + eps + u rho + Erlang(u, lam) <= t)   (eq. (3))."""
    tau = t - (gamma + eps + u * rho)
    if tau < 0:
        return 0.0
    if u == 0:
        return 1.0
    x = lam * tau
    return 1.0 - math.exp(-x) * sum(x ** v / math.factorial(v) for v in range(u))


def gc_cdf(t, n, sigma, lam, rho, eps, gamma, pe):
    """Lemma 1: P(T_GC <= t) for a code that needs n - sigma workers to finish sigma+1 tasks."""
    F = layer_cdf(sigma + 1, t, lam, rho, eps, gamma)
    total = 0.0
    for kappa in range(sigma + 1):
        alive = n - kappa
        cond = sum(math.comb(alive, m) * F ** m * (1.0 - F) ** (alive - m)
                   for m in range(n - sigma, alive + 1))
        total += cond * math.comb(n, kappa) * pe ** kappa * (1.0 - pe) ** (n - kappa)
    return total


def ngc_conditional_cdf(t, n, smax, kappa, lam, rho, eps, gamma, printed_limits=False):
    """Theorem 1, P(T_NGC <= t | kappa failed workers): one minus the probability of
    every configuration (i_1 .. i_{smax+1}) of "workers that have finished exactly u
    tasks" in which no layer has its n-u+1 finishers."""
    F = [layer_cdf(u, t, lam, rho, eps, gamma) for u in range(smax + 3)]
    alive = n - kappa
    top = smax + 1

    def inner(u, above, weight):
        # above = sum_{v>u} i_v ; weight = product of the factors of layers > u
        if u == 0:
            i0 = alive - above
            return weight * (1.0 - F[1]) ** i0
        if printed_limits:
            limit = min(n - u, alive - above)
        else:
            limit = min(n - u - above, alive - above)
        p = F[top] if u == top else F[u] - F[u + 1]
        acc = 0.0
        for iu in range(0, limit + 1):
            acc += inner(u - 1, above + iu, weight * math.comb(alive - above, iu) * p ** iu)
        return acc

    return 1.0 - inner(top, 0, 1.0)


def ngc_cdf(t, n, smax, lam, rho, eps, gamma, pe, printed_limits=False):
    """Theorem 1: P(T_NGC <= t), failures marginalised up to smax."""
    return sum(ngc_conditional_cdf(t, n, smax, kappa, lam, rho, eps, gamma, printed_limits)
               * math.comb(n, kappa) * pe ** kappa * (1.0 - pe) ** (n - kappa)
               for kappa in range(smax + 1))


def ngc_conditional_cdf_rho0(t, n, smax, kappa, lam, eps, gamma):
    """Corollary 1 (rho = 0): the middle factors become Poisson weights."""
    x = lam * max(t - gamma - eps, 0.0)
    if t - gamma - eps < 0:
        return 0.0
    alive = n - kappa
    top = smax + 1
    pois = [math.exp(-x) * x ** u / math.factorial(u) for u in range(top + 1)]
    F_top = 1.0 - sum(pois[:top])

    def inner(u, above, weight):
        if u == 0:
            return weight * pois[0] ** (alive - above)
        limit = min(n - u - above, alive - above)
        p = F_top if u == top else pois[u]
        return sum(inner(u - 1, above + iu, weight * math.comb(alive - above, iu) * p ** iu)
                   for iu in range(0, limit + 1))

    return 1.0 - inner(top, 0, 1.0)


# ---------------------------------------------------------------------------
# Monte-Carlo simulation of eq. (2), with random numbers from Philox-4x32-10
# (Salmon et al., SC'11) so that an independent implementation can reproduce
# every draw: key = seed, counter = (trial, worker, block, 0).
# ---------------------------------------------------------------------------
_M0, _M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)


def philox4x32(c0, c1, c2, c3, k0, k1):
    """Ten rounds of Philox-4x32 on arrays of 32-bit counters (held in uint64)."""
    c0, c1, c2, c3 = (np.asarray(c, np.uint64) & _MASK for c in (c0, c1, c2, c3))
    k0, k1 = int(k0) & 0xFFFFFFFF, int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        n0 = ((p1 >> np.uint64(32)) ^ c1 ^ np.uint64(k0)) & _MASK
        n1 = p1 & _MASK
        n2 = ((p0 >> np.uint64(32)) ^ c3 ^ np.uint64(k1)) & _MASK
        n3 = p0 & _MASK
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return c0, c1, c2, c3


def _uniforms(trials, n, count, seed):
    """U[trial, worker, j] in (0,1), j < count: word j%4 of block j//4."""
    tr = np.arange(trials, dtype=np.uint64)[:, None, None]
    wk = np.arange(n, dtype=np.uint64)[None, :, None]
    blocks = (count + 3) // 4
    bl = np.arange(blocks, dtype=np.uint64)[None, None, :]
    shape = (trials, n, blocks)
    words = philox4x32(np.broadcast_to(tr, shape), np.broadcast_to(wk, shape),
                       np.broadcast_to(bl, shape), np.zeros(shape, np.uint64),
                       seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    U = np.stack(words, axis=-1).reshape(trials, n, blocks * 4)[:, :, :count]
    return (U.astype(np.float64) + 0.5) / 4294967296.0


def simulate(trials, n, smax, lam, rho, eps, gamma, pe, seed=0):
    """Per trial: L[u-1] = time at which n-u+1 workers have finished u tasks, u = 1..smax+1
    (inf if never).  The conventional code with tolerance sigma has latency L[sigma], the
    nested code min_u L[u-1].  Word 0 of a worker decides failure (< p_e), words 1.. are
    its task times rho - log(U)/lam."""
    top = smax + 1
    U = _uniforms(trials, n, top + 1, seed)
    fail = U[:, :, 0] < pe
    task = rho - np.log(U[:, :, 1:]) / lam
    done = gamma + eps + np.cumsum(task, axis=2)                 # [trial, worker, u-1]
    done[fail] = np.inf
    srt = -np.sort(-done, axis=1)                                # descending over workers
    L = np.stack([srt[:, u - 1, u - 1] for u in range(1, top + 1)], axis=1)   # u-th largest
    return L


def empirical_cdf(samples, t):
    return float(np.mean(samples <= t))
