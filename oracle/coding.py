"""Encode, layer choice, decode-vector selection and decode  (Secs. II-C, III).

TEST INFRASTRUCTURE ONLY; fp64 unless a dtype is asked for.

Notation: G (k x l) stacks the partial gradients; worker i's message under the
component code sigma is row i of B_sigma G (the paper writes X = B G; C is used
here because X names the data in the workloads); a is the row of A_sigma whose
support lies inside the responder set, so that a B_sigma = 1 and
sum_i a_i c_i = 1^T G, the full gradient (Def. 1).

Readings:
* When more than n-sigma workers respond the paper asks only for *some* row of
  A_sigma supported on responders.  The least-2-norm solution over all
  responders is used: it is unique, equals the only solution when exactly
  n-sigma respond, and magnifies message rounding least.
* The layer used is the smallest tolerance s_u >= number of stragglers (the
  Observation after Def. 2); more stragglers than s_max cannot be decoded
  (Theorem 1 sums failures only up to s_max).
* Guarded layer choice (an option, off unless asked for): every component code
  with s_v >= number of stragglers recovers the gradient (Def. 1), and when all
  responders hold all their layers' messages the main node is free to take a
  larger one.  With exactly s_u stragglers the layer-u decode vector is the only
  one there is and can be huge for a real-valued code; the guard then moves up
  to the first layer whose estimated amplification of message rounding,
  kappa_hat = sum_i |a_i| ||b_i||_2 / sqrt(k)  (what `conditioning` gives for
  partial gradients with independent entries of equal variance), is within a
  limit, and to the layer of smallest kappa_hat if none is.
"""
import numpy as np

from .codes import min_norm_decode_vector


class Undecodable(Exception):
    """More stragglers than the largest tolerance."""


def encode(B, G):
    """C = B G: one message per worker (Sec. II-C)."""
    return np.asarray(B, np.float64) @ np.asarray(G, np.float64)


def encode_layers(Bs, G):
    """Messages of every layer, stacked [L, n, l]."""
    return np.stack([encode(B, G) for B in Bs])


def select_layer(layers, mask):
    """u* = min{u : s_u >= #stragglers}; mask[i] = 1 marks worker i a straggler."""
    s = int(np.count_nonzero(mask))
    for u, su in enumerate(layers):
        if su >= s:
            return u
    raise Undecodable("%d stragglers exceed tolerance %d" % (s, layers[-1]))


def decode_vector(B, mask):
    """Least-norm a with a^T B = 1^T and a_i = 0 at stragglers; also max |a^T B - 1|."""
    S = np.flatnonzero(np.asarray(mask) == 0)
    a = min_norm_decode_vector(np.asarray(B, np.float64), S)
    resid = float(np.max(np.abs(a @ B - 1.0)))
    return a, resid


def decode_vector_first(B, sigma, mask):
    """The row of A_sigma for the n-sigma responders of lowest index (a literal
    row of the decoding matrix of Def. 1)."""
    S = np.flatnonzero(np.asarray(mask) == 0)[: B.shape[0] - sigma]
    a = min_norm_decode_vector(np.asarray(B, np.float64), S)
    return a, float(np.max(np.abs(a @ B - 1.0)))


def decode(a, C):
    """g_hat = sum_{i in S} a_i c_i."""
    a = np.asarray(a, np.float64)
    S = np.flatnonzero(a != 0.0)
    return a[S] @ np.asarray(C, np.float64)[S]


def conditioning(a, C, g):
    """kappa = sum_i |a_i| ||c_i||_2 / ||g||_2: bound on how rounding of the
    messages (relative size eps each) shows up in the decoded vector."""
    C = np.asarray(C, np.float64)
    return float(np.abs(a) @ np.linalg.norm(C, axis=1) / max(np.linalg.norm(g), 1e-300))


def amplification(B, a):
    """kappa_hat = sum_i |a_i| ||b_i||_2 / sqrt(k) for the decode vector a of the code B."""
    B = np.asarray(B, np.float64)
    return float(np.abs(np.asarray(a, np.float64)) @ np.linalg.norm(B, axis=1) / np.sqrt(B.shape[1]))


def select_guarded(Bs, layers, mask, kappa_limit):
    """(u, a): the smallest layer u with s_u >= #stragglers whose decode vector has
    kappa_hat <= kappa_limit; the layer of smallest kappa_hat (the lowest of them on a tie)
    if no layer meets the limit.  kappa_limit = inf is the plain rule of `select_layer`."""
    u0 = select_layer(layers, mask)
    best = None
    for u in range(u0, len(layers)):
        a, _ = decode_vector(Bs[u], mask)
        kh = amplification(Bs[u], a)
        if kh <= kappa_limit:
            return u, a
        if best is None or kh < best[0]:
            best = (kh, u, a)
    return best[1], best[2]


def coded_gradient(Bs, layers, G, mask, message_dtype=np.float64):
    """One iteration's main-node result: (u*, a, g_hat).

    message_dtype=float32 rounds each worker message to fp32 before decoding,
    as a worker that sends fp32 does.
    """
    u = select_layer(layers, mask)
    a, _ = decode_vector(Bs[u], mask)
    C = encode(Bs[u], G).astype(message_dtype)
    return u, a, decode(a, C)
