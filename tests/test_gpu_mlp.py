"""Parity of the 2-layer-perceptron partition gradients (MFMA route) against the
fp64 oracle, through the C ABI.  Bar: rel-L2 <= 1e-4 per partition and per
parameter block (W1, b1, W2, b2)."""
import numpy as np
import pytest

from oracle import codes, coding, gradients
from paper_2212_08580_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-4


def rel(x, ref):
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300))


def mlp_workload(n, rows, d_in, hidden, classes, layers=(0,)):
    import dataclasses
    return dataclasses.replace(wl.C4, name="mlp-%d-%d-%d" % (d_in, hidden, classes), n=n, rows=rows,
                               d_in=d_in, hidden=hidden, classes=classes,
                               d=wl.mlp_param_count(d_in, hidden, classes), layers=tuple(layers))


def run_grads(ngc, torch, w, X, Y, th):
    dev = torch.device("cuda:0")
    ctx = ngc.ngc_create(w.n, w.n, w.layers, w.d, torch.cuda.current_stream().cuda_stream)
    try:
        ngc.ngc_set_mlp2_shape(ctx, w.d_in, w.hidden, w.classes)
        G = torch.empty((w.n, w.d), dtype=torch.float32, device=dev)
        ngc.ngc_partition_grads(ctx, wl.LOSS_MLP2, torch.from_numpy(X).to(dev),
                                torch.from_numpy(Y).to(dev), torch.from_numpy(th).to(dev), w.rows, G)
        ngc.ngc_sync(ctx)
        out = G.cpu().numpy()
        ngc.ngc_partition_grads(ctx, wl.LOSS_MLP2, torch.from_numpy(X).to(dev),
                                torch.from_numpy(Y).to(dev), torch.from_numpy(th).to(dev), w.rows, G)
        ngc.ngc_sync(ctx)
        assert np.array_equal(out, G.cpu().numpy())          # fixed summation order
        return out
    finally:
        ngc.ngc_destroy(ctx)


def check_partition(w, Xj, Yj, th, g, g_o):
    """One partition's gradient against the oracle, block by block.

    ReLU'(z) = [z > 0] is a decision taken on a floating-point number.  Where the
    oracle's fp64 pre-activation z is closer to 0 than fp32 rounding of the dot
    product can resolve, both decisions are valid results; such a (sample, unit)
    pair only moves column `unit` of dW1 and entry `unit` of db1, by x_i * dh and
    dh.  Columns without such a pair are compared as they are; a column with some
    must match the oracle for one assignment of its undecidable pairs.
    """
    d_in, hid, cls = w.d_in, w.hidden, w.classes
    o1 = d_in * hid
    o2 = o1 + hid
    o3 = o2 + hid * cls
    W1, b1, W2, b2 = gradients.mlp2_unpack(th, d_in, hid, cls)
    X = Xj.astype(np.float64)
    Z1 = X @ W1 + b1
    eps32 = 2.0 ** -24
    tau = 8 * eps32 * (np.linalg.norm(X, axis=1)[:, None] * np.linalg.norm(W1, axis=0)[None, :]
                       + np.abs(b1)[None, :])
    ties = np.argwhere(np.abs(Z1) <= tau)
    tied_cols = np.unique(ties[:, 1]) if ties.size else np.array([], int)
    free = np.ones(hid, bool)
    free[tied_cols] = False
    dW1, dW1_o = g[:o1].reshape(d_in, hid).astype(np.float64), g_o[:o1].reshape(d_in, hid)
    db1, db1_o = g[o1:o2].astype(np.float64), g_o[o1:o2]
    assert rel(dW1[:, free], dW1_o[:, free]) <= TOL
    assert rel(db1[free], db1_o[free]) <= TOL
    assert rel(g[o2:o3], g_o[o2:o3]) <= TOL          # dW2
    assert rel(g[o3:], g_o[o3:]) <= TOL              # db2
    if ties.size:
        rows_t = np.unique(ties[:, 0])
        Hh = np.maximum(Z1[rows_t], 0.0)
        Z2 = Hh @ W2 + b2
        E = np.exp(Z2 - Z2.max(axis=1, keepdims=True))
        dZ2 = E / E.sum(axis=1, keepdims=True)
        dZ2[np.arange(rows_t.size), Yj[rows_t]] -= 1.0
        dH = dict(zip(rows_t.tolist(), dZ2 @ W2.T))
        for h in tied_cols:
            members = [int(i) for i, hh in ties if hh == h]
            assert len(members) <= 10
            best = np.inf
            for bits in range(1 << len(members)):
                col, bias = dW1_o[:, h].copy(), db1_o[h]
                for q, i in enumerate(members):
                    if (bits >> q) & 1:                       # take the other decision for pair (i, h)
                        sign = -1.0 if Z1[i, h] > 0 else 1.0
                        col += sign * X[i] * dH[i][h]
                        bias += sign * dH[i][h]
                err = np.sqrt(np.sum((dW1[:, h] - col) ** 2) + (db1[h] - bias) ** 2) / \
                    np.sqrt(np.sum(dW1_o[:, h] ** 2) + db1_o[h] ** 2)
                best = min(best, err)
            assert best <= TOL, (h, members, best)
    return int(ties.shape[0])


def check_blocks(w, X, Y, th, G, G_o):
    undecidable = 0
    for j in range(w.n):
        undecidable += check_partition(w, X[j], Y[j], th, G[j], G_o[j])
    return undecidable


@pytest.mark.parametrize("n,rows,d_in,hidden,classes", [
    (2, 12, 8, 6, 3),            # nothing is a multiple of 4: scalar load/store paths
    (3, 37, 20, 12, 2),
    (2, 130, 100, 256, 10),      # one N tile of two, ragged M and K
    (2, 300, 784, 1024, 10),     # the real layer sizes, few rows
    (1, 257, 33, 1000, 16),
    (2, 5, 784, 1024, 10),       # fewer rows than one K tile
    (2, 40, 256, 64, 5),         # d_in a multiple of 128: backward GEMM on 128-row tiles
    (1, 70, 300, 260, 7),        # both tile shapes ragged in every dimension
    (2, 45, 64, 2048, 10),       # hidden layer wider than one 1024-unit slice of the backward kernel
    (1, 33, 40, 1500, 4),        # ... and a ragged second slice
    (4, 1024, 112, 256, 10),     # backward product: 8 tiles of 112 rows, every one cut along K into pieces
    (5, 1032, 784, 1024, 10),    # ... 280 tiles: 32 whole and 3 cut per XCD, k tiles not a multiple of the pieces
    (3, 1024, 112, 128, 4),      # ... 3 tiles: no multiple of 8, plain launch
    (2, 50, 32, 1024, 4),        # 1024 hidden units: the head in one pass over H, 4 / 16 classes, ragged last trip
    (1, 41, 16, 1024, 16),
    (3, 8, 24, 1024, 10),        # ... exactly one trip of 8 rows per block
])
def test_mlp_partition_gradients_match_oracle(ngc, n, rows, d_in, hidden, classes):
    import torch
    w = mlp_workload(n, rows, d_in, hidden, classes)
    X, Y = wl.dataset(w, seed=rows, threads=1)
    th = wl.theta(w, seed=1)
    # non-zero biases so that the bias paths are exercised
    rng = np.random.default_rng(0)
    o1 = d_in * hidden
    th[o1:o1 + hidden] = 0.1 * rng.standard_normal(hidden).astype(np.float32)
    th[-classes:] = 0.1 * rng.standard_normal(classes).astype(np.float32)
    G = run_grads(ngc, torch, w, X, Y, th)
    G_o = gradients.partial_gradients(wl.LOSS_MLP2, X, Y, th, hidden, classes)
    assert np.all(np.isfinite(G))
    check_blocks(w, X, Y, th, G, G_o)


def test_mlp_needs_shape_and_limits(ngc):
    import torch
    dev = torch.device("cuda:0")
    w = mlp_workload(2, 4, 8, 6, 3)
    ctx = ngc.ngc_create(w.n, w.n, w.layers, w.d, 0)
    try:
        z = torch.zeros(w.d * 2, dtype=torch.float32, device=dev)
        lab = torch.zeros(8, dtype=torch.int32, device=dev)
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_partition_grads(ctx, wl.LOSS_MLP2, z, lab, z, 4, z)
        assert e.value.code == ngc.NGC_ERR_STATE
        with pytest.raises(ngc.NgcError):
            ngc.ngc_set_mlp2_shape(ctx, 8, 7, 3)              # parameter count != d
    finally:
        ngc.ngc_destroy(ctx)


def test_c4_scaled_pipeline(ngc):
    """C4 with fewer rows: n = 20, layers 0,1,4,9 cyclic, 784-1024-10."""
    import torch
    w = mlp_workload(20, 64, 784, 1024, 10, layers=wl.C4.layers)
    X, Y = wl.dataset(w, 0, threads=4)
    th = wl.theta(w, 0)
    dev = torch.device("cuda:0")
    Bs = codes.nested_code(w.n, w.layers, "cyclic", seed=0, draws=2)
    ctx = ngc.ngc_create(w.n, w.n, w.layers, w.d, torch.cuda.current_stream().cuda_stream)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        ngc.ngc_set_mlp2_shape(ctx, w.d_in, w.hidden, w.classes)
        G = torch.empty((w.n, w.d), dtype=torch.float32, device=dev)
        C = torch.empty((len(w.layers), w.n, w.d), dtype=torch.float32, device=dev)
        g = torch.empty(w.d, dtype=torch.float32, device=dev)
        ngc.ngc_partition_grads(ctx, wl.LOSS_MLP2, torch.from_numpy(X).to(dev),
                                torch.from_numpy(Y).to(dev), torch.from_numpy(th).to(dev), w.rows, G)
        ngc.ngc_encode(ctx, G, -1, C)
        G_o = gradients.partial_gradients(wl.LOSS_MLP2, X, Y, th, w.hidden, w.classes)
        check_blocks(w, X, Y, th, G.cpu().numpy(), G_o)
        masks = wl.bernoulli_masks(w, 6, seed=0, p=0.2)
        for m in masks:
            if m.sum() > w.layers[-1]:
                continue
            u, a, r = ngc.ngc_select_decode_vec(ctx, m, w.n)
            ngc.ngc_decode(ctx, u, a, C, g)
            ngc.ngc_sync(ctx)
            u_o, a_o, g_o = coding.coded_gradient(Bs, w.layers, G_o, m)
            assert u == u_o and np.array_equal(a != 0, a_o != 0)
            kappa = coding.conditioning(a_o, coding.encode(Bs[u_o], G_o), g_o)
            err = rel(g.cpu().numpy(), g_o)
            assert err <= max(TOL, 4 * 2.0 ** -24 * kappa), (err, kappa)
    finally:
        ngc.ngc_destroy(ctx)


def test_c4_full_size_gradients(ngc):
    """C4 at full size (20 x 3000 x 784): every partition against the oracle."""
    import torch
    w = wl.C4
    X, Y = wl.dataset(w, 0, threads=8)
    th = wl.theta(w, 0)
    G = run_grads(ngc, torch, w, X, Y, th)
    G_o = gradients.partial_gradients(wl.LOSS_MLP2, X, Y, th, w.hidden, w.classes)
    ties = check_blocks(w, X, Y, th, G, G_o)
    print("C4 full size: %d undecidable ReLU pairs out of %d" % (ties, w.m * w.hidden))
