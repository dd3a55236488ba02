"""Parity of the redundancy-faithful worker execution (every worker computes its
own partial gradients layer by layer, encodes from its own copies; the main
node stops by the termination rule) against the oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import codes, coding, gradients, workers as ow
from paper_2212_08580_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-4


def rel(x, ref):
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300))


@pytest.mark.parametrize("base,n,rows,d,layers,kind", [
    (wl.C3, 8, 37, 4096, (0, 1, 3), "cyclic"),
    (wl.C2, 8, 50, 1024, (0, 1, 3, 7), "fracrep"),
    (wl.C1, 4, 256, 64, (0, 1), "fracrep"),          # two-pass route (d = 64)
    (wl.C3, 6, 21, 200, (0, 2, 3), "cyclic"),
])
def test_worker_execution_matches_oracle(ngc, base, n, rows, d, layers, kind):
    import torch
    dev = torch.device("cuda:0")
    w = base.scaled(rows=rows, d=d, n=n, layers=layers)
    X, Y = wl.dataset(w, seed=1, threads=1)
    scale = None if w.loss == wl.LOSS_LSQ else 2.0 / np.sqrt(d)
    th = wl.theta(w, seed=2, scale=scale)
    Bs = codes.nested_code(n, layers, kind, seed=0, draws=2)
    G_o = gradients.partial_gradients(w.loss, X, Y, th)
    full = G_o.sum(axis=0)
    ctx = ngc.ngc_create(n, n, layers, d, torch.cuda.current_stream().cuda_stream)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        T = ngc.ngc_worker_task_count(ctx)
        assert T == layers[-1] + 1
        Xd, Yd, thd = (torch.from_numpy(a).to(dev) for a in (X, Y, th))
        C = torch.empty((len(layers), n, d), dtype=torch.float32, device=dev)
        g = torch.empty(d, dtype=torch.float32, device=dev)
        rng = np.random.default_rng(3)
        cases = [np.full(n, T), np.full(n, 1), rng.integers(0, T + 1, n), rng.integers(0, T + 1, n),
                 np.array([0] + [T] * (n - 1))]
        decoded = 0
        for progress in cases:
            W = torch.full((n, T, d), 7.0, dtype=torch.float32, device=dev)
            ngc.ngc_worker_grads(ctx, w.loss, Xd, Yd, thd, rows, progress, W)
            ngc.ngc_worker_encode(ctx, W, progress, C)
            ngc.ngc_sync(ctx)
            Wh, Ch = W.cpu().numpy(), C.cpu().numpy()
            W_o = ow.worker_partials(w.loss, X, Y, th, Bs, progress)
            C_o = ow.worker_messages(Bs, W_o, progress)
            for i in range(n):
                for t in range(T):
                    if t < progress[i]:
                        assert rel(Wh[i, t], W_o[i][t]) <= TOL
                        # the worker's own copy is the same computation as the shared one: bit-equal
                        assert np.array_equal(Wh[i, t], Wh[ow.task_order(Bs, i)[t], 0]) or \
                            progress[ow.task_order(Bs, i)[t]] == 0
                    else:
                        assert np.all(Wh[i, t] == 7.0)               # untouched
            for u in range(len(layers)):
                for i in range(n):
                    if C_o[u][i] is None:
                        assert np.all(Ch[u, i] == 0.0)
                    else:
                        assert rel(Ch[u, i], C_o[u][i]) <= TOL
            for min_layer in (0, len(layers) - 1):
                try:
                    u_o, mask_o, a_o, g_o = ow.decode_from_workers(Bs, layers, W_o, progress, min_layer)
                except coding.Undecodable:
                    with pytest.raises(ngc.NgcError):
                        ngc.ngc_select_from_progress(ctx, progress, n, min_layer)
                    continue
                u, mask, a, r = ngc.ngc_select_from_progress(ctx, progress, n, min_layer)
                assert u == u_o and np.array_equal(mask, mask_o) and np.array_equal(a != 0, a_o != 0)
                ngc.ngc_decode(ctx, u, a, C, g)
                ngc.ngc_sync(ctx)
                msgs = np.stack([C_o[u_o][i] if C_o[u_o][i] is not None else np.zeros(d) for i in range(n)])
                kappa = coding.conditioning(a_o, msgs, full)
                err = rel(g.cpu().numpy(), full)                     # exact recovery of sum_j g_j
                assert err <= max(TOL, 4 * 2.0 ** -24 * kappa), (err, kappa)
                decoded += 1
        assert decoded >= 4
    finally:
        ngc.ngc_destroy(ctx)


@pytest.mark.parametrize("n,rows,d_in,hidden,classes,layers", [
    (5, 37, 20, 24, 5, (0, 1, 3)),          # guarded loads everywhere (nothing a multiple of 4 but d_in)
    (4, 150, 112, 128, 10, (0, 2)),         # vector loads, the 112-row tile of the backward product
])
def test_worker_execution_with_the_perceptron_loss(ngc, n, rows, d_in, hidden, classes, layers):
    """Each worker's own copies of the perceptron gradients (several units reading the same
    partition in one batched launch), the messages formed from them, and the decoded sum."""
    import dataclasses
    import torch
    dev = torch.device("cuda:0")
    d = wl.mlp_param_count(d_in, hidden, classes)
    w = dataclasses.replace(wl.C4, name="mlp-workers", n=n, rows=rows, d_in=d_in, hidden=hidden,
                            classes=classes, d=d, layers=tuple(layers))
    X, Y = wl.dataset(w, seed=4, threads=1)
    th = wl.theta(w, seed=5)
    Bs = codes.nested_code(n, layers, "cyclic", seed=0, draws=2)
    G_o = gradients.partial_gradients(wl.LOSS_MLP2, X, Y, th, hidden, classes)
    full = G_o.sum(axis=0)
    ctx = ngc.ngc_create(n, n, layers, d, torch.cuda.current_stream().cuda_stream)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        ngc.ngc_set_mlp2_shape(ctx, d_in, hidden, classes)
        T = ngc.ngc_worker_task_count(ctx)
        Xd, Yd, thd = (torch.from_numpy(a).to(dev) for a in (X, Y, th))
        C = torch.empty((len(layers), n, d), dtype=torch.float32, device=dev)
        g = torch.empty(d, dtype=torch.float32, device=dev)
        rng = np.random.default_rng(6)
        decoded = 0
        for progress in (np.full(n, T), rng.integers(1, T + 1, n), np.array([0] + [T] * (n - 1))):
            W = torch.full((n, T, d), 7.0, dtype=torch.float32, device=dev)
            ngc.ngc_worker_grads(ctx, wl.LOSS_MLP2, Xd, Yd, thd, rows, progress, W)
            ngc.ngc_worker_encode(ctx, W, progress, C)
            ngc.ngc_sync(ctx)
            Wh, Ch = W.cpu().numpy(), C.cpu().numpy()
            W_o = ow.worker_partials(wl.LOSS_MLP2, X, Y, th, Bs, progress, hidden, classes)
            C_o = ow.worker_messages(Bs, W_o, progress)
            for i in range(n):
                for t in range(T):
                    if t < progress[i]:
                        assert rel(Wh[i, t], W_o[i][t]) <= TOL, (i, t)
                    else:
                        assert np.all(Wh[i, t] == 7.0)
            for u in range(len(layers)):
                for i in range(n):
                    if C_o[u][i] is None:
                        assert np.all(Ch[u, i] == 0.0)
                    else:
                        assert rel(Ch[u, i], C_o[u][i]) <= TOL
            try:
                u_o, mask_o, a_o, g_o = ow.decode_from_workers(Bs, layers, W_o, progress, 0)
            except coding.Undecodable:
                continue
            u, mask, a, r = ngc.ngc_select_from_progress(ctx, progress, n, 0)
            assert u == u_o and np.array_equal(mask, mask_o)
            ngc.ngc_decode(ctx, u, a, C, g)
            ngc.ngc_sync(ctx)
            msgs = np.stack([C_o[u_o][i] if C_o[u_o][i] is not None else np.zeros(d) for i in range(n)])
            kappa = coding.conditioning(a_o, msgs, full)
            err = rel(g.cpu().numpy(), full)
            assert err <= max(TOL, 4 * 2.0 ** -24 * kappa), (err, kappa)
            decoded += 1
        assert decoded >= 2
    finally:
        ngc.ngc_destroy(ctx)


def test_worker_calls_reject_bad_arguments(ngc):
    import torch
    dev = torch.device("cuda:0")
    ctx = ngc.ngc_create(4, 4, (0, 1), 256, 0)
    try:
        z = torch.zeros(4 * 2 * 256, dtype=torch.float32, device=dev)
        with pytest.raises(ngc.NgcError) as e:                       # layer 1 has no code yet
            ngc.ngc_worker_grads(ctx, 0, z, z, z, 1, [1, 1, 1, 1], z)
        assert e.value.code == ngc.NGC_ERR_STATE
        ngc.ngc_build_code(ctx, ngc.NGC_CODE_FRACREP, 0)
        lab = torch.zeros(16, dtype=torch.int32, device=dev)
        with pytest.raises(ngc.NgcError) as e:                       # perceptron loss without its shape
            ngc.ngc_worker_grads(ctx, 2, z, lab, z, 1, [1, 1, 1, 1], z)
        assert e.value.code == ngc.NGC_ERR_STATE
        with pytest.raises(ngc.NgcError):
            ngc.ngc_worker_grads(ctx, 3, z, z, z, 1, [1, 1, 1, 1], z)    # no such loss
        # the binding checks what the library cannot see behind a bare pointer
        short = torch.zeros(100, dtype=torch.float32, device=dev)
        with pytest.raises(ValueError):
            ngc.ngc_worker_grads(ctx, 0, z, z, z, 1, [1, 1, 1, 1], short)   # W too small
        with pytest.raises(ValueError):
            ngc.ngc_worker_grads(ctx, 0, z, z, z, 1, [1, 1, 1], z)          # progress of the wrong length
        with pytest.raises(ValueError):
            ngc.ngc_partition_grads(ctx, 0, z, z.double(), z, 1, z)         # labels of the wrong type
        with pytest.raises(ValueError):
            ngc.ngc_partition_grads(ctx, 0, short, z, z, 1, z)              # X too small for k x rows x d
        with pytest.raises(ValueError):
            ngc.ngc_decode(ctx, 0, np.ones(3), z, z)                        # decode vector of the wrong length
        with pytest.raises(ngc.NgcError):
            ngc.ngc_worker_grads(ctx, 0, z, z, z, 1, [1, -1, 1, 1], z)
    finally:
        ngc.ngc_destroy(ctx)
