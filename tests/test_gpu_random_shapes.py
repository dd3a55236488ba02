"""Whole path on randomly drawn (seeded) configurations: number of workers, layer set, code
family, feature count (aligned, ragged, odd), rows per partition, loss.  Every step is
compared with the oracle, and the fused passes (whole iteration, encode + decode of one round,
of several rounds in one launch) with the stand-alone calls bit for bit."""
import numpy as np
import pytest

from oracle import coding, gradients
from paper_2212_08580_amd import workloads as wl

from test_gpu_parity import Pipeline, check_round, rel, torch_dev  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

FEATURES = [1, 3, 17, 64, 100, 255, 256, 300, 513, 1000, 1024, 1030, 2047, 2048, 3000, 3072, 4096, 5000, 7001]


def draw(rng):
    if rng.random() < 0.7:
        n = int(rng.integers(2, 25))
        smax = int(rng.integers(1, n))
        more = sorted(set(int(x) for x in rng.integers(1, smax + 1, size=int(rng.integers(1, 4)))))
        kind, layers = "cyclic", tuple([0] + more)
    else:
        n = int(rng.choice([4, 8, 12, 16, 24]))
        options = [(0, 1), (0, 1, 3), (0, 3)] + ([(0, 1, 3, 7)] if n % 8 == 0 else [])
        kind, layers = "fracrep", options[int(rng.integers(0, len(options)))]
    base = wl.C3 if rng.random() < 0.5 else wl.C2
    return kind, base.scaled(rows=int(rng.integers(1, 70)), d=int(rng.choice(FEATURES)), n=n, layers=layers,
                             name="random")


@pytest.mark.parametrize("seed", range(6))
def test_random_configurations(ngc, torch_dev, seed):
    torch = torch_dev
    rng = np.random.default_rng(1000 + seed)
    for it in range(10):
        kind, w = draw(rng)
        tag = (seed, it, kind, w.n, w.layers, w.d, w.rows, w.loss)
        X, Y = wl.dataset(w, seed=it, threads=1)
        th = wl.theta(w, seed=it + 1, scale=None if w.loss == wl.LOSS_LSQ else 2.0 / np.sqrt(w.d))
        p = Pipeline(ngc, torch, w, kind=kind, seed=it)
        try:
            G = p.grads(X, Y, th)
            G_o = gradients.partial_gradients(w.loss, X, Y, th)
            for j in range(w.n):
                assert rel(G[j], G_o[j]) <= 1e-4, tag
            C = p.encode()
            assert rel(C, coding.encode_layers(p.Bs, G_o)) <= 1e-4, tag
            for _ in range(3):
                m = np.zeros(w.n, np.uint8)
                m[rng.choice(w.n, size=int(rng.integers(0, w.layers[-1] + 1)), replace=False)] = 1
                check_round(p, G_o, m, C)
            # the fused iteration gives the bits of the stand-alone calls
            m = np.zeros(w.n, np.uint8)
            m[int(rng.integers(0, w.n))] = 1
            Xd, Yd, th1, th2 = p.to_dev(X), p.to_dev(Y), p.to_dev(th), p.to_dev(th)
            G2, C2, g2 = torch.empty_like(p.G), torch.empty_like(p.C), torch.empty_like(p.g)
            u, a = ngc.ngc_iteration(p.ctx, w.loss, Xd, Yd, th1, w.rows, m, 0.5 / w.m, G2, C2, g2, w.n)
            ngc.ngc_partition_grads(p.ctx, w.loss, Xd, Yd, th2, w.rows, p.G)
            ngc.ngc_encode(p.ctx, p.G, -1, p.C)
            ngc.ngc_decode(p.ctx, u, a, p.C, p.g)
            ngc.ngc_update(p.ctx, th2, p.g, 0.5 / w.m)
            ngc.ngc_sync(p.ctx)
            assert torch.equal(G2, p.G) and torch.equal(C2, p.C) and torch.equal(g2, p.g), tag
            assert torch.equal(th1, th2), tag
            # encode + decode of that round in one pass over G, and of several rounds in one launch
            # (some with one straggler too many): same bits as the stand-alone calls
            M1 = torch.full((w.n, w.d), -3.0, dtype=torch.float32, device=p.dev)
            g1 = torch.empty_like(p.g)
            ngc.ngc_encode_decode(p.ctx, p.G, u, a, M1, g1)
            ngc.ngc_sync(p.ctx)
            resp = torch.from_numpy(np.flatnonzero(a != 0)).to(p.dev)
            assert torch.equal(g1, p.g) and torch.equal(M1[resp], p.C[u][resp]), tag
            R = 7
            masks = np.zeros((R, w.n), np.uint8)
            for r in range(R):
                cnt = int(rng.integers(0, w.layers[-1] + 2))            # up to s_max + 1
                masks[r, rng.choice(w.n, size=min(cnt, w.n), replace=False)] = 1
            MR = torch.full((R, w.n, w.d), -3.0, dtype=torch.float32, device=p.dev)
            gR = torch.full((R, w.d), -3.0, dtype=torch.float32, device=p.dev)
            lay, aa = ngc.ngc_coded_rounds(p.ctx, p.G, 0, masks, MR, w.n * w.d, gR)
            ngc.ngc_sync(p.ctx)
            for r in range(R):
                if masks[r].sum() > w.layers[-1]:
                    assert lay[r] == -1 and bool((gR[r] == 0).all()) and bool((MR[r] == -3.0).all()), tag
                    continue
                u_o, a_o, g_o = coding.coded_gradient(p.Bs, w.layers, G_o, masks[r])
                assert lay[r] == u_o and np.array_equal(aa[r] != 0, a_o != 0), tag
                ngc.ngc_decode(p.ctx, int(lay[r]), aa[r], p.C, p.g)
                ngc.ngc_sync(p.ctx)
                resp = torch.from_numpy(np.flatnonzero(aa[r] != 0)).to(p.dev)
                assert torch.equal(gR[r], p.g) and torch.equal(MR[r][resp], p.C[int(lay[r])][resp]), tag
        finally:
            p.close()


@pytest.mark.parametrize("seed", range(4))
def test_random_short_rows(ngc, torch_dev, seed):
    """Partition gradients for rows of 1 to 255 features over row counts from one row to several
    blocks of several trips per partition (the kernels that pack several rows into a wave-wide
    load, or read a run of rows as one flat stretch): against the oracle, twice for the same bits."""
    rng = np.random.default_rng(2000 + seed)
    for it in range(25):
        d = int(rng.integers(1, 256))
        n = int(rng.integers(1, 7))
        rows = int(np.exp(rng.uniform(0.0, np.log(60000.0))))
        base = wl.C3 if rng.random() < 0.5 else wl.C2
        w = base.scaled(rows=rows, d=d, n=n, layers=(0,), name="short")
        tag = (seed, it, d, n, rows, w.loss)
        X, Y = wl.dataset(w, seed=it, threads=1)
        th = wl.theta(w, seed=it + 1, scale=None if w.loss == wl.LOSS_LSQ else 2.0 / np.sqrt(d))
        p = Pipeline(ngc, torch_dev, w, Bs=[np.eye(n)])
        try:
            G = p.grads(X, Y, th)
            G_o = gradients.partial_gradients(w.loss, X, Y, th)
            assert np.all(np.isfinite(G)), tag
            for j in range(n):
                assert rel(G[j], G_o[j]) <= 1e-4, (tag, j, rel(G[j], G_o[j]))
            assert np.array_equal(G, p.grads(X, Y, th)), tag
        finally:
            p.close()
