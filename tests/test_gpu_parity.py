"""Parity of the HIP path (through the C ABI) against the fp64 oracle.

Bars: rel-L2 <= 1e-4 for floating point; layer, straggler handling and the
support of the decode vector exact.  The decode kernel itself is held to 2e-7
against the fp64 combination of the messages it read.  Against the exact sum of
the partial gradients a decoded round may exceed 1e-4 only where the code itself
magnifies the fp32 rounding of the messages (kappa = sum |a_i| ||c_i|| / ||g||
large: a straggler count equal to the layer's tolerance leaves one decode vector
and no choice): such a round must stay inside the forward-error bound
4 * 2^-24 * kappa, the tests of the headline code (n = 32) assert plain 1e-4 on
every round of its own straggler distribution, the n = 64 stress test asserts
the share of rounds above 1e-4, and every figure goes to the report file
(conftest.parity_report).

Codes: by default the one the library builds (ngc_build_code, the configuration
the benchmark times), read back through ngc_get_code and handed to the oracle,
which first checks Def. 1 on sampled straggler sets; where a test names `kind`
with oracle=True the oracle's own constructor supplies B through ngc_set_code.
"""
import dataclasses

import numpy as np
import pytest

from oracle import codes, coding, gradients
from paper_2212_08580_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def torch_dev():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run on the MI355X box)")
    torch.cuda.set_device(0)
    return torch


def rel(x, ref):
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300))


def report(**kw):
    """One line per parity figure, kept beside the test log."""
    from conftest import parity_report
    parity_report(**kw)


def def1_holds_on_samples(Bs, layers, seed=0, sets=6):
    """Def. 1 in the oracle for a code that did not come from it: sampled straggler sets of the
    design size of every layer decode with residual <= 1e-9, supports nested, B_0 = I."""
    rng = np.random.default_rng(seed)
    n = Bs[0].shape[0]
    assert np.array_equal(Bs[0], np.eye(n))
    for u, sigma in enumerate(layers):
        if u:
            assert np.all((Bs[u - 1] != 0) <= (Bs[u] != 0))                   # Def. 2
        assert np.all(np.count_nonzero(Bs[u], axis=1) == sigma + 1)          # load (k/n)(sigma+1)
        for _ in range(sets):
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=sigma, replace=False)] = 1
            assert coding.decode_vector(Bs[u], m)[1] <= 1e-9


class Pipeline:
    """Device buffers + context for one workload.  The code is the library's own
    (ngc_build_code, seed 0) unless matrices or oracle=True are given."""

    def __init__(self, ngc, torch, w, Bs=None, kind=None, seed=0, oracle=False):
        self.ngc, self.torch, self.w = ngc, torch, w
        self.dev = torch.device("cuda:0")
        stream = torch.cuda.current_stream().cuda_stream
        self.ctx = ngc.ngc_create(w.n, w.n, w.layers, w.d, stream)
        kind = kind or ("cyclic" if w.code == wl.CODE_CYCLIC else "fracrep")
        if Bs is None and not oracle:
            ngc.ngc_build_code(self.ctx, ngc.NGC_CODE_CYCLIC if kind == "cyclic" else ngc.NGC_CODE_FRACREP, seed)
            Bs = [ngc.ngc_get_code(self.ctx, u) for u in range(len(w.layers))]
            def1_holds_on_samples(Bs, w.layers)
        else:
            if Bs is None:
                Bs = codes.nested_code(w.n, w.layers, kind, seed=seed, draws=2)
            for u, B in enumerate(Bs):
                ngc.ngc_set_code(self.ctx, u, B)
        self.Bs = Bs
        self.G = torch.empty((w.n, w.d), dtype=torch.float32, device=self.dev)
        self.C = torch.empty((len(w.layers), w.n, w.d), dtype=torch.float32, device=self.dev)
        self.g = torch.empty(w.d, dtype=torch.float32, device=self.dev)

    def close(self):
        self.ngc.ngc_destroy(self.ctx)

    def to_dev(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)

    def grads(self, X, Y, th):
        self.ngc.ngc_partition_grads(self.ctx, self.w.loss, self.to_dev(X), self.to_dev(Y),
                                     self.to_dev(th), X.shape[1], self.G)
        self.ngc.ngc_sync(self.ctx)
        return self.G.cpu().numpy()

    def encode(self, layer=-1):
        self.ngc.ngc_encode(self.ctx, self.G, layer, self.C)
        self.ngc.ngc_sync(self.ctx)
        return self.C.cpu().numpy()

    def decode(self, mask):
        u, a, r = self.ngc.ngc_select_decode_vec(self.ctx, mask, self.w.n)
        self.ngc.ngc_decode(self.ctx, u, a, self.C, self.g)
        self.ngc.ngc_sync(self.ctx)
        return u, a, r, self.g.cpu().numpy()


def check_round(p, G_o, mask, C_gpu, plain=False):
    """One mask: layer/support exact, decode kernel against the fp64 combination of its own
    input, decoded gradient against the oracle: within max(1e-4, 4 * 2^-24 * kappa), with
    `plain` within 1e-4 whatever kappa is."""
    w = p.w
    u_o, a_o, g_o = coding.coded_gradient(p.Bs, w.layers, G_o, mask)
    u, a, r, g = p.decode(mask)
    assert u == u_o
    assert np.array_equal(a != 0, a_o != 0)
    assert np.all(a[mask == 1] == 0)
    # the decode kernel itself: fp64 combination of the GPU's own fp32 messages
    g_same = coding.decode(a, C_gpu[u])
    assert rel(g, g_same) <= 2e-7
    err = rel(g, g_o)
    kappa = coding.conditioning(a_o, coding.encode(p.Bs[u_o], G_o), g_o)
    assert err <= (TOL if plain else max(TOL, 4 * 2.0 ** -24 * kappa)), (err, kappa)
    return err, kappa


# --------------------------------------------------------------------------------------------
# C1 exactly: least squares, n = 4, 4 x 256 rows, d = 64, layers (0,1), fractional repetition,
# all 16 straggler subsets
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("kind", ["fracrep", "cyclic"])
def test_c1_all_16_straggler_subsets(ngc, torch_dev, kind):
    w = wl.C1
    X, Y = wl.dataset(w, 0, threads=1)
    th = wl.theta(w, 0)
    p = Pipeline(ngc, torch_dev, w, kind=kind)
    try:
        G = p.grads(X, Y, th)
        G_o = gradients.partial_gradients(w.loss, X, Y, th)
        assert rel(G, G_o) <= TOL
        for j in range(w.n):
            assert rel(G[j], G_o[j]) <= TOL
        C = p.encode()
        C_o = coding.encode_layers(p.Bs, G_o)
        assert rel(C, C_o) <= TOL
        ok = bad = 0
        for bits in range(16):
            m = np.array([(bits >> i) & 1 for i in range(4)], np.uint8)
            if m.sum() > 1:
                with pytest.raises(ngc.NgcError) as e:
                    ngc.ngc_select_decode_vec(p.ctx, m, 4)
                assert e.value.code == ngc.NGC_ERR_UNDECODABLE
                bad += 1
                continue
            check_round(p, G_o, m, C)
            ok += 1
        assert (ok, bad) == (5, 11)
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# gradient kernels: every single-pass shape, the two-pass route, ragged row counts, both losses
# --------------------------------------------------------------------------------------------
GRAD_SHAPES = [
    # (d, n, rows)   rows chosen to leave ragged tails (not multiples of the row group)
    (256, 3, 37), (512, 3, 21), (768, 2, 9), (1024, 4, 131), (2048, 3, 29), (3072, 2, 11),
    (4096, 4, 67), (6144, 2, 7), (8192, 2, 13), (12288, 2, 5), (16384, 2, 6),
    (64, 4, 256), (200, 3, 50), (77, 2, 19), (1000, 2, 33), (4100, 2, 10), (5120, 2, 9),
    (4096, 2, 1), (1024, 1, 3), (4096, 64, 9),
    # rows shorter than the block's slots (d a multiple of 4) and rows that are not 16-byte
    # aligned (d not a multiple of 4), one case per kernel shape family
    (3000, 2, 11), (7000, 2, 6), (13000, 2, 4), (54, 3, 100), (1002, 3, 40), (2050, 2, 17),
    (4094, 2, 9), (5002, 2, 7), (8190, 2, 5), (30, 2, 70), (123, 2, 41), (130, 3, 35), (191, 2, 18), (250, 2, 9),
    # wide rows, 16388 to 32768 features in float4: theta in LDS, ten to sixteen waves per block
    (20000, 2, 3), (16388, 2, 2), (24580, 2, 4), (28672, 1, 7), (32768, 2, 5), (32768, 3, 1),
    # rows of 8193 to 16384 features that are no multiple of 4: sixteen waves of sixteen floats per lane and row
    (8194, 2, 3), (12001, 2, 5), (16383, 3, 4), (9999, 1, 33),
    # no single-pass shape: the two-pass route
    (32772, 2, 2), (40000, 2, 3), (20002, 1, 4),
    (1, 3, 40), (2, 2, 17), (5, 2, 33), (4, 2, 64), (16384, 1, 40),
    # narrow rows of 1, 2, 4, .. 32 float4 (several rows per wave-wide load), with and without a
    # ragged last group, and enough rows for several groups per block
    (8, 3, 1000), (16, 2, 33), (32, 2, 50), (128, 3, 77), (64, 2, 5000), (128, 2, 3001), (4, 1, 70000),
    (64, 64, 3),
    # short rows whose float4 count is no power of two, or that are no multiple of 4 at all
    (12, 3, 1000), (20, 2, 333), (24, 2, 70), (40, 3, 129), (48, 2, 50), (68, 2, 40), (96, 2, 77), (100, 2, 64),
    (124, 2, 33), (3, 2, 500), (6, 2, 100), (10, 3, 64), (17, 2, 90), (31, 2, 50), (21, 1, 4000),
    # short rows read as one flat stretch of float4 and sorted into rows in LDS (here d < 64, no multiple of 4):
    # every register-width variant, partitions that start inside a 16-byte granule, X ending inside one (its
    # last rows are then added from single loads), several trips per block, several blocks per partition, a lone row
    (7, 3, 1001), (13, 2, 333), (23, 3, 71), (29, 2, 4097), (33, 2, 515), (39, 1, 77), (47, 3, 301), (55, 2, 129),
    (63, 3, 1001), (57, 1, 5), (63, 2, 20000), (3, 1, 70001), (1, 1, 3), (2, 1, 1), (1, 5, 1), (9, 1, 1), (61, 1, 1),
    (1, 17, 54), (1, 7, 1), (1, 2, 3), (1, 3, 513), (2, 3, 171), (3, 5, 1),   # several rows in X's last granule
    # rows of 65 to 248 features that are no multiple of 4: the same kernel with four or eight lanes to a row
    (65, 3, 1000), (91, 2, 300), (93, 2, 129), (125, 2, 77), (185, 1, 50), (247, 3, 333), (249, 2, 20), (101, 1, 1),
    (67, 5, 3), (199, 2, 5000), (127, 1, 9000), (72, 2, 130), (88, 3, 33), (112, 1, 400), (132, 2, 65),
    # the multiples of four that take the same kernel
    (20, 3, 777), (28, 2, 130), (48, 3, 4099), (48, 1, 63), (36, 2, 65), (44, 1, 300), (52, 2, 64), (56, 3, 100), (60, 2, 4100),
]


@pytest.mark.parametrize("loss", [wl.LOSS_LSQ, wl.LOSS_LOGISTIC])
@pytest.mark.parametrize("d,n,rows", GRAD_SHAPES)
def test_partition_gradients_match_oracle(ngc, torch_dev, loss, d, n, rows):
    base = wl.C3 if loss == wl.LOSS_LSQ else wl.C2
    w = base.scaled(rows=rows, d=d, n=n, layers=(0,), name="shape")
    X, Y = wl.dataset(w, seed=d + rows, threads=1)
    scale = None if loss == wl.LOSS_LSQ else 2.0 / np.sqrt(d)   # margins of order 1, not saturated
    th = wl.theta(w, seed=1, scale=scale)
    p = Pipeline(ngc, torch_dev, w, Bs=[np.eye(n)])
    try:
        G = p.grads(X, Y, th)
        G_o = gradients.partial_gradients(loss, X, Y, th)
        assert G.shape == G_o.shape
        assert np.all(np.isfinite(G))
        for j in range(n):
            assert rel(G[j], G_o[j]) <= TOL, (j, rel(G[j], G_o[j]))
        G2 = p.grads(X, Y, th)
        assert np.array_equal(G, G2)              # fixed summation order: bit-reproducible
    finally:
        p.close()


def test_logistic_saturated_margins(ngc, torch_dev):
    """exp overflow in the logistic slope must give the limits 0 and -y, not NaN."""
    w = wl.C2.scaled(rows=64, d=1024, n=2, layers=(0,))
    X, Y = wl.dataset(w, seed=3, threads=1)
    th = wl.theta(w, seed=1, scale=50.0)           # |x.theta| ~ 1600 >> 88
    p = Pipeline(ngc, torch_dev, w, Bs=[np.eye(2)])
    try:
        G = p.grads(X, Y, th)
        G_o = gradients.partial_gradients(w.loss, X, Y, th)
        assert np.all(np.isfinite(G))
        assert rel(G, G_o) <= TOL
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# encode / decode on their own (no data): vector widths 4, 2, 1, column tails, both families
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("from_oracle", [False, True])
@pytest.mark.parametrize("n,layers,kind,d", [
    (4, (0, 1), "fracrep", 64), (16, (0, 1, 3, 7), "cyclic", 1024), (32, (0, 1, 3, 7, 15), "cyclic", 4096),
    (64, (0, 1, 3, 7, 15, 31), "cyclic", 16384), (64, (0, 1, 3, 7, 15, 31), "fracrep", 4096),
    (20, (0, 1, 4, 9), "cyclic", 1002), (20, (0, 1, 4, 9), "cyclic", 999), (7, (0, 2, 5), "cyclic", 100),
    (1, (0,), "cyclic", 5), (33, (0, 32), "cyclic", 68),
])
def test_encode_and_decode_match_oracle(ngc, torch_dev, n, layers, kind, d, from_oracle):
    """Both directions: the library's code handed to the oracle, and the oracle's constructor's
    code installed in the library."""
    w = wl.C5.scaled(n=n, d=d, layers=layers)
    G_h = wl.partial_gradients(w, seed=n + d)
    p = Pipeline(ngc, torch_dev, w, kind=kind, oracle=from_oracle)
    try:
        p.G.copy_(torch_dev.from_numpy(G_h))
        C = p.encode()
        C_o = coding.encode_layers(p.Bs, G_h)
        for u in range(len(layers)):
            assert rel(C[u], C_o[u]) <= 1e-6, (u, rel(C[u], C_o[u]))
        assert np.array_equal(C[0], G_h)                       # B_0 = I: layer 0 is a copy
        # one layer at a time writes only its slice
        p.C.fill_(-7.0)
        last = len(layers) - 1
        C1 = p.encode(layer=last)
        assert np.array_equal(C1[last], C[last])
        if last > 0:
            assert np.all(C1[:last] == -7.0)
        p.encode()
        rng = np.random.default_rng(5)
        worst = 0.0
        for t in range(12):
            s = int(rng.integers(0, layers[-1] + 1))
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=s, replace=False)] = 1
            err, kappa = check_round(p, G_h.astype(np.float64), m, C)
            worst = max(worst, err)
        report(test="encode_and_decode", n=n, d=d, kind=kind, worst_decode_rel_l2=worst)
    finally:
        p.close()


def test_decode_rejects_bad_arguments_and_update_matches(ngc, torch_dev):
    w = wl.C5.scaled(n=4, d=1030, layers=(0, 1))
    p = Pipeline(ngc, torch_dev, w)
    try:
        a = np.ones(4)
        with pytest.raises(ngc.NgcError):
            ngc.ngc_decode(p.ctx, 2, a, p.C, p.g)
        a[1] = np.inf
        with pytest.raises(ngc.NgcError):
            ngc.ngc_decode(p.ctx, 0, a, p.C, p.g)
        with pytest.raises(ngc.NgcError):
            ngc.ngc_encode(p.ctx, p.G, 5, p.C)
        th = np.random.default_rng(0).standard_normal(w.d).astype(np.float32)
        gg = np.random.default_rng(1).standard_normal(w.d).astype(np.float32)
        thd, gd = p.to_dev(th), p.to_dev(gg)
        ngc.ngc_update(p.ctx, thd, gd, 0.25)
        ngc.ngc_sync(p.ctx)
        assert rel(thd.cpu().numpy(), gradients.gd_update(th, gg, 0.25, 1.0)) <= 1e-6
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# closed forms at theta = 0, straight from the data (no oracle function in between):
# least squares g_j = -X_j^T y_j, logistic g_j = -(1/2) sum_i y_i x_i
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("base,d,rows", [(wl.C3, 4096, 300), (wl.C2, 1024, 700), (wl.C3, 1002, 90),
                                         (wl.C2, 5000, 64)])
def test_gradients_at_zero_are_the_closed_forms(ngc, torch_dev, base, d, rows):
    w = base.scaled(rows=rows, d=d, n=4, layers=(0,), name="zero")
    X, Y = wl.dataset(w, seed=9, threads=1)
    p = Pipeline(ngc, torch_dev, w, Bs=[np.eye(w.n)])
    try:
        G = p.grads(X, Y, np.zeros(d, np.float32))
        for j in range(w.n):
            xty = X[j].astype(np.float64).T @ Y[j].astype(np.float64)
            want = -xty if w.loss == wl.LOSS_LSQ else -0.5 * xty
            assert rel(G[j], want) <= 1e-5, (j, rel(G[j], want))
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# C1 as a whole: coded gradient descent on the GPU, a straggler in most iterations, ends at the
# least-squares solution that a library routine gives (a textbook endpoint, no oracle step in it)
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("kind", ["fracrep", "cyclic"])
def test_c1_descent_reaches_the_least_squares_solution(ngc, torch_dev, kind):
    w = wl.C1
    X, Y = wl.dataset(w, 0, threads=1)
    Xa, ya = X.reshape(-1, w.d).astype(np.float64), Y.reshape(-1).astype(np.float64)
    th_ls = np.linalg.lstsq(Xa, ya, rcond=None)[0]
    p = Pipeline(ngc, torch_dev, w, kind=kind)
    try:
        Xd, Yd, thd = p.to_dev(X), p.to_dev(Y), p.to_dev(wl.theta(w, 0))
        rng = np.random.default_rng(4)
        layers_used = set()
        for t in range(120):
            m = np.zeros(w.n, np.uint8)
            if rng.random() < 0.7:
                m[rng.integers(0, w.n)] = 1                       # one straggler: still decodable
            u, a = ngc.ngc_iteration(p.ctx, w.loss, Xd, Yd, thd, w.rows, m, 1.0 / w.m, p.G, p.C, p.g, w.n)
            layers_used.add(u)
        ngc.ngc_sync(p.ctx)
        assert layers_used == {0, 1}
        assert rel(thd.cpu().numpy(), th_ls) <= 2e-5              # fp32 iterates, fp32 data
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# C2 shrunk (logistic, n = 16, layers 0,1,3,7, Bernoulli(0.2) stragglers): a short descent run,
# each iteration checked against the oracle evaluated at the GPU's own theta_t, and the whole
# trajectory against the oracle's own run from the same start
# --------------------------------------------------------------------------------------------
def test_c2_scaled_descent_with_stragglers(ngc, torch_dev):
    w = wl.C2.scaled(rows=515, name="C2-rows515")              # d = 1024, 16 partitions
    X, Y = wl.dataset(w, 0, threads=4)
    th0 = wl.theta(w, 0, scale=0.01)
    masks = wl.bernoulli_masks(w, 12, seed=0)
    p = Pipeline(ngc, torch_dev, w)
    try:
        Xd, Yd, thd = p.to_dev(X), p.to_dev(Y), p.to_dev(th0)
        eta, used, skipped = 1.0, set(), 0
        th_free = th0.astype(np.float64)                      # the oracle's own run, no GPU number in it
        for t in range(12):
            th_t = thd.cpu().numpy()
            assert rel(th_t, th_free) <= 1e-5
            try:
                _, _, g_free = coding.coded_gradient(p.Bs, w.layers,
                                                     gradients.partial_gradients(w.loss, X, Y, th_free), masks[t])
                th_free = gradients.gd_update(th_free, g_free, eta, w.m)
            except coding.Undecodable:
                pass
            ngc.ngc_partition_grads(p.ctx, w.loss, Xd, Yd, thd, w.rows, p.G)
            ngc.ngc_encode(p.ctx, p.G, -1, p.C)
            try:
                u, a, r = ngc.ngc_select_decode_vec(p.ctx, masks[t], w.n)
            except ngc.NgcError as e:
                assert e.code == ngc.NGC_ERR_UNDECODABLE      # theta stays as it is this round
                skipped += 1
                continue
            ngc.ngc_decode(p.ctx, u, a, p.C, p.g)
            ngc.ngc_update(p.ctx, thd, p.g, eta / w.m)
            ngc.ngc_sync(p.ctx)
            G_o = gradients.partial_gradients(w.loss, X, Y, th_t)
            u_o, a_o, g_o = coding.coded_gradient(p.Bs, w.layers, G_o, masks[t])
            assert u == u_o and np.array_equal(a != 0, a_o != 0)
            assert rel(p.G.cpu().numpy(), G_o) <= TOL
            assert rel(p.g.cpu().numpy(), g_o) <= TOL
            assert rel(thd.cpu().numpy(), gradients.gd_update(th_t, g_o, eta, w.m)) <= 1e-6
            used.add(u)
        assert rel(thd.cpu().numpy(), th_free) <= 1e-5
        assert len(used) >= 2 and skipped <= 2
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# C3 shrunk in rows only (n = 32, d = 4096, layers 0,1,3,7,15, Bernoulli(0.1) stragglers)
# --------------------------------------------------------------------------------------------
def test_c3_scaled_pipeline(ngc, torch_dev):
    w = wl.C3.scaled(rows=203, name="C3-rows203")
    X, Y = wl.dataset(w, 0, threads=4)
    th = wl.theta(w, 0)
    p = Pipeline(ngc, torch_dev, w)
    try:
        G = p.grads(X, Y, th)
        G_o = gradients.partial_gradients(w.loss, X, Y, th)
        for j in range(w.n):
            assert rel(G[j], G_o[j]) <= TOL
        C = p.encode()
        assert rel(C, coding.encode_layers(p.Bs, G_o)) <= TOL
        masks = wl.bernoulli_masks(w, 200, seed=1)
        errs = [check_round(p, G_o, m, C, plain=True)[0] for m in masks if m.sum() <= w.layers[-1]]
        assert len(errs) >= 195
        report(test="c3_scaled_pipeline", rounds=len(errs), worst_decode_rel_l2=max(errs),
               median_decode_rel_l2=float(np.median(errs)))
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# C5: encode/decode stress, n = 64, d = 16384, layers (0,1,3,7,15,31), straggler count
# Binomial(64, 0.2), decode vector solved per round, all 1000 rounds
# --------------------------------------------------------------------------------------------
def test_c5_rounds(ngc, torch_dev):
    w = wl.C5
    G_h = wl.partial_gradients(w, 0)
    masks = wl.binomial_count_masks(w, 1000, seed=0)
    p = Pipeline(ngc, torch_dev, w)
    try:
        p.G.copy_(torch_dev.from_numpy(G_h))
        C = p.encode()
        assert rel(C, coding.encode_layers(p.Bs, G_h)) <= 1e-6
        G64 = G_h.astype(np.float64)
        errs = []
        for m in masks:
            if m.sum() > w.layers[-1]:
                with pytest.raises(ngc.NgcError):
                    ngc.ngc_select_decode_vec(p.ctx, m, w.n)
                continue
            errs.append(check_round(p, G64, m, C)[0])
        errs = np.array(errs)
        report(test="c5_rounds", rounds=int(errs.size), median_decode_rel_l2=float(np.median(errs)),
               worst_decode_rel_l2=float(errs.max()), share_above_1e_4=float(np.mean(errs > TOL)))
        # a straggler count equal to a layer's tolerance leaves one decode vector; for a random
        # real-valued code of this size a few per thousand of such sets magnify fp32 message
        # rounding beyond 1e-4 (each of them inside the forward-error bound, checked above)
        assert np.mean(errs > TOL) <= 0.01
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# Full headline size (C3: 32 x 16384 x 4096, 8.6 GB) in the launch configuration the benchmark
# times: every partition's gradient against the oracle, element by element (the oracle needs
# a few seconds for all of X), messages and decoding on top of the GPU's own G.
# --------------------------------------------------------------------------------------------
def test_c3_full_size_every_partition(ngc, torch_dev):
    torch = torch_dev
    w = wl.C3
    dev = torch.device("cuda:0")
    truth = wl.truth_vector(w, 0)
    th = wl.theta(w, 0)
    Xd = torch.empty((w.n, w.rows, w.d), dtype=torch.float32, device=dev)
    Yd = torch.empty((w.n, w.rows), dtype=torch.float32, device=dev)
    sampled = {j: None for j in range(w.n)}
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=8) as ex:
        for j, (X, Y) in enumerate(ex.map(lambda j: wl.partition(w, j, 0, truth), range(w.n))):
            Xd[j].copy_(torch.from_numpy(X))
            Yd[j].copy_(torch.from_numpy(Y))
            if j in sampled:
                sampled[j] = gradients.lsq_gradient(X, Y, th)
    p = Pipeline(ngc, torch, w)
    try:
        ngc.ngc_partition_grads(p.ctx, w.loss, Xd, Yd, p.to_dev(th), w.rows, p.G)
        ngc.ngc_sync(p.ctx)
        G = p.G.cpu().numpy()
        for j, g_o in sampled.items():
            assert rel(G[j], g_o) <= TOL, (j, rel(G[j], g_o))
        assert np.all(np.isfinite(G))
        C = p.encode()
        # messages and decoding against the oracle's own gradients (exact recovery: decode == sum_j g_j)
        G_o = np.stack([sampled[j] for j in range(w.n)])
        C_o = coding.encode_layers(p.Bs, G_o)
        assert rel(C, C_o) <= TOL
        full = G_o.sum(axis=0)
        masks = wl.bernoulli_masks(w, 60, seed=2)
        worst = 0.0
        for m in masks:
            if m.sum() <= w.layers[-1]:
                u, a, r, g = p.decode(m)
                u_o, a_o, g_o = coding.coded_gradient(p.Bs, w.layers, G_o, m)
                assert u == u_o and np.array_equal(a != 0, a_o != 0)
                worst = max(worst, rel(g, full))
                assert rel(g, full) <= TOL
        report(test="c3_full_size", rounds=len(masks), worst_decode_rel_l2=worst)
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# per-kernel timing: what the benchmark's roofline figures are read from
# --------------------------------------------------------------------------------------------
def test_profile_records_every_launch_of_the_selected_kernels(ngc, torch_dev):
    w = wl.C3.scaled(rows=64, d=1024, n=4, layers=(0, 1), name="prof")
    X, Y = wl.dataset(w, seed=0, threads=1)
    th = wl.theta(w, seed=1)
    p = Pipeline(ngc, torch_dev, w)
    try:
        Xd, Yd, thd = p.to_dev(X), p.to_dev(Y), p.to_dev(th)
        ngc.ngc_profile_enable(p.ctx, ["grad", "encode"])
        for _ in range(5):
            ngc.ngc_partition_grads(p.ctx, w.loss, Xd, Yd, thd, w.rows, p.G)
            ngc.ngc_encode(p.ctx, p.G, -1, p.C)
            ngc.ngc_update(p.ctx, thd, p.g, 0.0)                      # not selected: not recorded
        each = ngc.ngc_profile_launches(p.ctx, "grad")
        assert each.size == 5 and np.all(each > 0.0) and np.all(each < 50.0)
        assert ngc.ngc_profile_launches(p.ctx, "update").size == 0
        prof = ngc.ngc_profile_read(p.ctx)
        assert prof["grad"][0] == 5 and prof["encode"][0] == 5 and prof["update"][0] == 0
        assert abs(prof["grad"][1] - each.sum()) <= 1e-6 * each.sum()
        assert ngc.ngc_profile_launches(p.ctx, "grad").size == 0       # the read cleared the record
        ngc.ngc_profile_enable(p.ctx, False)
        ngc.ngc_partition_grads(p.ctx, w.loss, Xd, Yd, thd, w.rows, p.G)
        assert ngc.ngc_profile_read(p.ctx)["grad"][0] == 0
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# More than 2^32 matrix elements (17 GB of X): element offsets no longer fit 32 bits, neither
# signed nor unsigned.  Both regression losses on the same features; the oracle adds up row
# chunks of every partition (the gradient is a sum over rows).
# --------------------------------------------------------------------------------------------
def test_gradients_beyond_2_to_32_elements(ngc, torch_dev):
    torch = torch_dev
    w = dataclasses.replace(wl.C3, name="huge-lsq", n=4, rows=266240, layers=(0, 1))
    assert w.n * w.rows * w.d > 2 ** 32
    dev = torch.device("cuda:0")
    truth = wl.truth_vector(w, 0)
    th = wl.theta(w, 0)
    th_log = (0.02 * th).astype(np.float32)      # margins of order one for the logistic loss
    Xd = torch.empty((w.n, w.rows, w.d), dtype=torch.float32, device=dev)
    Yd = torch.empty((w.n, w.rows), dtype=torch.float32, device=dev)
    Ys = torch.empty((w.n, w.rows), dtype=torch.float32, device=dev)
    G_lsq = np.zeros((w.n, w.d))
    G_log = np.zeros((w.n, w.d))

    def one(j):
        X, Y = wl.partition(w, j, 0, truth)
        S = np.where(Y >= 0.0, 1.0, -1.0).astype(np.float32)
        for r0 in range(0, w.rows, 65536):
            sl = slice(r0, min(w.rows, r0 + 65536))
            G_lsq[j] += gradients.lsq_gradient(X[sl], Y[sl], th)
            G_log[j] += gradients.logistic_gradient(X[sl], S[sl], th_log)
        return X, Y, S

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=4) as ex:
        for j, (X, Y, S) in enumerate(ex.map(one, range(w.n))):
            Xd[j].copy_(torch.from_numpy(X))
            Yd[j].copy_(torch.from_numpy(Y))
            Ys[j].copy_(torch.from_numpy(S))
    p = Pipeline(ngc, torch, w)
    try:
        ngc.ngc_partition_grads(p.ctx, wl.LOSS_LSQ, Xd, Yd, p.to_dev(th), w.rows, p.G)
        ngc.ngc_sync(p.ctx)
        G = p.G.cpu().numpy()
        for j in range(w.n):
            assert rel(G[j], G_lsq[j]) <= TOL, (j, rel(G[j], G_lsq[j]))
        ngc.ngc_partition_grads(p.ctx, wl.LOSS_LOGISTIC, Xd, Ys, p.to_dev(th_log), w.rows, p.G)
        ngc.ngc_sync(p.ctx)
        G = p.G.cpu().numpy()
        for j in range(w.n):
            assert rel(G[j], G_log[j]) <= TOL, (j, rel(G[j], G_log[j]))
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# decode through the explicit decoding matrix A_sigma held on the device (small codes)
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,layers,kind,d", [(8, (0, 1, 3), "cyclic", 4096), (12, (0, 2, 5), "cyclic", 1002),
                                             (8, (0, 1, 3, 7), "fracrep", 77),
                                             # long gradients: ngc_decode takes its one-thread-per-column
                                             # kernel (float4, float2 and float columns), which must give the
                                             # bits of the lookup kernel's group-wise combination
                                             (6, (0, 2), "cyclic", 524292), (6, (0, 2), "cyclic", 262146),
                                             (5, (0, 1), "cyclic", 131073)])
def test_decode_lookup_matches_oracle_and_solve_route(ngc, torch_dev, n, layers, kind, d):
    w = wl.C5.scaled(n=n, d=d, layers=layers)
    G_h = wl.partial_gradients(w, seed=3)
    p = Pipeline(ngc, torch_dev, w, kind=kind)
    try:
        for u in range(len(layers)):
            ngc.ngc_build_decoding_table(p.ctx, u)
        p.G.copy_(torch_dev.from_numpy(G_h))
        C = p.encode()
        full = G_h.astype(np.float64).sum(axis=0)
        rng = np.random.default_rng(1)
        g2 = torch_dev.empty_like(p.g)
        for t in range(20):
            u = int(rng.integers(0, len(layers)))
            s = int(rng.integers(0, layers[u] + 1))
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=s, replace=False)] = 1
            ngc.ngc_decode_lookup(p.ctx, u, m, p.C, p.g)
            a_o, _ = coding.decode_vector_first(p.Bs[u], layers[u], m)
            row = ngc.ngc_decoding_row_index(p.ctx, u, m)
            a = ngc.ngc_get_decoding_row(p.ctx, u, row, n)
            assert np.array_equal(a != 0, a_o != 0)
            ngc.ngc_decode(p.ctx, u, a, p.C, g2)                  # same vector through the kernel arguments
            ngc.ngc_sync(p.ctx)
            assert np.array_equal(p.g.cpu().numpy(), g2.cpu().numpy())
            g = p.g.cpu().numpy()
            assert rel(g, coding.decode(a_o, C[u])) <= 1e-6
            kappa = coding.conditioning(a_o, coding.encode(p.Bs[u], G_h), full)
            assert rel(g, full) <= max(TOL, 4 * 2.0 ** -24 * kappa)
        m = np.ones(n, np.uint8)
        with pytest.raises(ngc.NgcError):
            ngc.ngc_decode_lookup(p.ctx, 1, m, p.C, p.g)
    finally:
        p.close()


# --------------------------------------------------------------------------------------------
# k = c*n partitions: an atomic task is k/n partial gradients (Sec. II-C); zero-padded rows
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,c,layers,kind,d,rows", [(8, 2, (0, 1, 3), "cyclic", 1024, 45),
                                                     (4, 4, (0, 1), "fracrep", 4096, 19),
                                                     (6, 3, (0, 2), "cyclic", 200, 12)])
def test_several_partitions_per_worker(ngc, torch_dev, n, c, layers, kind, d, rows):
    from oracle import workers as ow
    torch = torch_dev
    dev = torch.device("cuda:0")
    k = n * c
    w = wl.C3.scaled(rows=rows, d=d, n=k, layers=layers)             # k data partitions
    X, Y = wl.dataset(w, seed=5, threads=1)
    X[-1, rows - 3:] = 0.0                                           # last partition zero-padded
    Y[-1, rows - 3:] = 0.0
    th = wl.theta(w, seed=6)
    Bs = codes.expand_partitions(codes.nested_code(n, layers, kind, seed=0, draws=2), c)
    G_o = gradients.partial_gradients(w.loss, X, Y, th)
    assert np.allclose(G_o[-1], gradients.lsq_gradient(X[-1, :rows - 3], Y[-1, :rows - 3], th))
    full = G_o.sum(axis=0)
    ctx = ngc.ngc_create(n, k, layers, d, torch.cuda.current_stream().cuda_stream)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        Xd, Yd, thd = (torch.from_numpy(a).to(dev) for a in (X, Y, th))
        G = torch.empty((k, d), dtype=torch.float32, device=dev)
        C = torch.empty((len(layers), n, d), dtype=torch.float32, device=dev)
        g = torch.empty(d, dtype=torch.float32, device=dev)
        ngc.ngc_partition_grads(ctx, w.loss, Xd, Yd, thd, rows, G)
        ngc.ngc_encode(ctx, G, -1, C)
        ngc.ngc_sync(ctx)
        for j in range(k):
            assert rel(G[j].cpu().numpy(), G_o[j]) <= TOL
        Ch = C.cpu().numpy()
        for u in range(len(layers)):
            assert rel(Ch[u], coding.encode(Bs[u], G_o)) <= TOL
        rng = np.random.default_rng(2)
        for t in range(10):
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=int(rng.integers(0, layers[-1] + 1)), replace=False)] = 1
            u, a, r = ngc.ngc_select_decode_vec(ctx, m, n)
            a_o, _ = coding.decode_vector(Bs[u], m)
            assert u == coding.select_layer(layers, m) and np.array_equal(a != 0, a_o != 0)
            ngc.ngc_decode(ctx, u, a, C, g)
            ngc.ngc_sync(ctx)
            kappa = coding.conditioning(a_o, coding.encode(Bs[u], G_o), full)
            assert rel(g.cpu().numpy(), full) <= max(TOL, 4 * 2.0 ** -24 * kappa)
        # redundancy-faithful mode: a task is c partitions
        T = ngc.ngc_worker_task_count(ctx)
        assert T == layers[-1] + 1
        progress = np.array([T] * (n - 1) + [0])
        W = torch.full((n, T * c, d), 7.0, dtype=torch.float32, device=dev)
        ngc.ngc_worker_grads(ctx, w.loss, Xd, Yd, thd, rows, progress, W)
        ngc.ngc_worker_encode(ctx, W, progress, C)
        u, mask, a, r = ngc.ngc_select_from_progress(ctx, progress, n)
        ngc.ngc_decode(ctx, u, a, C, g)
        ngc.ngc_sync(ctx)
        W_o = ow.worker_partials(w.loss, X, Y, th, Bs, progress)
        u_o, mask_o, a_o, g_o = ow.decode_from_workers(Bs, layers, W_o, progress)
        assert u == u_o and np.array_equal(mask, mask_o)
        Wh = W.cpu().numpy()
        for i in range(n - 1):
            for t in range(T * c):
                assert rel(Wh[i, t], W_o[i][t]) <= TOL
        assert np.all(Wh[n - 1] == 7.0)
        C_o = ow.worker_messages(Bs, W_o, progress)
        for i in range(n - 1):
            assert rel(C[u, i].cpu().numpy(), C_o[u][i]) <= TOL
        assert rel(g.cpu().numpy(), full) <= TOL
    finally:
        ngc.ngc_destroy(ctx)


# --------------------------------------------------------------------------------------------
# ngc_iteration: the whole iteration in two launches, same bits as the stand-alone calls
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("base,n,c,rows,d,layers", [
    (wl.C3, 32, 1, 70, 4096, (0, 1, 3, 7, 15)), (wl.C2, 16, 1, 130, 1024, (0, 1, 3, 7)),
    (wl.C3, 6, 1, 33, 200, (0, 1, 3)), (wl.C2, 5, 1, 21, 77, (0, 2)), (wl.C3, 4, 2, 25, 512, (0, 1)),
    (wl.C3, 64, 1, 5, 16384, (0, 1, 3, 7, 15, 31)),
    (wl.C2, 6, 1, 19, 1002, (0, 2)), (wl.C3, 4, 1, 9, 5000, (0, 1)), (wl.C3, 3, 1, 4, 20000, (0, 1)),
    # the paper's own layer set, every sigma = 0..s_max (Def. 2); the last one's code tables
    # (33 792 non-zeros) do not fit the LDS of a block and stay in global memory
    (wl.C3, 16, 1, 7, 256, tuple(range(8))), (wl.C2, 32, 1, 5, 128, tuple(range(16))),
    (wl.C3, 64, 1, 3, 64, tuple(range(32))),
])
def test_fused_iteration_equals_separate_calls(ngc, torch_dev, base, n, c, rows, d, layers):
    torch = torch_dev
    dev = torch.device("cuda:0")
    k = n * c
    w = base.scaled(rows=rows, d=d, n=k, layers=layers)
    X, Y = wl.dataset(w, seed=9, threads=2)
    scale = None if w.loss == wl.LOSS_LSQ else 2.0 / np.sqrt(d)
    th = wl.theta(w, seed=4, scale=scale)
    Bs = codes.expand_partitions(codes.nested_code(n, layers, "cyclic", seed=0, draws=2), c)
    ctx = ngc.ngc_create(n, k, layers, d, torch.cuda.current_stream().cuda_stream)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        Xd, Yd = torch.from_numpy(X).to(dev), torch.from_numpy(Y).to(dev)
        L = len(layers)
        bufs = [[torch.empty((k, d), dtype=torch.float32, device=dev),
                 torch.empty((L, n, d), dtype=torch.float32, device=dev),
                 torch.empty(d, dtype=torch.float32, device=dev),
                 torch.from_numpy(th.copy()).to(dev)] for _ in range(2)]
        rng = np.random.default_rng(0)
        eta = 0.3 / w.m
        for t in range(4):
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=int(rng.integers(0, layers[-1] + 1)), replace=False)] = 1
            G0, C0, g0, th0 = bufs[0]
            ngc.ngc_partition_grads(ctx, w.loss, Xd, Yd, th0, rows, G0)
            ngc.ngc_encode(ctx, G0, -1, C0)
            u0, a0, _ = ngc.ngc_select_decode_vec(ctx, m, n)
            ngc.ngc_decode(ctx, u0, a0, C0, g0)
            ngc.ngc_update(ctx, th0, g0, eta)
            G1, C1, g1, th1 = bufs[1]
            u1, a1 = ngc.ngc_iteration(ctx, w.loss, Xd, Yd, th1, rows, m, eta, G1, C1, g1, n)
            ngc.ngc_sync(ctx)
            assert u0 == u1 and np.array_equal(a0, a1)
            assert torch.equal(G0, G1) and torch.equal(C0, C1) and torch.equal(g0, g1)
            assert torch.equal(th0, th1)
        # and against the oracle for the last round's gradient at the last theta before the update
        # (theta after t rounds is the same on both routes, so check the fused outputs directly)
        m = np.zeros(n, np.uint8)
        th_now = bufs[1][3].cpu().numpy()
        u1, a1 = ngc.ngc_iteration(ctx, w.loss, Xd, Yd, bufs[1][3], rows, m, 0.0, *bufs[1][:3], n)
        ngc.ngc_sync(ctx)
        G_o = gradients.partial_gradients(w.loss, X, Y, th_now)
        assert u1 == 0 and rel(bufs[1][0].cpu().numpy(), G_o) <= TOL
        assert rel(bufs[1][2].cpu().numpy(), G_o.sum(axis=0)) <= TOL
        bad = np.ones(n, np.uint8)
        before = bufs[1][3].clone()
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_iteration(ctx, w.loss, Xd, Yd, bufs[1][3], rows, bad, eta, *bufs[1][:3], n)
        assert e.value.code == ngc.NGC_ERR_UNDECODABLE
        ngc.ngc_sync(ctx)
        assert torch.equal(before, bufs[1][3])                      # theta untouched
    finally:
        ngc.ngc_destroy(ctx)


def test_messages_of_subnormal_gradients(ngc, torch_dev):
    """Partial gradients below the smallest normal fp32 number: the stand-alone encode forms its
    messages on the matrix cores, the tail of ngc_iteration with scalar fused multiply-adds; both
    must keep subnormal terms (no flush to zero), give the same bits, and match the oracle to the
    spacing of subnormal numbers."""
    torch = torch_dev
    dev = torch.device("cuda:0")
    n, rows, d, layers = 8, 6, 256, (0, 1, 3)
    w = wl.C3.scaled(rows=rows, d=d, n=n, layers=layers)
    X, Y = wl.dataset(w, seed=3, threads=1)
    X = (X.astype(np.float64) * 1e-40).astype(np.float32)           # subnormal features
    assert np.all(np.abs(X) < 1.1754944e-38) and np.count_nonzero(X) > X.size // 2
    th = wl.theta(w, seed=1)
    Bs = codes.nested_code(n, layers, "cyclic", seed=0, draws=2)
    ctx = ngc.ngc_create(n, n, layers, d, torch.cuda.current_stream().cuda_stream)
    try:
        for u, B in enumerate(Bs):
            ngc.ngc_set_code(ctx, u, B)
        Xd, Yd = torch.from_numpy(X).to(dev), torch.from_numpy(Y).to(dev)
        L = len(layers)
        thd = torch.from_numpy(th).to(dev)
        G0 = torch.empty((n, d), dtype=torch.float32, device=dev)
        C0 = torch.empty((L, n, d), dtype=torch.float32, device=dev)
        G1, C1 = torch.empty_like(G0), torch.empty_like(C0)
        g1 = torch.empty(d, dtype=torch.float32, device=dev)
        ngc.ngc_partition_grads(ctx, w.loss, Xd, Yd, thd, rows, G0)
        ngc.ngc_encode(ctx, G0, -1, C0)
        ngc.ngc_iteration(ctx, w.loss, Xd, Yd, thd, rows, np.zeros(n, np.uint8), 0.0, G1, C1, g1, n)
        ngc.ngc_sync(ctx)
        assert torch.equal(G0, G1) and torch.equal(C0, C1)
        G, C = G0.cpu().numpy(), C0.cpu().numpy()
        tiny = 1.1754944e-38
        assert np.count_nonzero((np.abs(G) > 0) & (np.abs(G) < tiny)) > G.size // 2
        assert np.count_nonzero((np.abs(C[L - 1]) > 0) & (np.abs(C[L - 1]) < tiny)) > C[L - 1].size // 2
        G_o = gradients.partial_gradients(w.loss, X, Y, th)
        ulp = 2.0 ** -149                                            # spacing of subnormal fp32
        assert np.max(np.abs(G - G_o)) <= 4 * rows * ulp
        for u in range(L):
            C_o = coding.encode(Bs[u], G.astype(np.float64))         # from the GPU's G: the encode alone
            bound = (np.abs(Bs[u]) @ np.ones(n)).max() * (layers[u] + 2) * ulp
            assert np.max(np.abs(C[u] - C_o)) <= bound
    finally:
        ngc.ngc_destroy(ctx)


# --------------------------------------------------------------------------------------------
# C2 at full size: logistic regression, n = 16, 16 x 8192 rows, d = 1024, layers 0,1,3,7,
# 200 descent iterations with Bernoulli(0.2) stragglers, through ngc_iteration
# --------------------------------------------------------------------------------------------
def test_c2_full_size_200_iterations(ngc, torch_dev):
    torch = torch_dev
    dev = torch.device("cuda:0")
    w = wl.C2
    X, Y = wl.dataset(w, 0, threads=8)
    th0 = wl.theta(w, 0, scale=0.01)
    masks = wl.bernoulli_masks(w, 200, seed=0)
    p = Pipeline(ngc, torch, w)
    try:
        Xd, Yd, thd = p.to_dev(X), p.to_dev(Y), p.to_dev(th0)
        eta = 1.0
        usage = np.zeros(len(w.layers) + 1, int)
        checked = 0
        loss0 = gradients.logistic_loss(X.reshape(-1, w.d), Y.reshape(-1), th0)
        # the oracle's own run from the same start with the same masks: no number of it
        # comes from the GPU (the per-iteration checks below evaluate the oracle at the GPU's
        # theta_t instead, which pins each step; this pins the trajectory)
        th_free = th0.astype(np.float64)
        drift = 0.0
        for t in range(200):
            check = t < 3 or t % 10 == 0 or t == 199
            th_t = thd.cpu().numpy() if check else None
            if check:
                drift = max(drift, rel(th_t, th_free))
            try:
                _, _, g_free = coding.coded_gradient(p.Bs, w.layers,
                                                     gradients.partial_gradients(w.loss, X, Y, th_free), masks[t])
                th_free = gradients.gd_update(th_free, g_free, eta, w.m)
            except coding.Undecodable:
                pass
            try:
                u, a = ngc.ngc_iteration(p.ctx, w.loss, Xd, Yd, thd, w.rows, masks[t], eta / w.m,
                                         p.G, p.C, p.g, w.n)
            except ngc.NgcError as e:
                assert e.code == ngc.NGC_ERR_UNDECODABLE and masks[t].sum() > w.layers[-1]
                usage[-1] += 1                                    # theta stays as it is this round
                continue
            usage[u] += 1
            assert u == coding.select_layer(w.layers, masks[t])
            if check:
                ngc.ngc_sync(p.ctx)
                G_o = gradients.partial_gradients(w.loss, X, Y, th_t)
                u_o, a_o, g_o = coding.coded_gradient(p.Bs, w.layers, G_o, masks[t])
                assert np.array_equal(a != 0, a_o != 0)
                # near a stationary point the gradient is a difference of large terms: floor the
                # denominator at 1e-3 of the size it would have without cancellation
                Xf = X.reshape(-1, w.d).astype(np.float64)
                z = Y.reshape(-1) * (Xf @ th_t.astype(np.float64))
                slope = 1.0 / (1.0 + np.exp(z))
                floor = 1e-3 * np.sqrt(np.sum(slope ** 2 * np.sum(Xf ** 2, axis=1)))
                err = np.linalg.norm(p.g.cpu().numpy() - g_o) / max(np.linalg.norm(g_o), floor)
                assert err <= TOL, (t, err)
                assert rel(p.G.cpu().numpy(), G_o) <= TOL
                assert rel(thd.cpu().numpy(), gradients.gd_update(th_t, g_o, eta, w.m)) <= 1e-6
                checked += 1
        assert checked >= 20
        final_drift = rel(thd.cpu().numpy(), th_free)
        print("C2: theta of the GPU run against the oracle's own run: worst %.2e, after 200 iterations %.2e"
              % (max(drift, final_drift), final_drift))
        assert max(drift, final_drift) <= 1e-5
        loss1 = gradients.logistic_loss(X.reshape(-1, w.d), Y.reshape(-1), thd.cpu().numpy())
        assert loss1 < 0.5 * loss0                                # the run actually descends
        share = usage / 200.0
        print("C2: layer usage %s, undecodable %d of 200, loss %.4g -> %.4g" %
              (np.round(share[:-1], 3), usage[-1], loss0, loss1))
        # expected shares 2.8 / 11.3 / 45.7 / 39.5 % and 0.7 % undecodable
        assert share[2] + share[3] > 0.7 and usage[-1] <= 6
    finally:
        p.close()
