"""Fused encode + decode (Sec. II-C, X = B G, then the recovery of Def. 1) through the C ABI:
one round (ngc_encode_decode) and many rounds in one launch (ngc_coded_rounds).

Checked per round: layer and support of the decode vector exact against the oracle; every
message that is written against the oracle's B G (rel-L2 <= 1e-6) and bit for bit against
ngc_encode; the recovered gradient against the oracle's fp64 combination of the fp32-rounded
messages (<= 2e-7: the kernel must use the rounded message, not the unrounded sum), bit for bit
against ngc_decode, and against the exact sum of the partial gradients within
max(1e-4, 4 * 2^-24 * kappa).
"""
import numpy as np
import pytest

from conftest import parity_report
from oracle import codes, coding
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


def make_ctx(ngc, torch, n, k, layers, d, Bs):
    ctx = ngc.ngc_create(n, k, layers, d, torch.cuda.current_stream().cuda_stream)
    for u, B in enumerate(Bs):
        ngc.ngc_set_code(ctx, u, B)
    return ctx


def library_code(ngc, torch, n, layers, d, kind="cyclic"):
    """Context with the code the library builds (what the benchmark times) and that code read back
    for the oracle, which checks Def. 1 on sampled straggler sets first."""
    ctx = ngc.ngc_create(n, n, layers, d, torch.cuda.current_stream().cuda_stream)
    ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC if kind == "cyclic" else ngc.NGC_CODE_FRACREP, 0)
    Bs = [ngc.ngc_get_code(ctx, u) for u in range(len(layers))]
    rng = np.random.default_rng(0)
    for u, sigma in enumerate(layers):
        for _ in range(6):
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=sigma, replace=False)] = 1
            assert coding.decode_vector(Bs[u], m)[1] <= 1e-9
    return ctx, Bs


def random_masks(rng, n, smax, rounds):
    masks = np.zeros((rounds, n), np.uint8)
    for t in range(rounds):
        s = int(rng.integers(0, smax + 1))
        masks[t, rng.choice(n, size=s, replace=False)] = 1
    return masks


def oracle_round(Bs, layers, G64, mask, guard=None):
    """layer, decode vector, fp32-rounded messages of the layer, their fp64 combination, kappa;
    guard: limit of the guarded layer choice, None for the plain rule."""
    if guard is None:
        u = coding.select_layer(layers, mask)
        a, _ = coding.decode_vector(Bs[u], mask)
    else:
        u, a = coding.select_guarded(Bs, layers, mask, guard)
    C = coding.encode(Bs[u], G64)
    C32 = C.astype(np.float32)
    g = coding.decode(a, C32)
    kappa = coding.conditioning(a, C, G64.sum(axis=0))
    return u, a, C, C32, g, kappa


@pytest.mark.parametrize("n,c,layers,kind,d", [
    (4, 1, (0, 1), "fracrep", 64), (16, 1, (0, 1, 3, 7), "cyclic", 1024), (32, 1, (0, 1, 3, 7, 15), "cyclic", 4096),
    (64, 1, (0, 1, 3, 7, 15, 31), "cyclic", 16384), (64, 1, (0, 1, 3, 7, 15, 31), "fracrep", 4096),
    (20, 1, (0, 1, 4, 9), "cyclic", 1002), (20, 1, (0, 1, 4, 9), "cyclic", 999), (7, 1, (0, 2, 5), "cyclic", 100),
    (1, 1, (0,), "cyclic", 5), (33, 1, (0, 32), "cyclic", 68), (8, 2, (0, 1, 3), "cyclic", 1024),
    (6, 3, (0, 2), "cyclic", 200), (16, 1, tuple(range(8)), "cyclic", 300),
])
def test_one_round_fused_equals_encode_then_decode(ngc, torch_dev, n, c, layers, kind, d):
    torch = torch_dev
    dev = torch.device("cuda:0")
    k = n * c
    w = wl.C5.scaled(n=k, d=d, layers=layers)
    G_h = wl.partial_gradients(w, seed=n + d)
    G64 = G_h.astype(np.float64)
    Bs = codes.expand_partitions(codes.nested_code(n, layers, kind, seed=0, draws=2), c)
    ctx = make_ctx(ngc, torch, n, k, layers, d, Bs)
    try:
        L = len(layers)
        G = torch.from_numpy(G_h).to(dev)
        C = torch.empty((L, n, d), dtype=torch.float32, device=dev)
        g_sep = torch.empty(d, dtype=torch.float32, device=dev)
        g_fused = torch.empty(d, dtype=torch.float32, device=dev)
        ngc.ngc_encode(ctx, G, -1, C)
        rng = np.random.default_rng(7)
        for mask in random_masks(rng, n, layers[-1], 10):
            u, a, resid = ngc.ngc_select_decode_vec(ctx, mask, n)
            u_o, a_o, C_o, C32_o, g_o, kappa = oracle_round(Bs, layers, G64, mask)
            assert u == u_o and np.array_equal(a != 0, a_o != 0)
            M = torch.full((n, d), -7.0, dtype=torch.float32, device=dev)
            ngc.ngc_decode(ctx, u, a, C, g_sep)
            ngc.ngc_encode_decode(ctx, G, u, a, M, g_fused)
            ngc.ngc_sync(ctx)
            resp = np.flatnonzero(a != 0)
            out = np.flatnonzero(a == 0)
            ridx = torch.from_numpy(resp).to(dev)
            assert torch.equal(M[ridx], C[u][ridx])                      # same bits as ngc_encode
            assert torch.equal(g_fused, g_sep)                           # same bits as ngc_decode
            if out.size:
                assert bool((M[torch.from_numpy(out).to(dev)] == -7.0).all())   # stragglers send nothing
            Mh = M.cpu().numpy()
            for i in resp:
                assert rel(Mh[i], C_o[i]) <= 1e-6
            gh = g_fused.cpu().numpy()
            assert rel(gh, coding.decode(a, Mh)) <= 2e-7                 # fp64 combination of the written messages
            assert rel(gh, G64.sum(axis=0)) <= max(TOL, 4 * 2.0 ** -24 * kappa)
    finally:
        ngc.ngc_destroy(ctx)


def run_rounds(ngc, torch, ctx, w, Bs, G_h, masks, g_stride, check_messages_every=1, oracle_every=1, guard=None):
    """ngc_coded_rounds over `masks`, checked round by round.  G_h: [k, d] (g_stride 0) or
    [rounds, k, d].  guard: the limit set with ngc_set_decode_guard, if any.  Returns the decode
    errors against the exact gradient sum."""
    dev = torch.device("cuda:0")
    n, d, layers = w.n, w.d, w.layers
    rounds = masks.shape[0]
    L = len(layers)
    G = torch.from_numpy(G_h).to(dev)
    M = torch.full((rounds, n, d), -7.0, dtype=torch.float32, device=dev)
    gh = torch.full((rounds, d), -7.0, dtype=torch.float32, device=dev)
    lay, a_all = ngc.ngc_coded_rounds(ctx, G, g_stride, masks, M, n * d, gh)
    ngc.ngc_sync(ctx)
    C = torch.empty((L, n, d), dtype=torch.float32, device=dev)
    g_sep = torch.empty(d, dtype=torch.float32, device=dev)
    if g_stride == 0:
        ngc.ngc_encode(ctx, G, -1, C)
    errs, worst_msg, worst_comb = [], 0.0, 0.0
    for r in range(rounds):
        Gr = G_h if g_stride == 0 else G_h[r]
        mask = masks[r]
        if mask.sum() > layers[-1]:
            assert lay[r] == -1 and not a_all[r].any()
            assert bool((gh[r] == 0.0).all()) and bool((M[r] == -7.0).all())
            continue
        u, a = int(lay[r]), a_all[r]
        assert u >= coding.select_layer(layers, mask) and (guard is not None or u == coding.select_layer(layers, mask))
        assert np.all(a[mask == 1] == 0)
        resp = np.flatnonzero(a != 0)
        ridx = torch.from_numpy(resp).to(dev)
        if r % check_messages_every == 0:
            # bit for bit against the separate calls
            if g_stride != 0:
                ngc.ngc_encode(ctx, G[r], u, C)
            ngc.ngc_decode(ctx, u, a, C, g_sep)
            ngc.ngc_sync(ctx)
            assert torch.equal(M[r][ridx], C[u][ridx]), r
            assert torch.equal(gh[r], g_sep), r
            out = np.flatnonzero(a == 0)
            if out.size:
                assert bool((M[r][torch.from_numpy(out).to(dev)] == -7.0).all())
        if r % oracle_every == 0:
            G64 = Gr.astype(np.float64)
            u_o, a_o, C_o, C32_o, g_o, kappa = oracle_round(Bs, layers, G64, mask, guard)
            assert u == u_o and np.array_equal(a != 0, a_o != 0)
            Mh = M[r].cpu().numpy()
            worst_msg = max(worst_msg, max(rel(Mh[i], C_o[i]) for i in resp))
            g_r = gh[r].cpu().numpy()
            worst_comb = max(worst_comb, rel(g_r, coding.decode(a, Mh)))
            err = rel(g_r, G64.sum(axis=0))
            assert err <= max(TOL, 4 * 2.0 ** -24 * kappa), (r, err, kappa)
            errs.append(err)
    assert worst_msg <= 1e-6 and worst_comb <= 2e-7, (worst_msg, worst_comb)
    return np.array(errs)


def test_coded_rounds_c5_all_1000_rounds(ngc, torch_dev):
    """The encode/decode stress workload as a whole: n = 64, d = 16384, layers 0..31 in six steps,
    1000 rounds with Binomial(64, 0.2) straggler counts, one G, one launch."""
    w = wl.C5
    G_h = wl.partial_gradients(w, 0)
    masks = wl.binomial_count_masks(w, 1000, seed=0)
    ctx, Bs = library_code(ngc, torch_dev, w.n, w.layers, w.d)
    try:
        errs = run_rounds(ngc, torch_dev, ctx, w, Bs, G_h, masks, 0)
        assert errs.size >= 990
        # every round is inside the forward-error bound (run_rounds); those above 1e-4 are rounds whose
        # straggler count equals the layer's tolerance (one decode vector, no choice)
        assert float(np.mean(errs > TOL)) <= 0.01
        parity_report(test="coded_rounds_c5", rounds=int(errs.size), median_decode_rel_l2=float(np.median(errs)),
                      worst_decode_rel_l2=float(errs.max()), share_above_1e_4=float(np.mean(errs > TOL)))
    finally:
        ngc.ngc_destroy(ctx)


def test_coded_rounds_c5_guarded_layer_choice(ngc, torch_dev):
    """The same 1000 rounds with the guarded layer choice (limit 1000 on the estimated
    amplification): the rounds whose only decode vector is huge move one layer up, layers and
    supports are the oracle's guarded ones, and every round is within plain 1e-4."""
    w = wl.C5
    G_h = wl.partial_gradients(w, 0)
    masks = wl.binomial_count_masks(w, 1000, seed=0)
    ctx, Bs = library_code(ngc, torch_dev, w.n, w.layers, w.d)
    try:
        ngc.ngc_set_decode_guard(ctx, 1000.0)
        errs = run_rounds(ngc, torch_dev, ctx, w, Bs, G_h, masks, 0, check_messages_every=10, guard=1000.0)
        assert errs.size >= 990 and errs.max() <= TOL
        moved = sum(coding.select_guarded(Bs, w.layers, m, 1000.0)[0] != coding.select_layer(w.layers, m)
                    for m in masks if m.sum() <= w.layers[-1])
        assert 0 < moved <= 0.1 * errs.size
        parity_report(test="coded_rounds_c5_guarded", rounds=int(errs.size), kappa_limit=1000.0, rounds_moved_up=int(moved),
                      median_decode_rel_l2=float(np.median(errs)), worst_decode_rel_l2=float(errs.max()),
                      share_above_1e_4=float(np.mean(errs > TOL)))
        ngc.ngc_set_decode_guard(ctx, 0.0)
    finally:
        ngc.ngc_destroy(ctx)


def test_coded_rounds_c3_masks(ngc, torch_dev):
    """The headline code (n = 32, d = 4096, layers 0,1,3,7,15) under its own Bernoulli(0.1)
    stragglers, 400 rounds on one G."""
    w = wl.C3
    G_h = wl.partial_gradients(wl.C5.scaled(n=w.n, d=w.d, layers=w.layers), 3)
    masks = wl.bernoulli_masks(w, 400, seed=5)
    ctx, Bs = library_code(ngc, torch_dev, w.n, w.layers, w.d)
    try:
        errs = run_rounds(ngc, torch_dev, ctx, w, Bs, G_h, masks, 0)
        assert errs.size >= 395 and errs.max() <= TOL                   # plain 1e-4 on every round
        parity_report(test="coded_rounds_c3", rounds=int(errs.size), median_decode_rel_l2=float(np.median(errs)),
                      worst_decode_rel_l2=float(errs.max()))
    finally:
        ngc.ngc_destroy(ctx)


@pytest.mark.parametrize("n,layers,kind,d,rounds", [(16, (0, 1, 3, 7), "cyclic", 1000, 70),
                                                    (12, (0, 1, 2, 3, 5), "cyclic", 4099, 33),
                                                    (8, (0, 1, 3), "fracrep", 66, 300)])
def test_coded_rounds_with_a_gradient_per_round_and_undecodable_rounds(ngc, torch_dev, n, layers, kind, d, rounds):
    """Every round has its own G (stride k*d: the tile is staged anew each round); some rounds
    have more stragglers than the code tolerates: zero gradient, no message, not an error."""
    w = wl.C5.scaled(n=n, d=d, layers=layers)
    rng = np.random.default_rng(n + d)
    G_h = rng.standard_normal((rounds, n, d)).astype(np.float32)
    masks = random_masks(rng, n, layers[-1], rounds)
    for r in range(0, rounds, 9):
        masks[r] = 0
        masks[r, rng.choice(n, size=layers[-1] + 1, replace=False)] = 1      # one too many
    Bs = codes.nested_code(n, layers, kind, seed=0, draws=2)
    ctx = make_ctx(ngc, torch_dev, n, n, layers, d, Bs)
    try:
        run_rounds(ngc, torch_dev, ctx, w, Bs, G_h, masks, n * d)
        run_rounds(ngc, torch_dev, ctx, w, Bs, G_h[0], masks[:5], 0)        # fewer rounds afterwards
        # the guarded layer choice on the same rounds, then the plain rule again
        ngc.ngc_set_decode_guard(ctx, 50.0)
        run_rounds(ngc, torch_dev, ctx, w, Bs, G_h, masks, n * d, guard=50.0)
        ngc.ngc_set_decode_guard(ctx, 0.0)
        run_rounds(ngc, torch_dev, ctx, w, Bs, G_h[:7], masks[:7], n * d)
    finally:
        ngc.ngc_destroy(ctx)


@pytest.mark.parametrize("n,c,layers,d,rounds,g_pad,m_pad", [
    (7, 3, (0, 2, 5), 257, 40, 7, 5),          # n not a multiple of 4, k = 3 n, odd d, unaligned strides
    (13, 2, (0, 1, 4, 9), 1028, 130, 4, 4),    # 16-byte aligned strides with gaps
    (62, 1, (0, 1, 4), 100, 33, 0, 8),         # one G for all rounds, gaps between the rounds' messages
    (1, 1, (0,), 5, 3, 3, 1),                  # a single worker
    (21, 3, (0, 20), 64, 600, 0, 0),           # k = 63, full tolerance, more rounds than one launch takes
])
def test_coded_rounds_with_padded_strides_and_several_partitions_per_worker(ngc, torch_dev, n, c, layers, d, rounds,
                                                                            g_pad, m_pad):
    """k = c n partitions (Sec. II-A), strides larger than one round's data: the gaps keep their
    contents, every round equals the stand-alone calls bit for bit and the oracle's B G within
    the message tolerance."""
    torch = torch_dev
    dev = torch.device("cuda:0")
    k = n * c
    rng = np.random.default_rng(1000 * n + d)
    ctx = ngc.ngc_create(n, k, layers, d, torch.cuda.current_stream().cuda_stream)
    try:
        ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC, 3)
        Bs = [ngc.ngc_get_code(ctx, u) for u in range(len(layers))]
        assert all(B.shape == (n, k) for B in Bs)
        gs = k * d + g_pad if g_pad else 0
        ms = n * d + m_pad
        G = torch.from_numpy(rng.standard_normal((rounds - 1) * gs + k * d).astype(np.float32)).to(dev)
        M = torch.full(((rounds - 1) * ms + n * d,), -7.0, dtype=torch.float32, device=dev)
        gh = torch.full((rounds, d), -7.0, dtype=torch.float32, device=dev)
        masks = random_masks(rng, n, layers[-1], rounds)
        if layers[-1] + 1 <= n:
            masks[rounds // 2] = 0
            masks[rounds // 2, rng.choice(n, size=layers[-1] + 1, replace=False)] = 1
        lay, a_all = ngc.ngc_coded_rounds(ctx, G, gs, masks, M, ms, gh)
        ngc.ngc_sync(ctx)
        C = torch.empty((len(layers), n, d), dtype=torch.float32, device=dev)
        g_sep = torch.empty(d, dtype=torch.float32, device=dev)
        for r in range(rounds):
            Gr = G[r * gs: r * gs + k * d]
            Mr = M[r * ms: r * ms + n * d].view(n, d)
            if r + 1 < rounds and m_pad:
                assert bool((M[r * ms + n * d: (r + 1) * ms] == -7.0).all()), r
            if masks[r].sum() > layers[-1]:
                assert lay[r] == -1 and bool((gh[r] == 0).all()) and bool((Mr == -7.0).all()), r
                continue
            u = coding.select_layer(layers, masks[r])
            a_o, _ = coding.decode_vector(Bs[u], masks[r])
            assert lay[r] == u and np.array_equal(a_all[r] != 0, a_o != 0), r
            ngc.ngc_encode(ctx, Gr, u, C)
            ngc.ngc_decode(ctx, u, a_all[r], C, g_sep)
            ngc.ngc_sync(ctx)
            resp = torch.from_numpy(np.flatnonzero(a_all[r] != 0)).to(dev)
            out = torch.from_numpy(np.flatnonzero(a_all[r] == 0)).to(dev)
            assert torch.equal(Mr[resp], C[u][resp]) and torch.equal(gh[r], g_sep), r
            assert bool((Mr[out] == -7.0).all()), r
            if r % 16 == 0:
                G64 = Gr.cpu().numpy().astype(np.float64).reshape(k, d)
                C_o = coding.encode(Bs[u], G64)
                Mh = Mr.cpu().numpy()
                for i in np.flatnonzero(a_all[r] != 0):
                    assert rel(Mh[i], C_o[i]) <= 1e-6, (r, i)
                assert rel(g_sep.cpu().numpy(), coding.decode(a_all[r], Mh)) <= 2e-7, r
    finally:
        ngc.ngc_destroy(ctx)


def test_coded_rounds_rejects_bad_arguments(ngc, torch_dev):
    torch = torch_dev
    dev = torch.device("cuda:0")
    n, d, layers = 4, 64, (0, 1)
    Bs = codes.nested_code(n, layers, "cyclic", seed=0, draws=2)
    ctx = make_ctx(ngc, torch, n, n, layers, d, Bs)
    try:
        G = torch.zeros((3, n, d), dtype=torch.float32, device=dev)
        M = torch.zeros((3, n, d), dtype=torch.float32, device=dev)
        g = torch.zeros((3, d), dtype=torch.float32, device=dev)
        masks = np.zeros((3, n), np.uint8)
        with pytest.raises(ngc.NgcError):
            ngc.ngc_coded_rounds(ctx, G, 5, masks, M, n * d, g)               # stride neither 0 nor >= k*d
        with pytest.raises(ngc.NgcError):
            ngc.ngc_coded_rounds(ctx, G, 0, masks, M, n * d - 1, g)           # rounds' messages would overlap
        with pytest.raises(ValueError):
            ngc.ngc_coded_rounds(ctx, G, 0, masks, M[:2], n * d, g)           # buffer too small for 3 rounds
        with pytest.raises(ngc.NgcError):
            ngc.ngc_encode_decode(ctx, G, 2, np.ones(n), M, g)                # no such layer
        bad = np.ones(n)
        bad[1] = np.nan
        with pytest.raises(ngc.NgcError):
            ngc.ngc_encode_decode(ctx, G, 1, bad, M, g)
    finally:
        ngc.ngc_destroy(ctx)
