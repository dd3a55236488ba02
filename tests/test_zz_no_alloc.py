"""The entry point that allocates nothing (ngc_partition_grads_static) against ngc_partition_grads.

Two calls in a row through the C ABI on one GPU, the second on a smaller input, so that
what the first call left in the shared static scratch must not show in the second result;
each compared bit for bit with the allocating entry point (same kernels, same launch shape)
and to rel-L2 <= 1e-4 with the fp64 oracle.  Also the documented refusals.
"""
import numpy as np
import pytest

from oracle import gradients
from paper_2212_08580_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-4


def rel(x, ref):
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300))


def run_both(ngc, torch, w, seed, scale=None):
    dev = torch.device("cuda:0")
    X, Y = wl.dataset(w, seed=seed, threads=2)
    th = wl.theta(w, seed=seed + 1, scale=scale)
    ctx = ngc.ngc_create(w.n, w.n, (0,), w.d, torch.cuda.current_stream().cuda_stream)
    try:
        Xd, Yd, thd = (torch.from_numpy(a).to(dev) for a in (X, Y, th))
        G_static = torch.full((w.n, w.d), 7.0, dtype=torch.float32, device=dev)
        G_alloc = torch.full((w.n, w.d), -7.0, dtype=torch.float32, device=dev)
        ngc.ngc_partition_grads_static(ctx, w.loss, Xd, Yd, thd, w.rows, G_static)
        ngc.ngc_sync(ctx)
        return ctx, (Xd, Yd, thd), G_static, G_alloc, X, Y, th
    except Exception:
        ngc.ngc_destroy(ctx)
        raise


def test_static_scratch_entry_point_two_calls_in_a_row(ngc):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run on the MI355X box)")
    torch.cuda.set_device(0)
    # first call: the headline shape shrunk in rows only (n = 32, d = 4096, ragged row count);
    # second call: a smaller problem (fewer partitions, shorter unaligned rows, other loss)
    # before them: rows wider than 16384 features (theta in LDS), still one pass and within the scratch
    cases = [(wl.C3.scaled(rows=9, d=20000, n=2, layers=(0,), name="static-0"), 10, None),
             (wl.C3.scaled(rows=203, name="static-1"), 11, None),
             (wl.C2.scaled(rows=50, d=1002, n=3, layers=(0,), name="static-2"), 12, 2.0 / np.sqrt(1002)),
             # short rows read as one flat stretch: one lane per row, then eight lanes per row; X ends inside a float4
             (wl.C3.scaled(rows=3001, d=54, n=3, layers=(0,), name="static-3"), 13, None),
             (wl.C2.scaled(rows=77, d=199, n=1, layers=(0,), name="static-4"), 14, 2.0 / np.sqrt(199))]
    for w, seed, scale in cases:
        print("static entry point: n=%d rows=%d d=%d loss=%d" % (w.n, w.rows, w.d, w.loss), flush=True)
        ctx, (Xd, Yd, thd), G_static, G_alloc, X, Y, th = run_both(ngc, torch, w, seed, scale)
        try:
            first = G_static.clone()
            ngc.ngc_partition_grads(ctx, w.loss, Xd, Yd, thd, w.rows, G_alloc)
            ngc.ngc_sync(ctx)
            assert torch.equal(G_static, G_alloc)
            G_o = gradients.partial_gradients(w.loss, X, Y, th)
            Gh = G_static.cpu().numpy()
            assert np.all(np.isfinite(Gh))
            for j in range(w.n):
                assert rel(Gh[j], G_o[j]) <= TOL, (j, rel(Gh[j], G_o[j]))
            # and once more after the allocating call used its own workspace
            ngc.ngc_partition_grads_static(ctx, w.loss, Xd, Yd, thd, w.rows, G_static)
            ngc.ngc_sync(ctx)
            assert torch.equal(G_static, first)
        finally:
            ngc.ngc_destroy(ctx)


def test_static_scratch_entry_point_refusals(ngc):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run on the MI355X box)")
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    # a gradient too long for the 20 MiB of static scratch (two partitions of 3 000 000 floats)
    d = 3_000_000
    ctx = ngc.ngc_create(2, 2, (0,), d, stream)
    try:
        X = torch.zeros((2, 1, d), dtype=torch.float32, device=dev)
        y = torch.zeros((2, 1), dtype=torch.float32, device=dev)
        th = torch.zeros(d, dtype=torch.float32, device=dev)
        G = torch.full((2, d), 3.0, dtype=torch.float32, device=dev)
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_partition_grads_static(ctx, wl.LOSS_LSQ, X, y, th, 1, G)
        assert e.value.code == ngc.NGC_ERR_INVALID and "static scratch" in str(e.value)
        ngc.ngc_sync(ctx)
        assert bool((G == 3.0).all())                          # nothing was launched
        ngc.ngc_partition_grads(ctx, wl.LOSS_LSQ, X, y, th, 1, G)   # the allocating call takes it
        ngc.ngc_sync(ctx)
        assert bool((G == 0.0).all())
    finally:
        ngc.ngc_destroy(ctx)
    # the perceptron loss is refused outright
    w = wl.C4.scaled(rows=8, n=2, layers=(0,), name="static-mlp")
    ctx = ngc.ngc_create(w.n, w.n, (0,), w.d, stream)
    try:
        ngc.ngc_set_mlp2_shape(ctx, w.d_in, w.hidden, w.classes)
        X = torch.zeros((w.n, w.rows, w.d_in), dtype=torch.float32, device=dev)
        y = torch.zeros((w.n, w.rows), dtype=torch.int32, device=dev)
        th = torch.zeros(w.d, dtype=torch.float32, device=dev)
        G = torch.zeros((w.n, w.d), dtype=torch.float32, device=dev)
        with pytest.raises(ngc.NgcError) as e:
            ngc.ngc_partition_grads_static(ctx, wl.LOSS_MLP2, X, y, th, w.rows, G)
        assert e.value.code == ngc.NGC_ERR_INVALID
    finally:
        ngc.ngc_destroy(ctx)
