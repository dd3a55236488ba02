#!/usr/bin/env python3
"""Benchmark of the coded-gradient hot path on one MI355X.

A step is one iteration of nested gradient coding on the headline workload
(least squares, n = k = 32 workers/partitions, 32 x 16384 rows, d = 4096 fp32):
partition gradients -> encode of every layer -> host: straggler mask -> layer
and decode vector -> decode -> descent update.  X, y and theta are resident in
HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3|C2|C1] [--no-cpu-baseline]
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published


def metric_name(n, d):
    """The headline metric is quoted at n=32, d=4096; other workloads say their own shape."""
    return "partition-gradient samples/s + encode/decode GB/s vs HBM peak, n=%d d=%d" % (n, d)



def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured(summary, key):
    """(value, source) of the line 'key: value' in a committed rocprofv3 counter summary under
    profiles/, or (None, None) if a kernel source has changed since those counters were taken:
    the summary names every source file its kernels are built from with its sha256."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", summary)
    try:
        text = open(path).read()
    except OSError:
        return None, None
    named = re.findall(r"^source-sha256 (\S+): ([0-9a-f]{64})$", text, flags=re.M)
    if not named:
        return None, None
    for rel_path, sha in named:
        try:
            now = hashlib.sha256(open(os.path.join(ROOT, rel_path), "rb").read()).hexdigest()
        except OSError:
            return None, None
        if now != sha:
            return None, None
    for line in text.splitlines():
        if line.startswith(key + ":"):
            return float(line.split(":")[1]), ("profiles/%s (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs, committed; "
                                               "taken with the kernel sources as they are now)" % summary)
    return None, None


def with_traffic(roofline, summary, key="traffic-bytes-per-launch"):
    """Adds the measured HBM bytes per launch (or null) and where they come from."""
    value, source = measured(summary, key)
    roofline["traffic"] = value
    roofline["traffic_source"] = source
    return roofline


def blas_threads():
    """Threads the oracle's NumPy/BLAS calls run on."""
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline(w, wl, parts_host, theta, masks, budget_parts, Bs, layers):
    """The fp64 checker timed on the host cores over a bounded sample of the same
    workload: `budget_parts` partitions for the gradients, then encode of all
    layers, layer/decode-vector selection and decode at full n and d."""
    import numpy as np
    from oracle import coding, gradients
    cores = blas_threads()
    t0 = time.perf_counter()
    rows = []
    for X, Y in parts_host[:budget_parts]:
        rows.append(gradients.partial_gradients(w.loss, X[None], Y[None], theta, w.hidden, w.classes)[0])
    t_grad = time.perf_counter() - t0
    G = np.stack(rows + [rows[-1]] * (w.n - len(rows)))      # pad to n rows for the coding steps
    t1 = time.perf_counter()
    C = coding.encode_layers(Bs, G)
    u = coding.select_layer(layers, masks[0])
    a, _ = coding.decode_vector(Bs[u], masks[0])
    coding.decode(a, C[u])
    t_code = time.perf_counter() - t1
    samples = budget_parts * w.rows
    # whole-iteration time extrapolated: gradients scale with the partitions, coding does not
    t_iter = t_grad * (w.n / budget_parts) + t_code
    return {
        "value": w.m / t_iter, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
        "sample": "%d of %d partitions (%d samples) for the gradients in %.2f s, scaled by %g; "
                  "encode+select+decode at full n,d in %.3f s" %
                  (budget_parts, w.n, samples, t_grad, w.n / budget_parts, t_code),
    }


def oracle_code(ngc, ctx, L):
    """The code the library built, read back through the C ABI, as the oracle's input."""
    return [ngc.ngc_get_code(ctx, u) for u in range(L)]


def def1_residual(np, Bs, layers, seed=0, sets_per_layer=4):
    """Def. 1 checked in the oracle on sampled straggler sets of the design size sigma of every
    layer: largest |a B - 1| of the decode vectors (the responders must span the all-ones row)."""
    from oracle import coding
    rng = np.random.default_rng(seed)
    n = Bs[0].shape[0]
    worst = 0.0
    for u, sigma in enumerate(layers):
        for _ in range(sets_per_layer):
            m = np.zeros(n, np.uint8)
            m[rng.choice(n, size=sigma, replace=False)] = 1
            worst = max(worst, coding.decode_vector(Bs[u], m)[1])
    return worst


def rel_l2(np, x, ref):
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300))


def codec_parity(np, Bs, layers, G64, masks, lay, a_all, M_rows, g_rows):
    """Rounds of the fused encode + decode against the oracle.  M_rows(r) / g_rows(r) give the
    GPU's messages [n, d] and recovered gradient [d] of round r as host arrays."""
    from oracle import coding
    full = G64.sum(axis=0)
    msg, errs, kappas = 0.0, [], []
    layer_ok = support_ok = True
    for r in range(masks.shape[0]):
        u_o = coding.select_layer(layers, masks[r])
        a_o, _ = coding.decode_vector(Bs[u_o], masks[r])
        layer_ok &= int(lay[r]) == u_o
        support_ok &= bool(np.array_equal(a_all[r] != 0, a_o != 0))
        C_o = coding.encode(Bs[u_o], G64)
        Mh = M_rows(r)
        resp = np.flatnonzero(a_o != 0)
        msg = max(msg, rel_l2(np, Mh[resp], C_o[resp]))
        errs.append(rel_l2(np, g_rows(r), full))
        kappas.append(coding.conditioning(a_o, C_o, full))
    errs = np.array(errs)
    return {"rounds_checked": int(errs.size), "messages_rel_l2_max": msg,
            "decoded_rel_l2_max": float(errs.max()), "decoded_rel_l2_median": float(np.median(errs)),
            "share_of_rounds_within_1e-4": float(np.mean(errs <= 1e-4)), "kappa_max": float(max(kappas)),
            "decoded_within_4eps_kappa": bool(np.all(errs <= np.maximum(1e-4, 4 * 2.0 ** -24 * np.array(kappas)))),
            "layer_exact": bool(layer_ok), "support_exact": bool(support_ok)}


def bench_codec(args, w, wl, ngc, torch, np, rounds=None, cpu_leg=True):
    """Encode/decode stress (no data), n = 64 partial gradients of length 16384 resident in HBM.
    A step is one round: the messages of the round's layer for the responders of a
    Binomial(n, 0.2) straggler set and the recovered gradient.  Timed as the workload states it,
    `rounds` rounds with decode vectors solved per round: one ngc_coded_rounds call (host
    bookkeeping of every round, one table upload, one launch).  Beside it: the same with a new G
    every round (the tile cannot stay in LDS: every byte comes from HBM), the stand-alone
    kernels, and a loop of one launch pair per round with the host in it."""
    dev = torch.device("cuda:0")
    K = rounds if rounds is not None else args.steps
    W = args.warmup
    L = len(w.layers)
    n, d = w.n, w.d
    G = torch.from_numpy(wl.partial_gradients(w, 0)).to(dev)
    C = torch.empty((L, n, d), dtype=torch.float32, device=dev)
    g = torch.empty(d, dtype=torch.float32, device=dev)
    M = torch.empty((K, n, d), dtype=torch.float32, device=dev)
    gh = torch.empty((K, d), dtype=torch.float32, device=dev)
    masks = wl.binomial_count_masks(w, K, seed=0)
    masks[masks.sum(axis=1) > w.layers[-1]] = 0
    ctx = ngc.ngc_create(n, n, w.layers, d, torch.cuda.current_stream().cuda_stream)
    ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC if w.code == wl.CODE_CYCLIC else ngc.NGC_CODE_FRACREP, 0)

    # ---- the timed region: all K rounds in one call (warm-up calls first) ---------------------
    t_settle = time.perf_counter()                          # untimed: 100 ms of calls bring the card's clocks up
    while time.perf_counter() - t_settle < 0.1:
        ngc.ngc_coded_rounds(ctx, G, 0, masks, M, n * d, gh)
        torch.cuda.synchronize()
    for _ in range(max(1, min(W, 3))):
        ngc.ngc_coded_rounds(ctx, G, 0, masks, M, n * d, gh)
    torch.cuda.synchronize()
    ngc.ngc_profile_enable(ctx, ["rounds"])
    CALLS = 5                                               # the timed region: five calls of K rounds each
    t_host, walls = 0.0, []
    t0 = time.perf_counter()
    for _ in range(CALLS):
        tw = time.perf_counter()
        lay, a_all = ngc.ngc_coded_rounds(ctx, G, 0, masks, M, n * d, gh)
        t_host += time.perf_counter() - tw
        torch.cuda.synchronize()
        walls.append(time.perf_counter() - tw)
    elapsed = (time.perf_counter() - t0) / CALLS            # per call of K rounds
    t_host /= CALLS
    per_launch = ngc.ngc_profile_launches(ctx, "rounds")
    launches, kern_total_ms = ngc.ngc_profile_read(ctx)["rounds"]
    kern_ms = kern_total_ms / CALLS                         # kernel time of one call's K rounds
    per_call_launches = max(1, launches // CALLS)           # a call goes in runs (64, then 256 rounds each), one launch per run
    launch_ms = kern_total_ms / max(1, launches)
    resp = float(np.count_nonzero(a_all)) / K
    fused_bytes = 4.0 * d * (n + resp + 1)                  # G read + responders' messages written + gradient
    achieved = fused_bytes * K / (kern_ms * 1e-3) / 1e9
    # parity of exactly these rounds against the oracle (the library-built code goes to the oracle),
    # on rounds spread over the run, taken before the buffers are used again below
    Bs = oracle_code(ngc, ctx, L)
    G64 = G.cpu().numpy().astype(np.float64)
    sel = np.linspace(0, K - 1, min(K, 24)).astype(int)
    M_sel = [M[int(r)].cpu().numpy() for r in sel]
    g_sel = [gh[int(r)].cpu().numpy() for r in sel]
    parity = codec_parity(np, Bs, w.layers, G64, masks[sel], lay[sel], a_all[sel], lambda r: M_sel[r], lambda r: g_sel[r])
    parity["code"] = "ngc_build_code(seed 0), read back with ngc_get_code and handed to the oracle"
    parity["def1_residual_max"] = def1_residual(np, Bs, w.layers)
    del M_sel, g_sel
    # every round's recovered gradient against the exact sum of the partial gradients (fp64, host),
    # with the paper's layer rule (what was timed) and once more with the guarded layer choice
    full = G64.sum(axis=0)

    def all_round_errors(layers_chosen):
        gh_h = gh.cpu().numpy().astype(np.float64)
        e = np.linalg.norm(gh_h - full, axis=1) / np.linalg.norm(full)
        return e[layers_chosen >= 0]
    e_plain = all_round_errors(lay)
    parity["all_rounds"] = {"rounds": int(e_plain.size), "decoded_rel_l2_max": float(e_plain.max()),
                            "share_within_1e-4": float(np.mean(e_plain <= 1e-4))}
    if not args.only_timed:
        ngc.ngc_set_decode_guard(ctx, 1000.0)
        lay_g, _ = ngc.ngc_coded_rounds(ctx, G, 0, masks, M, n * d, gh)
        torch.cuda.synchronize()
        ngc.ngc_set_decode_guard(ctx, 0.0)
        e_guard = all_round_errors(lay_g)
        parity["all_rounds_guarded_choice"] = {
            "kappa_limit": 1000.0, "rounds": int(e_guard.size), "rounds_moved_up": int(np.count_nonzero(lay_g != lay)),
            "decoded_rel_l2_max": float(e_guard.max()), "share_within_1e-4": float(np.mean(e_guard <= 1e-4))}

    side = not args.only_timed
    # ---- the same rounds with a G of its own per round (streamed from HBM) --------------------
    Ks = min(K, 256) if side else 0
    if side:
        Gs = torch.randn((Ks, n, d), dtype=torch.float32, device=dev)
        ngc.ngc_coded_rounds(ctx, Gs, n * d, masks[:Ks], M, n * d, gh)
        ngc.ngc_profile_read(ctx)
        for _ in range(3):
            ngc.ngc_coded_rounds(ctx, Gs, n * d, masks[:Ks], M, n * d, gh)
        _, ms_s = ngc.ngc_profile_read(ctx)["rounds"]          # kernel time of the three calls (a call is several launches)
        resp_s = float(np.count_nonzero(a_all[:Ks])) / Ks
        stream_GBps = 4.0 * d * (n + resp_s + 1) * Ks * 3 / (ms_s * 1e-3) / 1e9
        del Gs

        # ---- stand-alone kernels and the per-round loop (host in the loop) ---------------------
        Kl = min(K, 300)
        ngc.ngc_profile_enable(ctx, ["encode", "decode", "rounds"])
        for t in range(Kl):
            ngc.ngc_encode(ctx, G, -1, C)
            ngc.ngc_decode(ctx, int(lay[t]), a_all[t], C, g)
            ngc.ngc_encode_decode(ctx, G, int(lay[t]), a_all[t], M[0], g)
        prof = ngc.ngc_profile_read(ctx)
        enc_ms = prof["encode"][1] / max(1, prof["encode"][0])
        dec_ms = prof["decode"][1] / max(1, prof["decode"][0])
        one_ms = prof["rounds"][1] / max(1, prof["rounds"][0])
        torch.cuda.synchronize()
        tl = time.perf_counter()
        for t in range(Kl):
            u, a, _ = ngc.ngc_select_decode_vec(ctx, masks[t], n)
            ngc.ngc_encode_decode(ctx, G, u, a, M[0], g)
        torch.cuda.synchronize()
        loop_ms = (time.perf_counter() - tl) / Kl * 1e3
    ngc.ngc_profile_enable(ctx, False)
    enc_bytes = 4.0 * n * d * (1 + L)
    dec_bytes = 4.0 * d * (resp + 1)

    stages = {"host_bookkeeping_ms_per_call": round(t_host * 1e3, 3),
              "call_ms_repeats": [round(x * 1e3, 3) for x in walls],
              "kernel_us_per_round": round(kern_ms / K * 1e3, 4),
              "batched_GBps": round(achieved, 1)}
    if side:
        stages.update({
            "batched_GBps_new_G_every_round": round(stream_GBps, 1),
            "encode_all_layers_ms": round(enc_ms, 4), "encode_GBps": round(enc_bytes / (enc_ms * 1e-3) / 1e9, 1),
            "decode_ms": round(dec_ms, 4), "decode_GBps": round(dec_bytes / (dec_ms * 1e-3) / 1e9, 1),
            "fused_one_round_ms": round(one_ms, 4),
            "fused_one_round_GBps": round(fused_bytes / (one_ms * 1e-3) / 1e9, 1),
            "round_ms_host_in_loop": round(loop_ms, 4)})
    roofline = with_traffic(
        {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(achieved / HBM_PEAK_GBS, 4), "algorithmic_bytes": fused_bytes * K / per_call_launches,
         "kernel": "coded_rounds_kernel (%d rounds per call in %d launches, one G for all rounds)" % (K, per_call_launches),
         "avg_ms": round(launch_ms, 4), "launches": launches,
         "median_ms": round(float(np.median(per_launch)), 4) if per_launch.size else None,
         "note": "algorithmic bytes per round = 4 n d (G) + 4 n_S d (messages written) + 4 d; with one G for all "
                 "rounds a block reads its tile of G once and keeps it in LDS, so the HBM traffic is mostly the "
                 "messages (see traffic)"},
        "coded_rounds_%s.txt" % w.name)
    out = {
        "metric": metric_name(n, d),
        "value": round(fused_bytes * K / elapsed / 1e9, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": K * CALLS, "warmup": W, "ms_per_step": round(elapsed / K * 1e3, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n": n, "d": d, "layers": list(w.layers),
                   "p_straggle": w.p_straggle, "mean_responders": resp, "rounds_per_call": K, "calls": CALLS},
        "roofline": roofline,
        "stages": stages,
        "parity": parity,
    }
    if cpu_leg and not args.no_cpu_baseline:
        from oracle import coding
        cnt = min(K, 20)
        t0 = time.perf_counter()
        for t in range(cnt):
            u = coding.select_layer(w.layers, masks[t])
            a, _ = coding.decode_vector(Bs[u], masks[t])
            coding.decode(a, coding.encode(Bs[u], G64).astype(np.float32))
        dt = (time.perf_counter() - t0) / cnt
        out["cpu_baseline"] = {"value": fused_bytes / dt / 1e9, "unit": "GB/s",
                               "cores": blas_threads(), "kind": "oracle",
                               "sample": "%d rounds of layer choice, decode vector, encode of the layer and decode at full n, d" % cnt}
    ngc.ngc_destroy(ctx)
    return out


def bench_workers(args, w, wl, ngc, torch, np):
    """Redundancy-faithful execution under stragglers: every simulated worker computes its own
    partial gradients layer by layer (a partition held by s+1 workers is read s+1 times).
    Workers advance in lockstep, stragglers (Bernoulli per worker) never report; the main node
    stops at the first decodable layer.  Timed for the nested code and for a conventional
    gradient code with fixed sigma = s_max on the same masks; the value is useful (unique)
    samples per second of the nested code."""
    dev = torch.device("cuda:0")
    K, W = args.steps, args.warmup
    L = len(w.layers)
    Xd = torch.empty((w.n, w.rows, w.d_in), dtype=torch.float32, device=dev)
    mlp = w.loss == wl.LOSS_MLP2
    Yd = torch.empty((w.n, w.rows), dtype=torch.int32 if mlp else torch.float32, device=dev)
    truth = None if mlp else wl.truth_vector(w, 0)
    keep = None                                          # host copies for the oracle's leg
    if not args.no_cpu_baseline:
        keep = (np.empty((w.n, w.rows, w.d_in), np.float32), np.empty((w.n, w.rows), np.int32 if mlp else np.float32))
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        for j, (X, Y) in enumerate(ex.map(lambda j: wl.partition(w, j, 0, truth), range(w.n))):
            Xd[j].copy_(torch.from_numpy(X))
            Yd[j].copy_(torch.from_numpy(Y))
            if keep is not None:
                keep[0][j] = X
                keep[1][j] = Y
    theta_h = wl.theta(w, 0)
    thd = torch.from_numpy(theta_h).to(dev)
    masks = wl.bernoulli_masks(w, K + W, seed=0)
    masks[masks.sum(axis=1) > w.layers[-1]] = 0
    ctx = ngc.ngc_create(w.n, w.n, w.layers, w.d, torch.cuda.current_stream().cuda_stream)
    ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC if w.code == wl.CODE_CYCLIC else ngc.NGC_CODE_FRACREP, 0)
    if mlp:
        ngc.ngc_set_mlp2_shape(ctx, w.d_in, w.hidden, w.classes)
    T = ngc.ngc_worker_task_count(ctx)
    Wd = torch.empty((w.n, T, w.d), dtype=torch.float32, device=dev)
    C = torch.empty((L, w.n, w.d), dtype=torch.float32, device=dev)
    g = torch.empty(w.d, dtype=torch.float32, device=dev)

    def iteration(mask, min_layer):
        # lockstep workers: all responders have finished t tasks after t steps
        alive = (mask == 0).astype(np.int32)
        for t in range(1, T + 1):
            progress = alive * t
            try:
                u, m2, a, _ = ngc.ngc_select_from_progress(ctx, progress, w.n, min_layer)
                break
            except ngc.NgcError as e:
                if e.code != ngc.NGC_ERR_UNDECODABLE:
                    raise
        ngc.ngc_worker_grads(ctx, w.loss, Xd, Yd, thd, w.rows, progress, Wd)
        ngc.ngc_worker_encode(ctx, Wd, progress, C)
        ngc.ngc_decode(ctx, u, a, C, g)
        return int(progress.sum())

    res = {}
    kern = "mlp" if mlp else "grad"
    for name, min_layer in (("nested", 0), ("fixed_sigma", L - 1)):
        for t in range(W):
            iteration(masks[t], min_layer)
        torch.cuda.synchronize()
        if name == "nested":
            ngc.ngc_profile_enable(ctx, [kern])          # events around the gradient kernels
        tasks = 0
        t0 = time.perf_counter()
        for t in range(W, W + K):
            tasks += iteration(masks[t], min_layer)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if name == "nested":
            launches, kern_ms = ngc.ngc_profile_read(ctx)[kern]
            ngc.ngc_profile_enable(ctx, False)
            nested_tasks = tasks
        res[name] = {"ms_per_iteration": round(dt / K * 1e3, 4), "tasks_per_iteration": tasks / K,
                     "useful_samples_per_s": round(w.m * K / dt, 1),
                     "computed_samples_per_s": round(tasks * w.rows / dt, 1)}
    # Roofline of the gradient kernel over the timed iterations of the nested code.  Algorithmic
    # work counts every worker's own pass over each partition it computes (the paper's model:
    # every worker holds its copies); workers that read the same partition at the same time
    # share the caches, so the HBM traffic is lower than these bytes.
    if mlp:
        flops = nested_tasks * w.rows * (2.0 * w.d_in * w.hidden * 2 + 2.0 * w.hidden * w.classes * 3)
        achieved = flops / (kern_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": 157.3, "unit": "TFLOP/s",
                    "frac": round(achieved / 157.3, 4), "traffic": None, "traffic_source": None,
                    "algorithmic_flops": flops / K,
                    "kernel": "mlp_gemm_kernel (whole MLP gradient call, one unit per worker task)",
                    "avg_ms": round(kern_ms / max(1, launches), 4), "launches": launches}
    else:
        nbytes = nested_tasks * w.rows * (4.0 * w.d + 4.0) + K * 4.0 * w.d
        achieved = nbytes / (kern_ms * 1e-3) / 1e9
        roofline = with_traffic(
            {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
             "frac": round(achieved / HBM_PEAK_GBS, 4),
             "algorithmic_bytes": nbytes / K, "kernel": "grad_stream_kernel (one unit per worker task)",
             "avg_ms": round(kern_ms / max(1, launches), 4), "launches": launches,
             "note": "algorithmic bytes count every worker's own pass over each partition it computes; workers "
                     "that read the same partition in one launch share the caches, so the HBM traffic (mean per "
                     "launch over the same iterations) is lower than these bytes and `achieved` is not an HBM rate"},
            "worker_execution_%s.txt" % w.name)
    out = {
        "metric": metric_name(w.n, w.d) + " (worker execution, useful samples/s)",
        "value": res["nested"]["useful_samples_per_s"], "unit": "samples/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": res["nested"]["ms_per_iteration"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name + " (redundancy-faithful worker execution)", "n": w.n,
                   "rows_per_partition": w.rows, "d": w.d, "layers": list(w.layers),
                   "p_straggle": w.p_straggle},
        "nested_code": res["nested"], "fixed_sigma_code": res["fixed_sigma"],
        "speedup_over_fixed_sigma": round(res["fixed_sigma"]["ms_per_iteration"] /
                                          res["nested"]["ms_per_iteration"], 3),
        "roofline": roofline,
    }
    Bs = oracle_code(ngc, ctx, L)        # the code the timed run used goes to the oracle's leg
    ngc.ngc_destroy(ctx)
    if keep is not None:
        # the oracle's worker execution of one iteration (the first timed straggler pattern):
        # every task of every worker recomputed in fp64, messages, termination rule, decoding
        from oracle import coding, workers as ow
        Xh, Yh = keep
        alive = (masks[W] == 0).astype(np.int64)
        for t in range(1, T + 1):
            progress = alive * t
            try:
                ow.terminate(Bs, w.layers, progress, 0)
                break
            except coding.Undecodable:
                continue
        t0 = time.perf_counter()
        Wp = ow.worker_partials(w.loss, Xh, Yh, theta_h, Bs, progress, w.hidden, w.classes)
        ow.decode_from_workers(Bs, w.layers, Wp, progress, 0)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": w.m / dt, "unit": "samples/s", "cores": blas_threads(), "kind": "oracle",
                               "sample": "one iteration of the worker execution (%d tasks of %d samples) in %.2f s"
                                         % (int(progress.sum()), w.rows, dt)}
    print(json.dumps(out), flush=True)


def bench_latency(args, ngc, torch, np):
    """Latency model of Sec. IV at the parameters of the paper's figures (n = k = 8, lambda = 0.5,
    rho = 0.5, eps = 0.1, p_e = 0.05, t - gamma in [2, 18]): closed-form CDFs of the nested code
    (s_max = 2, 3, 4, 6) and of conventional codes (sigma = 0..6), and a Monte-Carlo simulation of
    the same model on the GPU.  value = simulated trials per second for s_max = 6."""
    dev = torch.device("cuda:0")
    n, par = 8, (0.5, 0.5, 0.1, 0.0, 0.05)
    ts = np.linspace(2.0, 18.0, 33)
    trials = 1 << 22
    curves, worst = {}, 0.0
    rate = None
    for smax in (2, 3, 4, 6):
        L = torch.empty((smax + 1, trials), dtype=torch.float64, device=dev)
        T = torch.empty(trials, dtype=torch.float64, device=dev)
        stream = torch.cuda.current_stream().cuda_stream
        ngc.ngc_latency_simulate(stream, n, smax, *par, 99, trials, L, T)      # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for rep in range(args.steps):
            ngc.ngc_latency_simulate(stream, n, smax, *par, 100 + rep, trials, L, T)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        if smax == 6:
            rate = trials / dt
        closed = ngc.ngc_latency_cdf_ngc(n, smax, *par, ts)
        emp = np.array([float((T <= float(t)).double().mean().item()) for t in ts])
        worst = max(worst, float(np.max(np.abs(emp - closed))))
        curves["nested_smax_%d" % smax] = [round(float(v), 5) for v in closed[::4]]
    for sigma in (0, 1, 2, 3, 4, 6):
        curves["fixed_sigma_%d" % sigma] = [round(float(v), 5) for v in
                                            ngc.ngc_latency_cdf_gc(n, sigma, *par, ts)[::4]]
    out = {
        "metric": "latency-model simulated iterations/s (off the headline metric)",
        "value": round(rate, 1), "unit": "simulated iterations/s", "n_gpus": 1, "steps": args.steps,
        "warmup": 1, "ms_per_step": round(trials / rate * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "latency model, n=k=8, lambda=0.5, rho=0.5, eps=0.1, p_e=0.05",
                   "trials_per_step": trials},
        "t_minus_gamma": [float(t) for t in ts[::4]], "cdf": curves,
        "max_abs_deviation_simulation_vs_closed_form": round(worst, 6),
        "uncoded_limit": float(ngc.ngc_latency_cdf_gc(n, 0, *par, [1e6])[0]),
    }
    # Bound by plain vector arithmetic (integer Philox rounds, fp64 logarithms, compare-exchange
    # sorting): achieved = vector instructions per launch (counter summary) x 64 lanes / launch
    # time, against one vector instruction per SIMD every four clocks over 64 lanes
    # (256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz).
    valu, valu_source = measured("latency_sim_n8.txt", "valu-instructions-per-launch-smax6")
    peak = 256 * 4 * 16 * 2.4e9 / 1e12
    ach = None if valu is None else valu * 64.0 / (trials / rate) / 1e12
    out["roofline"] = {"bound": "alu", "achieved": None if ach is None else round(ach, 2), "peak": round(peak, 1),
                       "unit": "T lane-ops/s", "frac": None if ach is None else round(ach / peak, 4),
                       "traffic": None, "kernel": "latency_sim_kernel (s_max = 6)",
                       "note": "achieved = counted vector instructions of a launch x 64 lanes / launch time",
                       "avg_ms": round(trials / rate * 1e3, 4), "launches": args.steps}
    if not args.no_cpu_baseline:
        from oracle import latency as ol
        chunk, chunks = 1 << 20, 8                      # in pieces: the oracle holds a trial's draws in memory
        sample = chunk * chunks
        t0 = time.perf_counter()
        for q in range(chunks):
            ol.simulate(chunk, n, 6, *par, seed=1 + q)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": sample / dt, "unit": "simulated iterations/s", "cores": 1, "kind": "oracle",
                               "sample": "%d trials of the s_max = 6 model in %.2f s (NumPy, one thread)" % (sample, dt)}
    print(json.dumps(out), flush=True)


def bench_lookup(args, wl, ngc, torch, np):
    """Small cluster with explicit decoding matrices A_sigma (Def. 1) held on the device: per round
    the host only ranks the straggler set, the kernel reads its decode vector from the table.
    Timed beside the route that solves for the vector on the host, on the same messages and
    masks (n = 16, layers 0/1/3/7, gradient length 16384, Binomial(n, 0.2) stragglers)."""
    import dataclasses
    dev = torch.device("cuda:0")
    K, W = args.steps, args.warmup
    w = dataclasses.replace(wl.C5, name="lookup-n16", n=16, layers=(0, 1, 3, 7))
    L = len(w.layers)
    G = torch.from_numpy(wl.partial_gradients(w, 0)).to(dev)
    C = torch.empty((L, w.n, w.d), dtype=torch.float32, device=dev)
    g = torch.empty(w.d, dtype=torch.float32, device=dev)
    masks = wl.binomial_count_masks(w, K + W, seed=0)
    masks[masks.sum(axis=1) > w.layers[-1]] = 0
    ctx = ngc.ngc_create(w.n, w.n, w.layers, w.d, torch.cuda.current_stream().cuda_stream)
    ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC, 0)
    t0 = time.perf_counter()
    table_rows = [ngc.ngc_build_decoding_table(ctx, u) for u in range(L)]
    t_tables = time.perf_counter() - t0
    ngc.ngc_encode(ctx, G, -1, C)
    layer_of = [next(u for u, s in enumerate(w.layers) if s >= cnt) for cnt in range(w.layers[-1] + 1)]

    def by_lookup(t):
        u = layer_of[int(masks[t].sum())]
        ngc.ngc_decode_lookup(ctx, u, masks[t], C, g)
        return w.n - w.layers[u]                     # a table row is supported on n - sigma responders

    def by_solve(t):
        u, a, _ = ngc.ngc_select_decode_vec(ctx, masks[t], w.n)
        ngc.ngc_decode(ctx, u, a, C, g)
        return int(np.count_nonzero(a))

    res = {}
    for name, fn in (("lookup", by_lookup), ("solve", by_solve)):
        for t in range(W):
            fn(t)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        used = 0
        for t in range(W, W + K):
            used += fn(t)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ngc.ngc_profile_enable(ctx, ["decode"])      # kernel durations in a pass of their own
        for t in range(W, W + min(K, 200)):
            fn(t)
        cnt, ms = ngc.ngc_profile_read(ctx)["decode"]
        ngc.ngc_profile_enable(ctx, False)
        res[name] = {"us_per_round": round(dt / K * 1e6, 2), "kernel_us": round(ms / max(1, cnt) * 1e3, 2),
                     "messages_read_per_round": used / K}
    # host part alone: ranking a straggler set against solving for its decode vector
    t0 = time.perf_counter()
    for t in range(W, W + K):
        ngc.ngc_decoding_row_index(ctx, layer_of[int(masks[t].sum())], masks[t])
    res["lookup"]["host_us"] = round((time.perf_counter() - t0) / K * 1e6, 2)
    t0 = time.perf_counter()
    for t in range(W, W + K):
        ngc.ngc_select_decode_vec(ctx, masks[t], w.n)
    res["solve"]["host_us"] = round((time.perf_counter() - t0) / K * 1e6, 2)
    nbytes = 4.0 * w.d * (res["lookup"]["messages_read_per_round"] + 1) + 8.0 * w.n
    achieved = nbytes / (res["lookup"]["kernel_us"] * 1e-6) / 1e9
    out = {
        "metric": "decode rounds/s with the decode vector looked up in A_sigma on the device, n=%d d=%d" % (w.n, w.d),
        "value": round(1e6 / res["lookup"]["us_per_round"], 1), "unit": "rounds/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": round(res["lookup"]["us_per_round"] * 1e-3, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "explicit decoding matrices, n=%d, d=%d" % (w.n, w.d), "n": w.n, "d": w.d,
                   "layers": list(w.layers), "p_straggle": w.p_straggle, "table_rows": table_rows,
                   "table_build_s": round(t_tables, 3)},
        "lookup_route": res["lookup"], "solve_route": res["solve"],
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None, "algorithmic_bytes": nbytes,
                     "kernel": "decode_lookup_kernel", "avg_ms": round(res["lookup"]["kernel_us"] * 1e-3, 5),
                     "launches": min(K, 200)},
    }
    if not args.no_cpu_baseline:
        # the oracle's route: A_sigma of every layer built beforehand, per round the row of the
        # straggler set (padded to sigma stragglers with the responders of highest index) and the sum
        import itertools
        from oracle import codes, coding
        Bs = codes.nested_code(w.n, w.layers, "cyclic", seed=0, draws=2)
        Gh = G.cpu().numpy()
        Co = coding.encode_layers(Bs, Gh)
        tables, index = [], []
        for u, sigma in enumerate(w.layers):
            tables.append(codes.decoding_matrix(Bs[u], sigma))
            index.append({out_: r for r, out_ in enumerate(itertools.combinations(range(w.n), sigma))})
        rounds = min(K, 2000)
        t0 = time.perf_counter()
        for t in range(W, W + rounds):
            m = masks[t]
            u = coding.select_layer(w.layers, m)
            out_ = [i for i in range(w.n) if m[i]]
            for i in range(w.n - 1, -1, -1):          # fewer stragglers than sigma: the last responders idle
                if len(out_) == w.layers[u]:
                    break
                if not m[i]:
                    out_.append(i)
            coding.decode(tables[u][index[u][tuple(sorted(out_))]], Co[u])
        dt = (time.perf_counter() - t0) / rounds
        out["cpu_baseline"] = {"value": 1.0 / dt, "unit": "rounds/s", "cores": 1, "kind": "oracle",
                               "sample": "%d rounds of layer choice, table row and decode (tables built beforehand)" % rounds}
    ngc.ngc_destroy(ctx)
    print(json.dumps(out), flush=True)


def bench_pipeline(args, w, wl, ngc, torch, np, K, W, cpu_leg=True, probe=True, parity_parts=None):
    """One workload through the whole path.  A step is one iteration: partition gradients,
    every layer's messages, layer + decode vector for the round's stragglers, decode, update
    (two launches for the regression losses).  Returns the result line as a dict."""
    dev = torch.device("cuda:0")
    is_mlp = w.loss == wl.LOSS_MLP2
    # k = c n: the workload's w.n partitions go to nw = w.n / c workers, c to an atomic task; the
    # layers that such a smaller cluster can hold are kept
    c = args.parts_per_worker
    nw = w.n // c
    layers = tuple(s for s in w.layers if s < nw)
    L = len(layers)
    parity_parts = w.n if parity_parts is None else min(parity_parts, w.n)
    keep_parts = max(parity_parts, min(args.cpu_parts, w.n) if cpu_leg and not args.no_cpu_baseline else 0)

    # ---- inputs: generated per partition on the host, uploaded once -------------------------
    t0 = time.perf_counter()
    Xd = torch.empty((w.n, w.rows, w.d_in), dtype=torch.float32, device=dev)
    Yd = torch.empty((w.n, w.rows), dtype=torch.int32 if is_mlp else torch.float32, device=dev)
    truth = None if is_mlp else wl.truth_vector(w, 0)
    keep = []
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        for j, (X, Y) in enumerate(ex.map(lambda j: wl.partition(w, j, 0, truth), range(w.n))):
            Xd[j].copy_(torch.from_numpy(X))
            Yd[j].copy_(torch.from_numpy(Y))
            if j < keep_parts:
                keep.append((X, Y))
    theta_h = wl.theta(w, 0)
    thd = torch.from_numpy(theta_h).to(dev)
    masks = np.ascontiguousarray(wl.bernoulli_masks(w, K + W, seed=0)[:, :nw])
    # a round with more stragglers than the code tolerates cannot be decoded (prob. ~1e-8 here);
    # such a mask is replaced by "no stragglers" so that every timed step does the full work
    masks[masks.sum(axis=1) > layers[-1]] = 0
    torch.cuda.synchronize()
    log("%s: inputs ready in %.1f s (X %.2f GB in HBM)" % (w.name, time.perf_counter() - t0, Xd.numel() * 4 / 1e9))

    stream = torch.cuda.current_stream().cuda_stream
    ctx = ngc.ngc_create(nw, w.n, layers, w.d, stream)
    ngc.ngc_build_code(ctx, ngc.NGC_CODE_CYCLIC if w.code == wl.CODE_CYCLIC else ngc.NGC_CODE_FRACREP, 0)
    if is_mlp:
        ngc.ngc_set_mlp2_shape(ctx, w.d_in, w.hidden, w.classes)
    G = torch.empty((w.n, w.d), dtype=torch.float32, device=dev)
    C = torch.empty((L, nw, w.d), dtype=torch.float32, device=dev)
    g = torch.empty(w.d, dtype=torch.float32, device=dev)
    eta_over_m = 1e-3 / w.m

    def step(t):
        return ngc.ngc_iteration(ctx, w.loss, Xd, Yd, thd, w.rows, masks[t], eta_over_m, G, C, g, nw)

    def step_separate(t):
        ngc.ngc_partition_grads(ctx, w.loss, Xd, Yd, thd, w.rows, G)
        ngc.ngc_encode(ctx, G, -1, C)
        u, a, _ = ngc.ngc_select_decode_vec(ctx, masks[t], nw)
        ngc.ngc_decode(ctx, u, a, C, g)
        ngc.ngc_update(ctx, thd, g, eta_over_m)
        return u, a

    # Untimed: after an idle spell (the host just built and uploaded the data) the card needs some
    # tens of milliseconds of work before its clocks are up; steps run until 100 ms have passed, theta is
    # put back, then come the W warm-up steps.
    th_start = thd.clone()
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < 0.1:
        for t in range(4):
            step(t % (W + K))
        torch.cuda.synchronize()
    thd.copy_(th_start)
    for t in range(W):
        step(t)
    torch.cuda.synchronize()
    ngc.ngc_profile_enable(ctx, ["mlp" if is_mlp else "grad"])   # events around the dominant part only
    resp = 0
    t0 = time.perf_counter()
    for t in range(W, W + K):
        u, a = step(t)
        resp += int(np.count_nonzero(a))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_launch = ngc.ngc_profile_launches(ctx, "mlp" if is_mlp else "grad")
    prof = ngc.ngc_profile_read(ctx)
    ms_per_step = elapsed / K * 1e3
    # the small kernels are timed in a pass of their own, after the timed region
    ngc.ngc_profile_enable(ctx, True)
    for t in range(W, W + min(K, 10)):
        step(t)
    prof_tail = ngc.ngc_profile_read(ctx)
    for t in range(W, W + min(K, 10)):
        step_separate(t)
    prof_small = ngc.ngc_profile_read(ctx)
    ngc.ngc_profile_enable(ctx, False)
    for name in ("grad", "mlp", "reduce", "encode", "decode", "update"):
        if prof[name][0] == 0:
            prof[name] = prof_small[name]
    prof["tail"] = prof_tail["tail"]
    resp_per_step = resp / K

    # ---- roofline of the dominant kernel -------------------------------------------------------
    if is_mlp:
        # the two fp32 MFMA GEMMs (forward layer 1 and dW1) carry 98 % of the flops; timed here is
        # the whole gradient call (GEMM, head pass, GEMM, closing sums)
        grad_launches, grad_ms = prof["mlp"]
        grad_avg_ms = grad_ms / max(1, grad_launches)
        flops = w.m * (2.0 * w.d_in * w.hidden * 2 + 2.0 * w.hidden * w.classes * 3)
        achieved = flops / (grad_avg_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": 157.3, "unit": "TFLOP/s",
                    "frac": round(achieved / 157.3, 4), "traffic": None, "traffic_source": None,
                    "algorithmic_flops": flops,
                    "kernel": "mlp_gemm_kernel (whole MLP gradient call)", "avg_ms": round(grad_avg_ms, 4),
                    "launches": grad_launches}
        if w.name == wl.C4.name:                      # the counters were taken at this workload's shape
            with_traffic(roofline, "mlp_gemm_C4-mlp-n20.txt")
    else:
        grad_launches, grad_ms = prof["grad"]
        grad_avg_ms = grad_ms / max(1, grad_launches)
        # rows of 4, 8, .. 128 features take the kernel that loads several rows at once
        dq = w.d // 4
        grad_kernel = "grad_narrow_kernel" if (w.d % 4 == 0 and w.d <= 128 and dq & (dq - 1) == 0) else "grad_stream_kernel"
        # other rows of fewer than 64 features (all that are no multiple of 4) are read as one flat stretch
        if (w.d < 64 and (w.d % 4 != 0 or dq & (dq - 1) != 0)) or \
                (64 < w.d <= 248 and w.d != 128 and (w.d % 4 != 0 or w.d <= 132)):
            grad_kernel = "grad_flat_kernel"
        if w.d > 32768 or (w.d % 4 != 0 and w.d > 16384):   # no single-pass shape: X is read twice
            grad_kernel = "resid_kernel + xtr_kernel (two passes over X)"
        # algorithmic bytes per launch: X once + labels + theta + G  (4*d bytes per sample)
        grad_bytes = 4.0 * w.m * w.d + 4.0 * w.m + 4.0 * w.d + 4.0 * w.n * w.d
        achieved = grad_bytes / (grad_avg_ms * 1e-3) / 1e9
        roofline = with_traffic(
            {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
             "frac": round(achieved / HBM_PEAK_GBS, 4), "algorithmic_bytes": grad_bytes,
             "kernel": grad_kernel, "avg_ms": round(grad_avg_ms, 4), "launches": grad_launches},
            "%s_%s.txt" % (grad_kernel[:-len("_kernel")], w.name))
    if per_launch.size:
        # the same launches one by one (HIP events of the timed region): spread of the kernel's time
        roofline["median_ms"] = round(float(np.median(per_launch)), 4)
        roofline["min_ms"] = round(float(per_launch.min()), 4)
    enc_ms = prof["encode"][1] / max(1, prof["encode"][0])
    dec_ms = prof["decode"][1] / max(1, prof["decode"][0])
    enc_bytes = 4.0 * w.d * (w.n + L * nw)
    dec_bytes = 4.0 * w.d * (resp_per_step + 1)
    stages = {
        "grad_samples_per_s": round(w.m / (grad_avg_ms * 1e-3), 1),
        "reduce_ms": round(prof["reduce"][1] / max(1, prof["reduce"][0]), 4),
        "encode_ms": round(enc_ms, 4), "encode_GBps": round(enc_bytes / (enc_ms * 1e-3) / 1e9, 1),
        "decode_ms": round(dec_ms, 4), "decode_GBps": round(dec_bytes / (dec_ms * 1e-3) / 1e9, 1),
        "update_ms": round(prof["update"][1] / max(1, prof["update"][0]), 4),
        "fused_tail_ms": round(prof["tail"][1] / max(1, prof["tail"][0]), 4),
    }

    # ---- encode/decode of this workload's code batched: many rounds on this G in one launch ------
    if c == 1:
        Rb = int(max(8, min(512, (1 << 30) // (4 * nw * w.d))))          # at most 1 GiB of messages
        bm = wl.bernoulli_masks(w, Rb, seed=1)
        bm[bm.sum(axis=1) > layers[-1]] = 0
        Mb = torch.empty((Rb, nw, w.d), dtype=torch.float32, device=dev)
        gb = torch.empty((Rb, w.d), dtype=torch.float32, device=dev)
        ngc.ngc_partition_grads(ctx, w.loss, Xd, Yd, thd, w.rows, G)
        ngc.ngc_coded_rounds(ctx, G, 0, bm, Mb, nw * w.d, gb)
        torch.cuda.synchronize()
        ngc.ngc_profile_enable(ctx, ["rounds"])
        wall_b, call_b = [], []
        for _ in range(3):
            tb = time.perf_counter()
            lay_b, a_b = ngc.ngc_coded_rounds(ctx, G, 0, bm, Mb, nw * w.d, gb)
            call_b.append(time.perf_counter() - tb)
            torch.cuda.synchronize()
            wall_b.append(time.perf_counter() - tb)
        log("%s: batched rounds, wall per call %s ms, of which inside the call %s ms" %
            (w.name, [round(x * 1e3, 3) for x in wall_b], [round(x * 1e3, 3) for x in call_b]))
        wall_b = sorted(wall_b)[1]
        _, ms_b = ngc.ngc_profile_read(ctx)["rounds"]
        ms_b /= 3.0                                          # kernel time of one call (a call is several launches)
        ngc.ngc_profile_enable(ctx, False)
        rb = float(np.count_nonzero(a_b)) / Rb
        fb = 4.0 * w.d * (w.n + rb + 1)
        stages["batched_rounds"] = {"rounds_per_call": Rb, "kernel_us_per_round": round(ms_b / Rb * 1e3, 4),
                                    "GBps": round(fb * Rb / (ms_b * 1e-3) / 1e9, 1),
                                    "GBps_with_host_bookkeeping": round(fb * Rb / wall_b / 1e9, 1),
                                    "bytes_per_round": fb}
        del Mb, gb

    # ---- context figures outside the timed region: what a trivial kernel reaches ---------------
    ceiling = None
    if probe:
        ngc.ngc_profile_enable(ctx, True)
        for _ in range(3):
            ngc.ngc_probe_read(ctx, Xd, Xd.numel() * 4)
        n_read, ms_read = ngc.ngc_profile_read(ctx)["probe"]
        scratch = torch.empty(1 << 28, dtype=torch.float32, device=dev)          # 1 GiB
        nb = min(scratch.numel(), Xd[0].numel()) * 4
        for _ in range(3):
            ngc.ngc_probe_copy(ctx, Xd[0], scratch, nb)
        n_copy, ms_copy = ngc.ngc_profile_read(ctx)["probe"]
        ngc.ngc_profile_enable(ctx, False)
        del scratch
        ceiling = {"plain_read_GBps": round(Xd.numel() * 4 * n_read / (ms_read * 1e-3) / 1e9, 1),
                   "plain_copy_GBps_read_plus_write": round(2 * nb * n_copy / (ms_copy * 1e-3) / 1e9, 1),
                   "copy_bytes": nb}
    if ceiling and roofline.get("bound") == "hbm":
        # the same rate against what a plain read of the same buffer reaches on this machine
        roofline["frac_of_plain_read"] = round(roofline["achieved"] / ceiling["plain_read_GBps"], 4)

    out = {
        "metric": metric_name(nw, w.d),
        "value": round(w.m * K / elapsed, 1), "unit": "samples/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name if c == 1 else "%s, %d partitions per worker" % (w.name, c),
                   "loss": ("lsq", "logistic", "mlp2")[w.loss], "n": nw, "partitions": w.n,
                   "rows_per_partition": w.rows, "d": w.d, "layers": list(layers),
                   "p_straggle": w.p_straggle},
        "roofline": roofline, "stages": stages, "hbm_probe": ceiling,
    }

    # ---- parity of exactly this configuration against the oracle, after the timed region -------
    # the library-built code goes to the oracle; theta is reset to the start point; the oracle's
    # partial gradients come from the host copies of the same partitions
    ngc.ngc_sync(ctx)
    from oracle import coding, gradients
    Bs = oracle_code(ngc, ctx, L)
    thd.copy_(torch.from_numpy(theta_h))
    ngc.ngc_partition_grads(ctx, w.loss, Xd, Yd, thd, w.rows, G)
    ngc.ngc_encode(ctx, G, -1, C)
    ngc.ngc_sync(ctx)
    t_or = time.perf_counter()
    G_o = np.stack([gradients.partial_gradients(w.loss, X[None], Y[None], theta_h, w.hidden, w.classes)[0]
                    for X, Y in keep[:parity_parts]])
    t_or = time.perf_counter() - t_or
    Gh = G.cpu().numpy()
    parity = {"code": "ngc_build_code(seed 0), read back with ngc_get_code and handed to the oracle",
              "def1_residual_max": def1_residual(np, Bs, layers),
              "G_partitions_checked": parity_parts,
              "G_rel_l2_max": max(rel_l2(np, Gh[j], G_o[j]) for j in range(parity_parts))}
    if parity_parts == w.n:
        C_o = coding.encode_layers(Bs, G_o)
        parity["C_rel_l2"] = rel_l2(np, C.cpu().numpy(), C_o)
        Rp = min(K, 16)
        pm = masks[W:W + Rp]
        lay_p = np.zeros(Rp, np.int32)
        a_p = np.zeros((Rp, nw))
        g_p, M_p = [], []
        for r in range(Rp):
            lay_p[r], a_p[r], _ = ngc.ngc_select_decode_vec(ctx, pm[r], nw)
            ngc.ngc_decode(ctx, int(lay_p[r]), a_p[r], C, g)
            ngc.ngc_sync(ctx)
            g_p.append(g.cpu().numpy())
            M_p.append(C[int(lay_p[r])].cpu().numpy())
        parity.update(codec_parity(np, Bs, layers, G_o, pm, lay_p, a_p, lambda r: M_p[r], lambda r: g_p[r]))
    out["parity"] = parity

    if cpu_leg and not args.no_cpu_baseline:
        cb = cpu_baseline(w, wl, keep, theta_h, masks, min(args.cpu_parts, w.n), Bs, layers)
        # the same algorithmic bytes (fp32 sizes) per sample as the GPU figure, and the ratio
        cb["GBps"] = round(cb["value"] * 4.0 * w.d_in / 1e9, 2) if w.loss != wl.LOSS_MLP2 else None
        cb["gpu_over_oracle"] = round(out["value"] / cb["value"], 1) if cb["value"] else None
        out["cpu_baseline"] = cb
    ngc.ngc_destroy(ctx)
    del Xd, Yd, G, C, g, keep
    gc.collect()
    torch.cuda.empty_cache()
    return out


def compact(line):
    """What the other workloads contribute to the headline line."""
    keep = ("value", "unit", "steps", "ms_per_step", "dtype", "config", "roofline", "parity")
    out = {k: line[k] for k in keep if k in line}
    st = line.get("stages", {})
    out["stages"] = {k: st[k] for k in ("batched_GBps", "batched_GBps_new_G_every_round", "kernel_us_per_round",
                                        "encode_GBps", "decode_GBps", "fused_one_round_ms", "grad_samples_per_s",
                                        "fused_tail_ms", "batched_rounds") if k in st}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, help="C1..C5; default: C3 (the headline) followed by short "
                                                     "legs of C2, C4 and C5 under other_workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="headline workload only")
    ap.add_argument("--only-timed", action="store_true",
                    help="encode/decode stress: the timed batched launches only, none of the side measurements "
                         "(so that a kernel trace holds one kind of launch per kernel)")
    ap.add_argument("--mode", default="pipeline", choices=["pipeline", "workers", "latency", "lookup"])
    ap.add_argument("--cpu-parts", type=int, default=32)
    ap.add_argument("--rows", type=int, default=0,
                    help="rows per partition instead of the workload's own (same distributions): a longer "
                         "stream through the same kernel, named in config.workload")
    ap.add_argument("--features", type=int, default=0,
                    help="features per row instead of the workload's own (regression workloads; same "
                         "distributions): other shapes of the gradient kernel, named in config.workload")
    ap.add_argument("--parts-per-worker", type=int, default=1,
                    help="k = c n (Sec. II-C): the workload's partitions are shared out c to a worker")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: nested gradient coding here simulates all n workers on "
              "a single MI355X; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2212_08580_amd import ngc, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    # With torch imported a pass of the interpreter's cycle collector takes milliseconds, as long
    # as a thousand encode/decode rounds; the objects alive now are set aside and the collector
    # is run between the legs instead of whenever an allocation count trips it inside a timed region.
    gc.collect()
    gc.freeze()
    gc.disable()
    if args.mode == "latency":
        return bench_latency(args, ngc, torch, np)
    if args.mode == "lookup":
        return bench_lookup(args, wl, ngc, torch, np)
    headline_only = (args.workload is not None or args.no_others or args.parts_per_worker != 1 or
                     args.mode != "pipeline" or args.rows > 0 or args.features > 0)
    w = wl.CONFIGS[args.workload or "C3"]
    if args.rows > 0 and w.loss >= 0:
        import dataclasses
        w = dataclasses.replace(w, rows=args.rows, name="%s-rows%d" % (w.name, args.rows))
    if args.features > 0:
        if w.loss not in (wl.LOSS_LSQ, wl.LOSS_LOGISTIC):
            print("--features needs a regression workload (C1..C3)", file=sys.stderr)
            sys.exit(2)
        w = w.scaled(d=args.features, name="%s-d%d" % (w.name, args.features))
    if args.mode == "workers":
        if w.loss < 0:
            print("--mode workers needs a gradient workload (C1..C4)", file=sys.stderr)
            sys.exit(2)
        return bench_workers(args, w, wl, ngc, torch, np)
    if w.loss < 0:
        print(json.dumps(bench_codec(args, w, wl, ngc, torch, np)), flush=True)
        return
    if args.parts_per_worker < 1 or w.n % args.parts_per_worker:
        print("--parts-per-worker must divide the workload's %d partitions" % w.n, file=sys.stderr)
        sys.exit(2)
    out = bench_pipeline(args, w, wl, ngc, torch, np, args.steps, args.warmup, probe=not args.no_probe)
    if not headline_only:
        # the other workloads of the benchmark definition, short legs, same code path
        others = {}
        others["C2"] = compact(bench_pipeline(args, wl.C2, wl, ngc, torch, np, 100, 5, cpu_leg=False, probe=False))
        others["C4"] = compact(bench_pipeline(args, wl.C4, wl, ngc, torch, np, 10, 2, cpu_leg=False, probe=False,
                                              parity_parts=2))
        others["C5"] = compact(bench_codec(args, wl.C5, wl, ngc, torch, np, rounds=1000, cpu_leg=False))
        out["other_workloads"] = others
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
