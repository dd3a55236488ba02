"""Monte-Carlo latency simulation on the device against the oracle's simulation
(same counter-based random numbers, so every draw is compared) and against the
closed forms."""
import math

import numpy as np
import pytest

from oracle import latency as ol

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,smax,lam,rho,eps,gamma,pe,seed", [
    (8, 3, 0.5, 0.5, 0.1, 0.0, 0.05, 11),           # the paper's figure parameters
    (8, 6, 0.5, 0.5, 0.1, 0.0, 0.05, 12),
    (5, 0, 1.0, 0.0, 0.0, 0.3, 0.2, 13),
    (64, 15, 2.0, 0.1, 0.01, 0.0, 0.1, (7 << 32) | 5),
    (33, 8, 0.7, 0.2, 0.0, 0.0, 0.0, 14),
    (12, 5, 0.9, 0.3, 0.05, 0.1, 0.1, 15),          # 16 lanes per trial, four trials per wave
    (20, 9, 0.6, 0.4, 0.0, 0.0, 0.08, 16),          # 32 lanes per trial
])
def test_device_draws_equal_oracle_draws(ngc, n, smax, lam, rho, eps, gamma, pe, seed):
    import torch
    dev = torch.device("cuda:0")
    trials = 3001
    L = torch.empty((smax + 1, trials), dtype=torch.float64, device=dev)
    T = torch.empty(trials, dtype=torch.float64, device=dev)
    ngc.ngc_latency_simulate(torch.cuda.current_stream().cuda_stream, n, smax, lam, rho, eps, gamma, pe,
                             seed, trials, L, T)
    torch.cuda.synchronize()
    Lh, Th = L.cpu().numpy().T, T.cpu().numpy()
    Lo = ol.simulate(trials, n, smax, lam, rho, eps, gamma, pe, seed)
    assert np.array_equal(np.isinf(Lh), np.isinf(Lo))                 # same failures, exactly
    fin = np.isfinite(Lo)
    assert np.allclose(Lh[fin], Lo[fin], rtol=1e-12, atol=0.0)
    To = Lo.min(axis=1)
    assert np.array_equal(np.isinf(Th), np.isinf(To))
    assert np.allclose(Th[np.isfinite(To)], To[np.isfinite(To)], rtol=1e-12, atol=0.0)


def test_simulation_reproduces_the_closed_forms_of_the_figures(ngc):
    import torch
    dev = torch.device("cuda:0")
    n, trials = 8, 1 << 20
    par = (0.5, 0.5, 0.1, 0.0, 0.05)
    ts = np.linspace(2.0, 18.0, 17)
    tol = 4.0 * math.sqrt(0.25 / trials)
    for smax in (2, 3, 4, 6):
        L = torch.empty((smax + 1, trials), dtype=torch.float64, device=dev)
        T = torch.empty(trials, dtype=torch.float64, device=dev)
        ngc.ngc_latency_simulate(0, n, smax, *par, 1234 + smax, trials, L, T)
        torch.cuda.synchronize()
        Th, Lh = T.cpu().numpy(), L.cpu().numpy()
        nested = ngc.ngc_latency_cdf_ngc(n, smax, *par, ts)
        for q, t in enumerate(ts):
            assert abs(np.mean(Th <= t) - nested[q]) < tol
        for sigma in range(smax + 1):
            gc = ngc.ngc_latency_cdf_gc(n, sigma, *par, ts)
            for q, t in enumerate(ts):
                assert abs(np.mean(Lh[sigma] <= t) - gc[q]) < tol
