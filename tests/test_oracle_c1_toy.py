"""The least-squares toy (workload C1) run end to end on the CPU oracle.

Pins the qualitative claim of Section 5.2 ("1-bit compression"): with error compensation on
both passes, 1-bit DoubleSqueeze converges like uncompressed SGD per iteration, while 1-bit
compression without compensation is clearly worse.
"""
import numpy as np

import ds_workloads as W
import oracle as O


def run(cfg, prob, steps, gamma, compensate=True):
    n, d = cfg.n, cfg.d
    x = np.zeros(d, np.float32)
    delta = np.zeros((n, d), np.float32)
    delta_s = np.zeros(d, np.float32)
    losses = [prob.loss(x)]
    for t in range(steps):
        g = prob.gradients(x, t)
        if not compensate:            # drop the memory: plain compressed SGD on both passes
            delta[:] = 0
            delta_s[:] = 0
        pw = O.worker_compress(cfg, t, g, delta)
        ps = O.server_aggregate_compress(cfg, t, pw, delta_s)
        O.apply_update(cfg, ps, x, None, gamma)
        losses.append(prob.loss(x))
    return x, np.array(losses), delta, delta_s


def test_c1_sign_doublesqueeze_tracks_sgd():
    wl = W.c1()
    prob = W.least_squares()
    sign = O.Config(O.SIGN, n=wl.n, d=wl.d)
    ident = O.Config(O.IDENTITY, n=wl.n, d=wl.d)
    _, f_ds, delta, delta_s = run(sign, prob, 200, wl.gamma)
    _, f_sgd, _, _ = run(ident, prob, 200, wl.gamma)
    _, f_nc, _, _ = run(sign, prob, 200, wl.gamma, compensate=False)
    assert f_sgd[-1] < 0.5 * f_sgd[0]
    assert f_ds[-1] < 0.5 * f_ds[0]
    assert abs(f_ds[-1] - f_sgd[-1]) / f_sgd[-1] < 0.05
    # without compensation the same compressor lags behind
    assert f_nc[-1] > f_ds[-1] * 1.02
    # error buffers stay bounded (Assumption 1.3): comparable to a gradient, not growing
    gnorm = np.linalg.norm(prob.gradients(np.zeros(wl.d, np.float32), 0), axis=1).max()
    assert np.linalg.norm(delta, axis=1).max() < 10 * gnorm
    assert np.linalg.norm(delta_s) < 10 * gnorm
