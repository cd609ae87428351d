"""GPU parity: 1-bit compressor and identity, every route, against the CPU oracle."""
import dataclasses

import numpy as np
import pytest
import torch

import ds_workloads as W
import oracle as O
from parity_util import Pair, assert_close_rows

pytestmark = pytest.mark.gpu


def _run(wl, device, steps=2, sets=2, tag=""):
    pair = Pair(wl, device)
    try:
        gs = [wl.gradients(s, device) for s in range(sets)]
        for t in range(steps):
            pair.compared_step(t, gs[t % sets], tag)
    finally:
        pair.close()


def _sign_wl(d, n=3, **kw):
    base = dict(name=f"sign_d{d}", comp="sign", n=n, d=d, dist="normal", sigma=1e-2, gamma=0.05)
    base.update(kw)
    return W.Workload(**base)


@pytest.mark.parametrize("d", [1, 5, 64, 1000, 2048, 2049, 3 * 2048 + 37, 40_000 + 2])
def test_sign_whole_vector(gpu_device, d):
    _run(_sign_wl(d, scale_mode="whole"), gpu_device)


@pytest.mark.parametrize("chunk", [2048, 1024, 1920, 640, 576, 256, 320, 100, 64, 4096, 7])
@pytest.mark.parametrize("d", [6 * 2048, 5 * 2048 + 1280, 9001])
def test_sign_chunks(gpu_device, d, chunk):
    _run(_sign_wl(d, scale_mode="chunk", chunk=chunk), gpu_device)


@pytest.mark.parametrize("mode", ["whole", "chunk2048", "chunk320", "segments"])
def test_sign_rms_scale(gpu_device, mode):
    # scale = root mean square of the group (the l2 reading of the 1-bit compressor), every route
    if mode == "whole":
        wl = _sign_wl(3 * 2048 + 37, scale_mode="whole", sign_rms=True)
    elif mode == "segments":
        wl = dataclasses.replace(W.c2(d=300_001, n=3, n_seg=17, lo=64), sign_rms=True)
    else:
        wl = _sign_wl(5 * 2048 + 1280, scale_mode="chunk", chunk=int(mode[5:]), sign_rms=True)
    _run(wl, gpu_device, steps=3)


def test_sign_chunk_bf16_momentum_c5_slice(gpu_device):
    # 1/64-size slice of the large flat-gradient workload, 20 compared steps
    wl = W.c5(d=124_439_808 // 64, n=8)
    _run(wl, gpu_device, steps=20, sets=3)


def test_sign_segments_c2_scaled(gpu_device):
    # scaled-down per-segment workload: d mod 4 = 2, unaligned segment boundaries
    wl = W.c2(d=1_117_398, n=8, n_seg=62, lo=64)
    assert wl.d % 4 == 2
    _run(wl, gpu_device, steps=3, sets=2)


def test_sign_many_small_segments(gpu_device):
    off = np.concatenate([[0], np.cumsum(np.random.default_rng(3).integers(1, 90, 400))]).astype(np.int64)
    d = int(off[-1])
    wl = _sign_wl(d, scale_mode="segments", seg_offsets=off, seg_sigma=np.full(400, 1e-2), dist="segment_normal")
    _run(wl, gpu_device)


def test_sign_row_strides_and_bf16(gpu_device):
    # padded rows (stride > d) and bf16 gradients on the general route
    d, n = 5000, 4
    wl = _sign_wl(d, n=n, scale_mode="whole", grad_dtype="bf16")
    pair = Pair(wl, gpu_device)
    try:
        g_pad = torch.zeros((n, d + 24), dtype=torch.bfloat16, device=gpu_device)
        g = wl.gradients(0, gpu_device)
        g_pad[:, :d] = g
        delta_pad = torch.zeros((n, d + 8), dtype=torch.float32, device=gpu_device)
        pair.delta = delta_pad[:, :d]          # a strided view: stride(0) = d + 8
        pair.compared_step(0, g_pad[:, :d])
        pair.compared_step(1, g_pad[:, :d])
        assert not delta_pad[:, d:].any()      # padding untouched
    finally:
        pair.close()


@pytest.mark.parametrize("n", [1, 4, 8])
def test_identity_is_parallel_sgd(gpu_device, n):
    wl = W.Workload(name="identity", comp="identity", n=n, d=10_003, dist="normal", sigma=1.0, gamma=0.05)
    _run(wl, gpu_device, steps=3)


def test_identity_bf16_momentum(gpu_device):
    wl = W.Workload(name="identity_bf16", comp="identity", n=2, d=4099, grad_dtype="bf16", dist="normal",
                    sigma=1.0, gamma=0.1, beta=0.9)
    _run(wl, gpu_device, steps=3)


def test_c1_trajectory_200_steps(gpu_device):
    """Least-squares toy, free-running for 200 steps on both sides (no re-synchronisation):
    max-norm relative difference <= 1e-4 on x, delta_i, delta_s at steps 1, 50, 100, 200."""
    wl = W.c1()
    prob = W.least_squares()
    pair = Pair(wl, gpu_device)
    cfg = pair.cfg
    try:
        pair.x.zero_()
        hx = np.zeros(wl.d, np.float32)
        hd = np.zeros((wl.n, wl.d), np.float32)
        hs = np.zeros(wl.d, np.float32)
        for t in range(200):
            g_gpu = prob.gradients(pair.x.cpu().numpy(), t)
            pair.gpu_step(t, torch.from_numpy(g_gpu).to(gpu_device))
            g_ref = prob.gradients(hx, t)
            ps = O.server_aggregate_compress(cfg, t, O.worker_compress(cfg, t, g_ref, hd), hs)
            O.apply_update(cfg, ps, hx, None, wl.gamma)
            if t + 1 in (1, 50, 100, 200):
                assert_close_rows(pair.x.cpu().numpy(), hx, f"x step {t+1}", rel=1e-4)
                assert_close_rows(pair.delta.cpu().numpy(), hd, f"delta step {t+1}", rel=1e-4)
                assert_close_rows(pair.delta_s.cpu().numpy(), hs, f"delta_s step {t+1}", rel=1e-4)
        f0, fT = prob.loss(np.zeros(wl.d, np.float32)), prob.loss(pair.x.cpu().numpy())
        assert fT < 0.5 * f0
    finally:
        pair.close()


def test_same_call_twice_is_bit_identical(gpu_device):
    wl = W.c2(d=300_000, n=4, n_seg=20, lo=64)
    g = wl.gradients(0, gpu_device)
    outs = []
    for _ in range(2):
        pair = Pair(wl, gpu_device)
        pair.gpu_step(0, g)
        outs.append((pair.pw.to_numpy(), pair.ps.to_numpy(), pair.delta.cpu().numpy(), pair.x.cpu().numpy()))
        pair.close()
    for k in outs[0][0]:
        assert np.array_equal(outs[0][0][k], outs[1][0][k])
    for k in outs[0][1]:
        assert np.array_equal(outs[0][1][k], outs[1][1][k])
    assert np.array_equal(outs[0][2], outs[1][2]) and np.array_equal(outs[0][3], outs[1][3])


# ---------------------------------------------------------------------------------------
# deferred error form (ds_config_t::flags & DS_FLAG_DEFERRED_ERROR)
# ---------------------------------------------------------------------------------------
def _deferred_workloads():
    many = np.concatenate([[0], np.cumsum(np.random.default_rng(5).integers(1, 3000, 90))]).astype(np.int64)
    return [
        W.c2(d=1_117_398, n=4, n_seg=62, lo=64),
        _sign_wl(3 * 2048 + 37, scale_mode="whole"),
        _sign_wl(9001, scale_mode="chunk", chunk=320),
        _sign_wl(int(many[-1]), scale_mode="segments", seg_offsets=many, seg_sigma=np.full(90, 1e-2),
                 dist="segment_normal", grad_dtype="bf16", beta=0.9),
    ]


@pytest.mark.parametrize("wl", _deferred_workloads(), ids=lambda w: w.name + "_" + w.scale_mode)
def test_sign_deferred_error_equals_plain_form(gpu_device, wl):
    """The same steps on a plain and on a deferred context: every message and x (m) must be
    bit-identical at every step, and so must the errors once materialised -- also when the
    buffers are materialised in the middle of the run.  The plain form is what the other
    tests compare with the oracle call by call."""
    import parity_util
    import paper_1905_05957_amd as P
    plain = Pair(wl, gpu_device)
    parity_util.CONTEXT_FLAGS = P.FLAG_DEFERRED_ERROR
    try:
        lazy = Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        gs = [wl.gradients(s, gpu_device) for s in range(2)]
        for t in range(6):
            plain.gpu_step(t, gs[t % 2])
            lazy.gpu_step(t, gs[t % 2])
            for name, a in plain.pw.tensors().items():
                assert torch.equal(a, lazy.pw.tensors()[name]), f"{wl.name} t={t} worker {name}"
            for name, a in plain.ps.tensors().items():
                assert torch.equal(a, lazy.ps.tensors()[name]), f"{wl.name} t={t} server {name}"
            assert torch.equal(plain.x, lazy.x)
            if plain.m is not None:
                assert torch.equal(plain.m, lazy.m)
            if t == 2:
                lazy.ctx.materialize_error(lazy.delta, None)          # workers only; the server stays deferred
                assert torch.equal(plain.delta, lazy.delta)
                assert not torch.equal(plain.delta_s, lazy.delta_s)   # still holds v, not delta
            if t == 3:
                lazy.ctx.materialize_error(None, lazy.delta_s)
                assert torch.equal(plain.delta_s, lazy.delta_s)
        lazy.ctx.materialize_error(lazy.delta, lazy.delta_s)
        assert torch.equal(plain.delta, lazy.delta) and torch.equal(plain.delta_s, lazy.delta_s)
        lazy.ctx.materialize_error(lazy.delta, lazy.delta_s)          # a second time: nothing left to do
        assert torch.equal(plain.delta, lazy.delta) and torch.equal(plain.delta_s, lazy.delta_s)
    finally:
        plain.close()
        lazy.close()


def test_sign_deferred_error_against_oracle(gpu_device):
    """Two free-running steps in deferred form against two free-running oracle steps."""
    import parity_util
    import paper_1905_05957_amd as P
    from parity_util import host_grad, oracle_config, assert_payload_equal
    wl = W.c2(d=300_001, n=3, n_seg=17, lo=64)
    parity_util.CONTEXT_FLAGS = P.FLAG_DEFERRED_ERROR
    try:
        pair = Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        cfg = oracle_config(wl)
        h_delta = pair.delta.cpu().numpy().copy()
        h_ds = pair.delta_s.cpu().numpy().copy()
        h_x = pair.x.cpu().numpy().copy()
        for t in range(2):
            g = wl.gradients(t, gpu_device)
            pair.gpu_step(t, g)
            ref_w = O.worker_compress(cfg, t, host_grad(g), h_delta)
            ref_s = O.server_aggregate_compress(cfg, t, ref_w, h_ds)
            O.apply_update(cfg, ref_s, h_x, None, wl.gamma)
        assert_payload_equal(pair.pw.to_numpy(), ref_w, "deferred worker t=1")
        assert_payload_equal(pair.ps.to_numpy(), ref_s, "deferred server t=1")
        pair.ctx.materialize_error(pair.delta, pair.delta_s)
        assert_close_rows(pair.delta.cpu().numpy(), h_delta, "deferred delta")
        assert_close_rows(pair.delta_s.cpu().numpy(), h_ds, "deferred delta_s")
        assert_close_rows(pair.x.cpu().numpy(), h_x, "deferred x")
    finally:
        pair.close()
