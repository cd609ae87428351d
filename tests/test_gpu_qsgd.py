"""GPU parity: randomised quantisation (bucketed, Philox-driven) against the CPU oracle.
Level codes and sign planes must be bit-exact, bucket norms within 1e-6 relative."""
import numpy as np
import pytest
import torch

import ds_workloads as W
from parity_util import Pair

pytestmark = pytest.mark.gpu


def _wl(d, n=3, bucket=512, levels=15, **kw):
    base = dict(name=f"qsgd_d{d}_b{bucket}_s{levels}", comp="qsgd", n=n, d=d, bucket=bucket, levels=levels,
                dist="normal", sigma=1e-3, gamma=0.05, seed=0x5957)
    base.update(kw)
    return W.Workload(**base)


def _run(wl, device, steps=(0, 1), sets=2):
    pair = Pair(wl, device)
    try:
        gs = [wl.gradients(s, device) for s in range(sets)]
        for k, t in enumerate(steps):
            pair.compared_step(t, gs[k % sets])
    finally:
        pair.close()


@pytest.mark.parametrize("bucket", [64, 128, 256, 512, 1024, 2048])
@pytest.mark.parametrize("d", [2048 * 3, 2048 * 2 + 40, 4097, 1000, 3])
def test_qsgd_buckets_and_ragged_tails(gpu_device, bucket, d):
    _run(_wl(d, bucket=bucket), gpu_device)


@pytest.mark.parametrize("levels", [1, 4, 15])
def test_qsgd_levels(gpu_device, levels):
    _run(_wl(50_000 + 40, n=4, levels=levels), gpu_device)


def test_qsgd_step_counter_high_word(gpu_device):
    # steps 0, 1, 2 and 2^32 + 1: the step's high word reaches the Philox key
    _run(_wl(30_000, n=2), gpu_device, steps=(0, 1, 2, (1 << 32) + 1))


def test_qsgd_c4_scaled(gpu_device):
    # the 16-worker workload at 1/16 of its length (last bucket short), 3 compared steps
    wl = W.c4(d=25_557_032 // 16 + 40, n=16)
    assert wl.d % 512 != 0
    _run(wl, gpu_device, steps=(0, 1, 2))


def test_qsgd_bf16_momentum_and_zero_bucket(gpu_device):
    wl = _wl(8192, n=2, grad_dtype="bf16", beta=0.9)
    pair = Pair(wl, gpu_device)
    try:
        g = wl.gradients(0, gpu_device)
        g[:, 512:1024] = 0          # an all-zero bucket: codes 0, norm 0
        g[0, 2048:2560] = 0
        g[0, 2048 + 17] = -2.0 ** -9   # lone power of two: top level for every draw
        pair.compared_step(0, g)
        pair.compared_step(1, g)
    finally:
        pair.close()
