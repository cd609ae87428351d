"""GPU parity: clipping of low bits (Section 3.2 "Clipping") against the CPU oracle.  The
message bytes must be bit-exact; the error v - Q[v] is exact in fp32, so errors agree too."""
import pytest
import torch

import ds_workloads as W
from parity_util import Pair

pytestmark = pytest.mark.gpu


def _wl(d, bits, n=3, **kw):
    base = dict(name=f"clip{bits}_d{d}", comp="clip", n=n, d=d, clip_bits=bits, dist="normal", sigma=1e-2, gamma=0.05)
    base.update(kw)
    return W.Workload(**base)


def _run(wl, device, steps=2):
    pair = Pair(wl, device)
    try:
        for t in range(steps):
            pair.compared_step(t, wl.gradients(t % 2, device))
    finally:
        pair.close()


@pytest.mark.parametrize("bits", [1, 8, 16, 20, 24, 31])
@pytest.mark.parametrize("d", [1, 7, 2048, 2049, 5 * 2048 + 37, 100_003])
def test_clip_shapes_and_widths(gpu_device, d, bits):
    _run(_wl(d, bits), gpu_device)


def test_clip_bf16_gradients_and_momentum(gpu_device):
    _run(_wl(50_000, 16, n=4, grad_dtype="bf16", beta=0.9), gpu_device, steps=3)


def test_clip_many_workers_and_extreme_values(gpu_device):
    wl = _wl(30_001, 16, n=19)
    pair = Pair(wl, gpu_device)
    try:
        g = wl.gradients(0, gpu_device)
        g[:, :8] = torch.tensor([0.0, -0.0, 1e-40, -3e-42, 3.0e38, -1.17549435e-38, 1.0, -1.0], device=gpu_device)
        pair.compared_step(0, g)
        pair.compared_step(1, g)
    finally:
        pair.close()
