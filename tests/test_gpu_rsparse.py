"""GPU parity: randomised sparsification (Section 3.2 "Randomized Sparsification") against the
CPU oracle.  The kept-bit plane must be bit-exact, the packed values z/p equal, the errors
within 1e-6."""
import pytest
import torch

import ds_workloads as W
from parity_util import Pair

pytestmark = pytest.mark.gpu


def _wl(d, p, n=3, **kw):
    base = dict(name=f"rsparse_p{p}_d{d}", comp="rsparse", n=n, d=d, keep_prob=p, dist="normal", sigma=1e-2,
                gamma=0.05)
    base.update(kw)
    return W.Workload(**base)


def _run(wl, device, steps=3, t0=0):
    pair = Pair(wl, device)
    try:
        for t in range(steps):
            pair.compared_step(t0 + t, wl.gradients(t % 2, device))
    finally:
        pair.close()


@pytest.mark.parametrize("p", [0.6, 0.01, 1.0, 2.0 ** -24])
@pytest.mark.parametrize("d", [1, 7, 256, 257, 2048, 2049, 5 * 2048 + 37, 100_003])
def test_rsparse_shapes_and_probabilities(gpu_device, d, p):
    _run(_wl(d, p), gpu_device)


def test_rsparse_bf16_gradients_and_momentum(gpu_device):
    _run(_wl(50_000, 0.7, n=4, grad_dtype="bf16", beta=0.9), gpu_device, steps=4)


def test_rsparse_many_workers(gpu_device):
    _run(_wl(30_001, 0.55, n=19), gpu_device)


def test_rsparse_step_counter_high_word(gpu_device):
    _run(_wl(10_000, 0.6), gpu_device, steps=2, t0=(1 << 32) + 1)


def test_rsparse_reads_only_the_kept_bits_below_d(gpu_device):
    # a message whose pad bits are set (not what the library writes) must decode like the clean one
    wl = _wl(1000, 0.5, n=2)
    pair = Pair(wl, gpu_device)
    try:
        pair.gpu_step(0, wl.gradients(0, gpu_device))
        clean = torch.zeros(wl.d, device=gpu_device)
        pair.ctx.decompress(pair.ps, 0, clean)
        pair.ps.sign_words[0, -1] |= -1 << (wl.d % 64)            # set every bit at or past d
        dirty = torch.zeros(wl.d, device=gpu_device)
        pair.ctx.decompress(pair.ps, 0, dirty)
        assert torch.equal(clean, dirty)
    finally:
        pair.close()
