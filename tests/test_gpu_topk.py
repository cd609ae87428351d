"""GPU parity: top-k sparsification against the CPU oracle.  Index sets must be bit-exact
(ties towards the lower index, ascending order), values equal, error buffers within 1e-6."""
import numpy as np
import pytest
import torch

import ds_workloads as W
import paper_1905_05957_amd as P
import parity_util
from parity_util import Pair

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["single_launch", "multi_launch"])
def topk_route(request):
    """Every test of this module runs on both refinement routes of the library."""
    parity_util.CONTEXT_FLAGS = P.FLAG_TOPK_MULTI_LAUNCH if request.param == "multi_launch" else 0
    yield request.param
    parity_util.CONTEXT_FLAGS = 0


def _wl(d, n=3, k=None, **kw):
    base = dict(name=f"topk_d{d}", comp="topk", n=n, d=d, k=(max(1, d // 100) if k is None else k),
                dist="laplace_outliers", sigma=1e-3, gamma=0.05)
    base.update(kw)
    return W.Workload(**base)


def _run(wl, device, steps=2, sets=2, grads=None):
    pair = Pair(wl, device)
    try:
        gs = grads if grads is not None else [wl.gradients(s, device) for s in range(sets)]
        for t in range(steps):
            pair.compared_step(t, gs[t % len(gs)])
    finally:
        pair.close()


@pytest.mark.parametrize("d,k", [(1, 1), (7, 3), (2048, 20), (2049, 2049), (5 * 2048 + 37, 1), (5 * 2048 + 37, 103),
                                 (100_003, 1000), (100_003, 100_003), (40_000, 39_999)])
def test_topk_shapes(gpu_device, d, k):
    _run(_wl(d, k=k), gpu_device)


def test_topk_few_resident_workgroups(gpu_device):
    # 2 workgroups per row for 100 groups of 32768 elements: every wavefront of the single
    # launch walks several groups and the offsets run over several rounds
    parity_util.CONTEXT_KW = {"topk_max_workgroups": 6}
    try:
        _run(_wl(100 * 32768 + 999, n=3), gpu_device, steps=3)
    finally:
        parity_util.CONTEXT_KW = {}


def test_topk_single_launch_gives_up_cleanly_and_the_context_recovers(gpu_device, topk_route):
    """Failure handling of the single-launch refinement, forced from the host: without any
    polls every wait that is not satisfied at once fails, so workgroups give up; every kernel
    must still finish.  ds_status shows the failure without another call, the next step call
    reports it once and resets the context, and from then on the context works again (on the
    chain of launches) and matches the oracle."""
    if topk_route != "single_launch":
        pytest.skip("the chain of launches has no waits")
    parity_util.CONTEXT_KW = {"topk_spin_limit": -1}
    wl = _wl(1 << 20, n=4)
    try:
        pair = Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_KW = {}
    try:
        g = wl.gradients(0, gpu_device)
        assert pair.ctx.status() == 0
        failed_after = None
        for t in range(4):                            # a launch may get through: all arrivals can be in before the first poll
            pair.ctx.worker_compress(t, g, pair.delta, pair.pw)
            torch.cuda.synchronize()                  # must return: all workgroups exited
            if pair.ctx.status() != 0:
                failed_after = t
                break
        assert failed_after is not None, "no wait failed although no polls are allowed"
        assert pair.ctx.status() == 6                 # DS_ERR_DEVICE, and it stays until a call reports it
        with pytest.raises(P.DsError) as err:
            pair.ctx.worker_compress(9, g, pair.delta, pair.pw)
        assert err.value.code == 6
        torch.cuda.synchronize()
        assert pair.ctx.status() == 0
        # the failed call's outputs are undefined: start again from defined state
        pair.delta.copy_(wl.initial_delta(gpu_device))
        pair.delta_s.zero_()
        for t in range(10, 13):
            pair.compared_step(t, wl.gradients(t % 2, gpu_device))
        assert pair.ctx.status() == 0
    finally:
        pair.close()


def test_topk_all_zero_and_all_equal(gpu_device):
    d, n, k = 3 * 2048 + 5, 2, 77
    wl = _wl(d, n=n, k=k)
    zero = torch.zeros((n, d), device=gpu_device)
    _run(wl, gpu_device, steps=2, grads=[zero])           # keys all 0: indices 0..k-1
    same = torch.full((n, d), -0.5, device=gpu_device)
    same[1] = 0.25
    _run(wl, gpu_device, steps=2, grads=[same])
    pair = Pair(wl, gpu_device)
    try:
        pair.gpu_step(0, zero)
        assert pair.pw.to_numpy()["idx"].tolist() == [list(range(k))] * n
    finally:
        pair.close()


def test_topk_tie_heavy_levels(gpu_device):
    # magnitudes from 8 distinct values only: the threshold bin holds d/8 exact ties
    _run(W.c3_ties(d=1 << 20, n=4), gpu_device, steps=2)


def test_topk_pm_pairs_and_denormals(gpu_device):
    d, n = 20_000, 2
    wl = _wl(d, n=n, k=500)
    r = np.random.default_rng(0)
    base = np.repeat(r.standard_normal(d // 2), 2) * np.tile([1.0, -1.0], d // 2)
    g = np.stack([base, base[::-1] * 1e-42]).astype(np.float32)    # second row: denormals
    _run(wl, gpu_device, steps=2, grads=[torch.from_numpy(g).to(gpu_device)])


def test_topk_c3_scaled(gpu_device):
    wl = W.c3(d=25_557_032 // 16, n=8)
    _run(wl, gpu_device, steps=3)


def test_topk_bf16_momentum(gpu_device):
    _run(_wl(30_011, n=4, k=300, grad_dtype="bf16", beta=0.9, gamma=0.1), gpu_device, steps=3)


def test_topk_unaligned_rows(gpu_device):
    wl = _wl(10_002, n=3, k=100)       # d mod 4 = 2: rows 1, 2 start 8-byte aligned only
    _run(wl, gpu_device, steps=2)


def _sampled_subtiles(n_sub, ns=512):
    """The subtiles the selection kernel samples (evenly spread with a hashed jitter); kept in
    step with the kernel only to build an adversarial input for its verify-and-fall-back."""
    out = []
    for j in range(ns):
        lo, hi = (j * n_sub) // ns, ((j + 1) * n_sub) // ns
        span = hi - lo
        h = (j * 2654435761) & 0xFFFFFFFF
        out.append(lo + ((h >> 8) % span if span > 1 else 0))
    return out


def test_topk_sample_misjudges_and_falls_back(gpu_device):
    # large values exactly where the sampler looks, small ones elsewhere, k above the number
    # of large values: the sampled lower bound is too high and the exact route must take over
    d, n = 1 << 20, 2
    k = d // 5
    g = (torch.rand((n, d), device=gpu_device) * 1e-3 + 1e-4)
    g = g * (torch.randint(0, 2, (n, d), device=gpu_device) * 2 - 1)
    for s in _sampled_subtiles(d // 256):
        g[:, s * 256:(s + 1) * 256] = 1.0
    assert int((g[0].abs() >= 1.0).sum()) < k
    wl = _wl(d, n=n, k=k)
    _run(wl, gpu_device, steps=2, grads=[g])


def test_topk_outliers_far_above_the_bulk(gpu_device):
    # exactly k huge entries over a bulk 100 octaves smaller: the sampled lower bound sits in
    # the bulk, the k-th key lies far outside the windowed first-level histogram, and the
    # exact route must take over
    d, n, k = 1 << 20, 2, 2000
    gen = torch.Generator(device=gpu_device)
    gen.manual_seed(11)
    g = (1.0 + torch.rand((n, d), device=gpu_device, generator=gen)) * 1e-30
    for i in range(n):
        pos = torch.randperm(d, device=gpu_device, generator=gen)[:k]
        g[i, pos] = (1.0 + torch.rand(k, device=gpu_device, generator=gen)) * (1 if i == 0 else -1)
    _run(_wl(d, n=n, k=k), gpu_device, steps=2, grads=[g])
