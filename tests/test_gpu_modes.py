"""GPU parity of the two mode flags that turn Algorithm 1 into the comparison algorithms of
Section 5.1: DS_FLAG_SERVER_IDENTITY (the server does not compress: "MEM-SGD") and
DS_FLAG_NO_ERROR_FEEDBACK (no compensation: "Top-k SGD", "QSGD"), and of the ternary quantiser
of the paper's QSGD comparison system, which is built for that mode.  The oracle has no such
flags: every expected value is a composition of its plain functions (parity_util.Pair)."""
import dataclasses

import numpy as np
import pytest
import torch

import ds_workloads as W
import paper_1905_05957_amd as P
import parity_util
from parity_util import Pair

pytestmark = pytest.mark.gpu

SID, NOFB = P.FLAG_SERVER_IDENTITY, P.FLAG_NO_ERROR_FEEDBACK


def _ternary(d, n, grad_dtype="f32"):
    return W.Workload(f"ternary_d{d}", "ternary", n=n, d=d, dist="normal", sigma=1e-3, gamma=0.05, grad_dtype=grad_dtype)


def _cases():
    c = []
    for name, flags in (("mem_sgd", SID), ("uncompensated", NOFB), ("uncompensated_plain_server", NOFB | SID)):
        c += [
            (f"sign_chunk_{name}", W.c5(d=2048 * 30 + 1280, n=4, n_seg=8), flags),
            (f"sign_chunk_640_{name}", dataclasses.replace(W.c5(d=640 * 53 + 200, n=3, n_seg=8), chunk=640, beta=None), flags),
            (f"sign_segments_{name}", W.c2(d=200_002, n=3, n_seg=12, lo=64), flags),
            (f"sign_whole_{name}", W.c1(), flags),
            (f"qsgd_{name}", W.c4(d=2048 * 20 + 40, n=5), flags),
            (f"clip_{name}", W.clip16(d=50_001, n=3), flags),
        ]
    c += [
        ("topk_mem_sgd", W.c3(d=300_007, n=4), SID),
        ("topk_mem_sgd_multi_launch", W.c3(d=300_007, n=4), SID | P.FLAG_TOPK_MULTI_LAUNCH),
        ("topk_mem_sgd_bf16_momentum", dataclasses.replace(W.c3(d=100_003, n=3), grad_dtype="bf16", beta=0.9), SID),
        ("topk_sgd", W.c3(d=300_007, n=4), NOFB | SID),
        ("topk_sgd_multi_launch", W.c3(d=300_007, n=4), NOFB | SID | P.FLAG_TOPK_MULTI_LAUNCH),
        ("topk_sgd_17_workers", W.c3(d=40_001, n=17), NOFB | SID),
        ("ternary_qsgd", _ternary(2048 * 37 + 77, 4), NOFB | SID),
        ("ternary_qsgd_bf16", _ternary(50_002, 3, "bf16"), NOFB | SID),
        ("ternary_qsgd_tiny", _ternary(7, 2), NOFB | SID),
    ]
    return c


@pytest.mark.parametrize("name,wl,flags", _cases(), ids=[c[0] for c in _cases()])
def test_mode_flags_compared_steps(gpu_device, name, wl, flags):
    parity_util.CONTEXT_FLAGS = flags
    try:
        pair = Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        for t in range(3):
            pair.compared_step(t, wl.gradients(t % 2, gpu_device))
    finally:
        pair.close()


def test_topk_sgd_exact_route_reads_the_gradient(gpu_device):
    """Without compensation there is no buffer that holds v: when the sampled bound misjudges,
    the second look of the exact route reads the gradient itself (and writes nothing)."""
    d, n, k = 1 << 20, 2, 2000
    gen = torch.Generator(device=gpu_device)
    gen.manual_seed(11)
    g = (1.0 + torch.rand((n, d), device=gpu_device, generator=gen)) * 1e-30
    for i in range(n):
        pos = torch.randperm(d, device=gpu_device, generator=gen)[:k]
        g[i, pos] = (1.0 + torch.rand(k, device=gpu_device, generator=gen)) * (1 if i == 0 else -1)
    keep = g.clone()
    wl = W.Workload("topk_sgd_outliers", "topk", n=n, d=d, k=k, dist="laplace_outliers", sigma=1e-3, gamma=0.05)
    for flags in (NOFB | SID, NOFB | SID | P.FLAG_TOPK_MULTI_LAUNCH):
        parity_util.CONTEXT_FLAGS = flags
        try:
            pair = Pair(wl, gpu_device)
        finally:
            parity_util.CONTEXT_FLAGS = 0
        try:
            for t in range(2):
                pair.compared_step(t, g)
            assert torch.equal(g, keep)                          # the input is read only
        finally:
            pair.close()


def test_fused_server_update_equals_the_two_calls_in_every_mode(gpu_device):
    for name, wl, flags in _cases():
        parity_util.CONTEXT_FLAGS = flags
        try:
            two, one = Pair(wl, gpu_device), Pair(wl, gpu_device)
        finally:
            parity_util.CONTEXT_FLAGS = 0
        try:
            beta = 0.0 if wl.beta is None else wl.beta
            for t in range(3):
                g = wl.gradients(t % 2, gpu_device)
                two.gpu_step(t, g)
                one.ctx.worker_compress(t, g, one.delta, one.pw)
                # under SERVER_IDENTITY the average need not be written at all (third step)
                out = None if (one.sid and t == 2) else one.ps
                one.ctx.server_aggregate_compress_update(t, one.pw, one.delta_s, out, one.x, one.m, wl.gamma, beta)
                assert torch.equal(two.x, one.x), f"{name} t={t} x"
                if two.m is not None:
                    assert torch.equal(two.m, one.m), f"{name} t={t} m"
                if out is not None:
                    for key, a in two.ps.tensors().items():
                        assert torch.equal(a, one.ps.tensors()[key]), f"{name} t={t} server {key}"
        finally:
            two.close()
            one.close()


def test_unsupported_combinations_are_refused_at_create(gpu_device):
    def code(**kw):
        with pytest.raises(P.DsError) as err:
            P.Context(**kw)
        return err.value.code

    assert code(comp="ternary", n=2, d=100, flags=0) == 5                       # built for the comparison system's mode only
    assert code(comp="ternary", n=2, d=100, flags=NOFB) == 5
    assert code(comp="topk", n=2, d=100, k=3, flags=NOFB) == 5                  # needs the plain server
    assert code(comp="topk", n=2, d=100, k=3, flags=NOFB | SID, grad_dtype="bf16") == 5
    assert code(comp="rsparse", n=2, d=100, keep_prob=0.6, flags=SID) == 5
    assert code(comp="identity", n=2, d=100, flags=NOFB) == 5
