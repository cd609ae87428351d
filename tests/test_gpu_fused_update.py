"""GPU: ds_server_aggregate_compress_update must give, bit for bit, what the server call
followed by the update call gives (those two are compared with the oracle elsewhere)."""
import dataclasses

import pytest
import torch

import ds_workloads as W
import paper_1905_05957_amd as P
import parity_util
from parity_util import Pair

pytestmark = pytest.mark.gpu


def _cases():
    return [
        ("topk", W.c3(d=300_007, n=4), 0),
        ("topk_multi_launch", W.c3(d=300_007, n=4), P.FLAG_TOPK_MULTI_LAUNCH),
        ("topk_momentum", dataclasses.replace(W.c3(d=100_003, n=3), beta=0.9), 0),
        ("sign_chunk_momentum", W.c5(d=2048 * 30 + 1280, n=4, n_seg=8), 0),
        ("sign_chunk_plain_sgd_odd_length", dataclasses.replace(W.c5(d=2048 * 31 + 1283, n=3, n_seg=8), beta=None), 0),
        ("sign_chunk_rms_9_workers", dataclasses.replace(W.c5(d=2048 * 9 + 130, n=9, n_seg=4), sign_rms=True), 0),
        ("qsgd_momentum_odd_length", dataclasses.replace(W.c4(d=2048 * 11 + 37, n=3), beta=0.8), 0),
        ("sign_segments_deferred", W.c2(d=200_002, n=3, n_seg=12, lo=64), P.FLAG_DEFERRED_ERROR),
        ("qsgd", W.c4(d=2048 * 20 + 40, n=5), 0),
        ("clip", W.clip16(d=50_001, n=3), 0),
        ("rsparse", W.rsparse60(d=50_001, n=3), 0),
        ("identity", W.Workload("identity", "identity", n=3, d=10_001, gamma=0.05), 0),
    ]


@pytest.mark.parametrize("name,wl,flags", _cases(), ids=[c[0] for c in _cases()])
def test_fused_server_update_equals_the_two_calls(gpu_device, name, wl, flags):
    parity_util.CONTEXT_FLAGS = flags
    try:
        two, one = Pair(wl, gpu_device), Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        beta = 0.0 if wl.beta is None else wl.beta
        for t in range(4):
            g = wl.gradients(t % 2, gpu_device)
            two.gpu_step(t, g)
            one.ctx.worker_compress(t, g, one.delta, one.pw)
            one.ctx.server_aggregate_compress_update(t, one.pw, one.delta_s, one.ps, one.x, one.m, wl.gamma, beta)
            for key, a in two.ps.tensors().items():
                b = one.ps.tensors()[key]
                if name == "rsparse" and key == "dense":         # packed values: as far as the kept bits say
                    cnt = int(sum(bin(int(w) & 0xFFFFFFFFFFFFFFFF).count("1") for w in two.ps.sign_words[0].tolist()))
                    a, b = a[0, :cnt], b[0, :cnt]
                assert torch.equal(a, b), f"{name} t={t} server {key}"
            assert torch.equal(two.x, one.x), f"{name} t={t} x"
            if two.m is not None:
                assert torch.equal(two.m, one.m), f"{name} t={t} m"
            if not (flags & P.FLAG_DEFERRED_ERROR):
                assert torch.equal(two.delta_s, one.delta_s), f"{name} t={t} delta_s"
        two.ctx.materialize_error(two.delta, two.delta_s)
        one.ctx.materialize_error(one.delta, one.delta_s)
        assert torch.equal(two.delta_s, one.delta_s) and torch.equal(two.delta, one.delta)
    finally:
        two.close()
        one.close()
