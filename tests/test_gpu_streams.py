"""GPU: contexts keep no state outside themselves, so two of them can run their steps on two
streams at the same time; each must produce what it produces alone.  Top-k runs on both of its
refinement routes: in the single launch a workgroup waits only for workgroups of its own row,
which the dispatch order makes resident together, so two such launches that share the device
take turns row by row (and every wait is bounded, so a violated assumption would show as an
error, never as a hang)."""
import pytest
import torch

import ds_workloads as W
import paper_1905_05957_amd as P
import parity_util
from parity_util import Pair

pytestmark = pytest.mark.gpu


def _cases():
    return [
        ("sign_chunk", W.c5(d=2048 * 300 + 1280, n=4, n_seg=8), 0),
        ("sign_segments_deferred", W.c2(d=600_002, n=3, n_seg=12, lo=64), P.FLAG_DEFERRED_ERROR),
        ("qsgd", W.c4(d=2048 * 200 + 40, n=5), 0),
        ("topk_chain", W.c3(d=700_007, n=4), P.FLAG_TOPK_MULTI_LAUNCH),
        ("topk_single_launch", W.c3(d=700_007, n=4), 0),
        ("topk_single_launch_64_rows", W.c3(d=2_000_003, n=64), 0),    # 512 waiting workgroups per launch
        ("rsparse", W.rsparse60(d=500_001, n=3), 0),
    ]


@pytest.mark.parametrize("name,wl,flags", _cases(), ids=[c[0] for c in _cases()])
def test_two_contexts_on_two_streams(gpu_device, name, wl, flags):
    parity_util.CONTEXT_FLAGS = flags
    try:
        alone, a, b = Pair(wl, gpu_device), Pair(wl, gpu_device), Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        grads = [wl.gradients(t, gpu_device) for t in range(2)]
        beta = 0.0 if wl.beta is None else wl.beta
        for t in range(4):
            alone.gpu_step(t, grads[t % 2])
        torch.cuda.synchronize()
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        for t in range(4):
            for pair, s in zip((a, b), streams):
                pair.ctx.worker_compress(t, grads[t % 2], pair.delta, pair.pw, stream=s)
                pair.ctx.server_aggregate_compress(t, pair.pw, pair.delta_s, pair.ps, stream=s)
                pair.ctx.apply_update(pair.ps, pair.x, pair.m, wl.gamma, beta, stream=s)
        torch.cuda.synchronize()
        for pair in (alone, a, b):
            pair.ctx.materialize_error(pair.delta, pair.delta_s)
        torch.cuda.synchronize()
        for pair in (alone, a, b):
            assert pair.ctx.status() == 0
        for pair in (a, b):
            assert torch.equal(pair.x, alone.x) and torch.equal(pair.delta, alone.delta)
            assert torch.equal(pair.delta_s, alone.delta_s)
            if alone.m is not None:
                assert torch.equal(pair.m, alone.m)
    finally:
        for p in (alone, a, b):
            p.close()
