"""GPU: the step calls only enqueue kernels and keep no host-side state that changes from call
to call, so a captured step can be replayed.  Every replay is compared with the same step run
eagerly on a second context (the eager path is what the other tests compare with the oracle)."""
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
        ("topk", W.c3(d=400_003, n=4), 0),
        ("topk_multi_launch", W.c3(d=400_003, n=4), P.FLAG_TOPK_MULTI_LAUNCH),
        ("sign_chunk_momentum", W.c5(d=2048 * 40 + 1280, n=4, n_seg=8), 0),
        ("sign_segments_deferred", W.c2(d=200_002, n=3, n_seg=12, lo=64), P.FLAG_DEFERRED_ERROR),
        ("qsgd", W.c4(d=2048 * 20 + 40, n=5), 0),
        ("clip", W.clip16(d=50_001, n=3), 0),
        ("rsparse", W.rsparse60(d=50_001, n=3), 0),
    ]


@pytest.mark.parametrize("name,wl,flags", _cases(), ids=[c[0] for c in _cases()])
def test_captured_step_replays_like_the_eager_step(gpu_device, name, wl, flags):
    parity_util.CONTEXT_FLAGS = flags
    try:
        eager, graphed = Pair(wl, gpu_device), Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        beta = 0.0 if wl.beta is None else wl.beta
        grads = [wl.gradients(s, gpu_device) for s in range(2)]

        def step(pair, t, g):
            pair.ctx.worker_compress(t, g, pair.delta, pair.pw)
            pair.ctx.server_aggregate_compress_update(t, pair.pw, pair.delta_s, pair.ps, pair.x, pair.m, wl.gamma, beta)

        for pair in (eager, graphed):                      # one eager step first: steady state of both contexts
            step(pair, 0, grads[0])
        torch.cuda.synchronize()
        static_g = grads[1].clone()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step(graphed, 1, static_g)                     # the step counter is baked in: every replay draws like step 1
        torch.cuda.synchronize()
        for r in range(4):
            g = grads[(r + 1) % 2]
            static_g.copy_(g)
            graph.replay()
            step(eager, 1, g)
            torch.cuda.synchronize()
            for key, a in eager.ps.tensors().items():
                b = graphed.ps.tensors()[key]
                if name == "rsparse" and key == "dense":
                    cnt = sum(bin(int(w) & 0xFFFFFFFFFFFFFFFF).count("1") for w in eager.ps.sign_words[0].tolist())
                    a, b = a[0, :cnt], b[0, :cnt]
                assert torch.equal(a, b), f"{name} replay {r} server {key}"
            assert torch.equal(eager.x, graphed.x), f"{name} replay {r} x"
            if eager.m is not None:
                assert torch.equal(eager.m, graphed.m)
        for pair in (eager, graphed):
            pair.ctx.materialize_error(pair.delta, pair.delta_s)
        assert torch.equal(eager.delta, graphed.delta) and torch.equal(eager.delta_s, graphed.delta_s)
    finally:
        eager.close()
        graphed.close()
