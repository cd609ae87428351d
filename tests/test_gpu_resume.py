"""GPU: a run can be stopped and resumed.  The whole state of a DoubleSqueeze run is the
caller's buffers (x, m, the worker errors, the server error) and the step counter: ten steps in
one go must equal five steps, a checkpoint of those buffers on the host, a fresh context, the
buffers copied back in, and five more steps numbered 5..9.  The context itself carries nothing
that matters (top-k keeps its previous thresholds only to centre a sampling window; a context
in deferred error form is brought to plain form with ds_materialize_error before its buffers are
read)."""
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
        ("sign_chunk_momentum", W.c5(d=2048 * 30 + 1280, n=4, n_seg=8), 0),
        ("sign_segments", W.c2(d=200_002, n=3, n_seg=12, lo=64), 0),
        ("sign_segments_deferred", W.c2(d=200_002, n=3, n_seg=12, lo=64), P.FLAG_DEFERRED_ERROR),
        ("qsgd", W.c4(d=2048 * 20 + 40, n=5), 0),
        ("qsgd_momentum", dataclasses.replace(W.c4(d=2048 * 7 + 40, n=3), beta=0.9), 0),
        ("topk", W.c3(d=300_007, n=4), 0),
        ("topk_multi_launch", W.c3(d=300_007, n=4), P.FLAG_TOPK_MULTI_LAUNCH),
        ("clip", W.clip16(d=50_001, n=3), 0),
        ("rsparse", W.rsparse60(d=50_001, n=3), 0),
        ("sign_mem_sgd", W.c5(d=2048 * 10 + 1280, n=4, n_seg=8), P.FLAG_SERVER_IDENTITY),
    ]


def _step(pair, t, g):
    wl = pair.wl
    pair.ctx.worker_compress(t, g, pair.delta, pair.pw)
    pair.ctx.server_aggregate_compress_update(t, pair.pw, pair.delta_s, pair.ps, pair.x, pair.m, wl.gamma,
                                              0.0 if wl.beta is None else wl.beta)


@pytest.mark.parametrize("name,wl,flags", _cases(), ids=[c[0] for c in _cases()])
def test_five_steps_checkpoint_five_steps_equals_ten_steps(gpu_device, name, wl, flags):
    def make():
        parity_util.CONTEXT_FLAGS = flags
        try:
            return Pair(wl, gpu_device)
        finally:
            parity_util.CONTEXT_FLAGS = 0

    grads = [wl.gradients(s, gpu_device) for s in range(3)]
    straight = make()
    first = make()
    try:
        for t in range(10):
            _step(straight, t, grads[t % 3])
        for t in range(5):
            _step(first, t, grads[t % 3])
        # checkpoint: plain-form buffers to the host, the context is thrown away
        first.ctx.materialize_error(first.delta, first.delta_s)
        torch.cuda.synchronize()
        state = {k: (None if v is None else v.cpu().clone())
                 for k, v in (("delta", first.delta), ("delta_s", first.delta_s), ("x", first.x), ("m", first.m))}
    finally:
        first.close()
    second = make()
    try:
        for k, v in state.items():
            if v is not None:
                getattr(second, k).copy_(v)
        for t in range(5, 10):
            _step(second, t, grads[t % 3])
        for pair in (straight, second):
            pair.ctx.materialize_error(pair.delta, pair.delta_s)
        torch.cuda.synchronize()
        assert torch.equal(straight.x, second.x), f"{name}: x"
        for k in ("delta", "delta_s", "m"):
            a, b = getattr(straight, k), getattr(second, k)
            assert (a is None) == (b is None)
            if a is not None:
                assert torch.equal(a, b), f"{name}: {k}"
        for key, a in straight.pw.tensors().items():
            b = second.pw.tensors()[key]
            if wl.comp == "rsparse" and key == "dense":
                continue                                  # packed values past the kept count are unspecified
            assert torch.equal(a, b), f"{name}: last worker message {key}"
    finally:
        straight.close()
        second.close()
