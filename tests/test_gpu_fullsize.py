"""GPU parity at the full sizes of the benchmark workloads, through the same calls and launch
configuration that bench.py times.  The oracle finishes a whole step at every one of these sizes
within a minute (top-k: a full sort per row, about 6 s each), so C2, C3, C4 and C5 compare EVERY
element the kernels write, call by call from identical state, after warm-up steps that give the
error buffers a working distribution:
  C2  the whole step (8 x 11,173,962, 62 segments);
  C3  all 8 worker rows, the server pass and the update (8 x 25,557,032, k = 255,570);
  C4  all 16 worker rows (16 random streams), the server pass and the update;
  C5  all 60,762 chunks of all 8 rows, the server pass and the momentum update (8 x 124,439,808);
  X1, X2 (clipping, randomised sparsification at 8 x 25.6 M): the whole step as well.
Those comparisons go through the three calls of Algorithm 1; another test runs the call
sequence that bench.py times (worker call + the one-call server-and-update, sign per segment in
the deferred error form) beside them at full size and requires identical bits; the last one
compares the worker passes without compensation that bench.py times for C2 and C5.
"""
import pytest
import torch

import ds_workloads as W
import paper_1905_05957_amd as P
import parity_util
from parity_util import Pair

pytestmark = pytest.mark.gpu


def _full_step(wl, device, warm: int):
    pair = Pair(wl, device)
    try:
        for t in range(warm):                                   # warm-up: non-trivial error state
            pair.gpu_step(t, wl.gradients(t % 2, device))
        pair.compared_step(warm, wl.gradients(warm % 2, device))
        return pair
    except BaseException:
        pair.close()
        raise


def test_c2_full_step(gpu_device):
    _full_step(W.c2(), gpu_device, warm=1).close()


def test_c3_full_step(gpu_device):
    wl = W.c3()
    pair = _full_step(wl, gpu_device, warm=2)
    try:
        # what the message must look like, for every row, checked on the device as well
        idx = pair.pw.pairs[:, :, 0].long()
        assert idx.shape == (wl.n, wl.k) and bool((idx[:, 1:] > idx[:, :-1]).all())
        assert bool((idx >= 0).all()) and bool((idx < wl.d).all())
    finally:
        pair.close()


def test_c4_full_step(gpu_device):
    _full_step(W.c4(), gpu_device, warm=1).close()


def test_c5_full_step(gpu_device):
    wl = W.c5()
    pair = _full_step(wl, gpu_device, warm=1)
    try:
        # every decoded server element is +-scale of its chunk
        dec = torch.empty(wl.d, dtype=torch.float32, device=gpu_device)
        pair.ctx.decompress(pair.ps, 0, dec)
        sc = pair.ps.scales[0].repeat_interleave(wl.chunk)[:wl.d]
        assert torch.equal(dec.abs(), sc)
    finally:
        pair.close()


@pytest.mark.parametrize("which", ["clip16", "rsparse60"])
def test_x_full_step(gpu_device, which):
    """The two further compressors at 8 x 25.6 M: the whole step, every element."""
    _full_step(W.clip16() if which == "clip16" else W.rsparse60(), gpu_device, warm=1).close()


@pytest.mark.parametrize("which", ["c2", "c3", "c4", "c5", "clip16", "rsparse60"])
def test_timed_call_sequence_equals_three_calls(gpu_device, which):
    """Three steps at full size through the calls bench.py times against the three separate
    calls in the plain error form: messages, errors, x and m bit for bit."""
    wl = getattr(W, which)()
    three = Pair(wl, gpu_device)
    parity_util.CONTEXT_FLAGS = P.FLAG_DEFERRED_ERROR if wl.comp == "sign" else 0
    try:
        timed = Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        beta = 0.0 if wl.beta is None else wl.beta
        for t in range(3):
            g = wl.gradients(t % 2, gpu_device)
            three.gpu_step(t, g)
            timed.ctx.worker_compress(t, g, timed.delta, timed.pw)
            timed.ctx.server_aggregate_compress_update(t, timed.pw, timed.delta_s, timed.ps, timed.x, timed.m,
                                                       wl.gamma, beta)
            del g
            for side, a_p, b_p in (("worker", three.pw, timed.pw), ("server", three.ps, timed.ps)):
                for key, a in a_p.tensors().items():
                    b = b_p.tensors()[key]
                    if wl.comp == "rsparse" and key == "dense":     # packed values count as far as the kept bits say:
                        da = torch.empty(wl.d, dtype=torch.float32, device=gpu_device)      # compare what they decode to
                        db = torch.empty_like(da)
                        for r in range(a.shape[0]):
                            three.ctx.decompress(a_p, r, da)
                            timed.ctx.decompress(b_p, r, db)
                            assert torch.equal(da, db), f"{which} t={t} {side} decoded row {r}"
                        continue
                    assert torch.equal(a, b), f"{which} t={t} {side} {key}"
            assert torch.equal(three.x, timed.x), f"{which} t={t} x"
            if three.m is not None:
                assert torch.equal(three.m, timed.m), f"{which} t={t} m"
        timed.ctx.materialize_error(timed.delta, timed.delta_s)
        assert torch.equal(three.delta, timed.delta), f"{which} delta"
        assert torch.equal(three.delta_s, timed.delta_s), f"{which} delta_s"
    finally:
        three.close()
        timed.close()


@pytest.mark.parametrize("which", ["c2", "c5"])
def test_uncompensated_worker_pass_full_size(gpu_device, which):
    """bench.py also times the worker pass without compensation (DS_FLAG_NO_ERROR_FEEDBACK) at
    the full sizes of C2 and C5: every word of every row's message against the oracle (which has
    no such flag: its worker starts from a zero error that is thrown away)."""
    import numpy as np
    import oracle as O

    wl = getattr(W, which)()
    parity_util.CONTEXT_FLAGS = P.FLAG_NO_ERROR_FEEDBACK
    try:
        ctx = parity_util.gpu_context(wl)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        cfg = parity_util.oracle_config(wl)
        one = O.Config(cfg.comp, n=1, d=wl.d, grad_bf16=(wl.grad_dtype == "bf16"), group_off=wl.group_offsets(),
                       sign_rms=wl.sign_rms)
        pw = ctx.alloc_payload(wl.n, gpu_device)
        g = wl.gradients(0, gpu_device)
        ctx.worker_compress(5, g, None, pw)
        got = pw.to_numpy()
        h_g = parity_util.host_grad(g)
        del g
        for i in range(wl.n):                                     # row by row: bounded host memory
            ref = O.worker_compress(one, 5, h_g[i:i + 1], np.zeros((1, wl.d), np.float32))
            parity_util.assert_payload_equal({k: v[i:i + 1] for k, v in got.items()}, ref, f"{which} row {i}")
    finally:
        ctx.close()
