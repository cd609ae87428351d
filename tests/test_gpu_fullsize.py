"""GPU parity at the full sizes of the benchmark workloads, through the same calls and launch
configuration that bench.py times.  The oracle is too slow for whole steps at these sizes,
so each test compares what it can compute exactly in seconds:
  C5  a random sample of whole 2048-element chunks (chunks are independent under a per-chunk
      scale), gathered into a smaller problem with the same structure;
  C4  two whole worker rows (first and last stream), the whole server pass and update;
  C3  one whole worker row, the whole server pass and update, plus properties of every row;
  C2  the whole step;
  X1, X2 (clipping, randomised sparsification at 8 x 25.6 M)  as C4.
Those comparisons go through the three calls of Algorithm 1; the last test runs the call
sequence that bench.py times (worker call + the one-call server-and-update, sign per segment in
the deferred error form) beside them at full size and requires identical bits.
"""
import numpy as np
import pytest
import torch

import ds_workloads as W
import oracle as O
import paper_1905_05957_amd as P
import parity_util
from parity_util import Pair, assert_close_rows, assert_payload_equal, host_grad, oracle_config

pytestmark = pytest.mark.gpu


def test_c2_full_step(gpu_device):
    wl = W.c2()
    pair = Pair(wl, gpu_device)
    try:
        pair.gpu_step(0, wl.gradients(0, gpu_device))          # warm-up: non-trivial state
        pair.compared_step(1, wl.gradients(1, gpu_device))
    finally:
        pair.close()


def test_c5_sampled_chunks(gpu_device):
    wl = W.c5()
    n, d, chunk = wl.n, wl.d, wl.chunk
    S = (d + chunk - 1) // chunk
    rng = np.random.default_rng(7)
    chunks = np.unique(np.concatenate([rng.choice(S - 1, 1500, replace=False), [0, S - 2, S - 1]]))
    elem = np.concatenate([np.arange(c * chunk, min((c + 1) * chunk, d)) for c in chunks])
    words = np.concatenate([np.arange(c * chunk // 64, (min((c + 1) * chunk, d) + 63) // 64) for c in chunks])
    e_t = torch.from_numpy(elem).to(gpu_device)
    w_t = torch.from_numpy(words).to(gpu_device)
    c_t = torch.from_numpy(chunks).to(gpu_device)
    d_sub = len(elem)
    cfg = O.Config(O.SIGN, n=n, d=d_sub, grad_bf16=True, group_off=O.chunk_offsets(d_sub, chunk))
    assert cfg.n_groups == len(chunks) and cfg.n_words == len(words)

    pair = Pair(wl, gpu_device)
    try:
        pair.gpu_step(0, wl.gradients(0, gpu_device))
        g = wl.gradients(1, gpu_device)
        t = 1
        take = lambda a: a[..., e_t].contiguous()
        h_g = host_grad(take(g))
        h_delta, h_ds = take(pair.delta).cpu().numpy(), take(pair.delta_s).cpu().numpy()
        h_x, h_m = take(pair.x).cpu().numpy(), take(pair.m).cpu().numpy()
        pair.gpu_step(t, g)
        sub = lambda p: {"sign_words": p.sign_words[:, w_t].cpu().numpy().view(np.uint64),
                         "scales": p.scales[:, c_t].cpu().numpy()}
        gpu_pw, gpu_ps = sub(pair.pw), sub(pair.ps)
        ref_pw = O.worker_compress(cfg, t, h_g, h_delta)
        assert_payload_equal(gpu_pw, ref_pw, "C5 worker payload (sampled chunks)")
        assert_close_rows(take(pair.delta).cpu().numpy(), h_delta, "C5 delta")
        ref_ps = O.server_aggregate_compress(cfg, t, gpu_pw, h_ds)
        assert_payload_equal(gpu_ps, ref_ps, "C5 server payload (sampled chunks)")
        assert_close_rows(take(pair.delta_s).cpu().numpy(), h_ds, "C5 delta_s")
        O.apply_update(cfg, gpu_ps, h_x, h_m, wl.gamma, wl.beta)
        assert_close_rows(take(pair.x).cpu().numpy(), h_x, "C5 x")
        assert_close_rows(take(pair.m).cpu().numpy(), h_m, "C5 m")
        # property at full size: every decoded server element is +-scale of its chunk
        dec = torch.empty(d, dtype=torch.float32, device=gpu_device)
        pair.ctx.decompress(pair.ps, 0, dec)
        sc = pair.ps.scales[0].repeat_interleave(chunk)[:d]
        assert torch.equal(dec.abs(), sc)
    finally:
        pair.close()


def test_c4_rows_and_server(gpu_device):
    wl = W.c4()
    n, d = wl.n, wl.d
    cfg = oracle_config(wl)
    one = O.Config(O.QSGD, n=1, d=d, bucket=wl.bucket, levels=wl.levels, seed=wl.seed)
    pair = Pair(wl, gpu_device)
    try:
        pair.gpu_step(0, wl.gradients(0, gpu_device))
        g = wl.gradients(1, gpu_device)
        t = 1
        rows = [0, n - 1]
        v = {r: (g[r] + pair.delta[r]).cpu().numpy() for r in rows}      # one fp32 add per element
        h_ds = pair.delta_s.cpu().numpy().copy()
        h_x = pair.x.cpu().numpy().copy()
        pair.gpu_step(t, g)
        gpu_pw, gpu_ps = pair.pw.to_numpy(), pair.ps.to_numpy()
        for r in rows:
            ref = O.encode(one, t, r, v[r])                              # stream = worker index
            got = {k: a[r:r + 1] for k, a in gpu_pw.items()}
            assert_payload_equal(got, ref, f"C4 worker row {r}")
            assert_close_rows(pair.delta[r].cpu().numpy(), v[r] - O.decode(one, ref), f"C4 delta row {r}")
        ref_ps = O.server_aggregate_compress(cfg, t, gpu_pw, h_ds)
        assert_payload_equal(gpu_ps, ref_ps, "C4 server payload")
        assert_close_rows(pair.delta_s.cpu().numpy(), h_ds, "C4 delta_s")
        O.apply_update(cfg, gpu_ps, h_x, None, wl.gamma)
        assert_close_rows(pair.x.cpu().numpy(), h_x, "C4 x")
    finally:
        pair.close()


def test_c3_row_server_and_properties(gpu_device):
    wl = W.c3()
    n, d, k = wl.n, wl.d, wl.k
    cfg = oracle_config(wl)
    one = O.Config(O.TOPK, n=1, d=d, k=k)
    pair = Pair(wl, gpu_device)
    try:
        for t in range(2):                                               # warm-up: errors build up
            pair.gpu_step(t, wl.gradients(t, gpu_device))
        g = wl.gradients(0, gpu_device)
        t = 2
        v_all = g + pair.delta
        h_ds = pair.delta_s.cpu().numpy().copy()
        h_x = pair.x.cpu().numpy().copy()
        pair.gpu_step(t, g)
        gpu_pw, gpu_ps = pair.pw.to_numpy(), pair.ps.to_numpy()
        r = 3
        ref = O.encode(one, t, 0, v_all[r].cpu().numpy())
        assert_payload_equal({k_: a[r:r + 1] for k_, a in gpu_pw.items()}, ref, f"C3 worker row {r}")
        # properties of every row, checked on the device
        idx = pair.pw.pairs[:, :, 0].long()
        val = pair.pw.pairs[:, :, 1].contiguous().view(torch.float32)
        assert idx.shape == (n, k) and bool((idx[:, 1:] > idx[:, :-1]).all())
        assert bool((idx >= 0).all()) and bool((idx < d).all())
        assert torch.equal(val, torch.gather(v_all, 1, idx))
        kept = torch.zeros((n, d), dtype=torch.bool, device=gpu_device)
        kept.scatter_(1, idx, True)
        assert torch.equal(pair.delta, torch.where(kept, torch.zeros_like(v_all), v_all))
        mag = v_all.abs()
        floor_kept = torch.where(kept, mag, torch.full_like(mag, float("inf"))).amin(1)
        ceil_rest = torch.where(kept, torch.zeros_like(mag), mag).amax(1)
        assert bool((floor_kept >= ceil_rest).all())
        del kept, mag, v_all
        ref_ps = O.server_aggregate_compress(cfg, t, gpu_pw, h_ds)
        assert_payload_equal(gpu_ps, ref_ps, "C3 server payload")
        assert_close_rows(pair.delta_s.cpu().numpy(), h_ds, "C3 delta_s")
        O.apply_update(cfg, gpu_ps, h_x, None, wl.gamma)
        assert_close_rows(pair.x.cpu().numpy(), h_x, "C3 x")
    finally:
        pair.close()


@pytest.mark.parametrize("which", ["clip16", "rsparse60"])
def test_x_rows_and_server(gpu_device, which):
    """The two further compressors at 8 x 25.6 M: two whole worker rows (first and last stream),
    the whole server pass and the update."""
    from parity_util import keep_prob_24
    wl = W.clip16() if which == "clip16" else W.rsparse60()
    n, d = wl.n, wl.d
    cfg = oracle_config(wl)
    comp = O.CLIP if which == "clip16" else O.RSPARSE
    pair = Pair(wl, gpu_device)
    try:
        pair.gpu_step(0, wl.gradients(0, gpu_device))
        g = wl.gradients(1, gpu_device)
        t = 1
        rows = [0, n - 1]
        v = {r: (g[r] + pair.delta[r]).cpu().numpy() for r in rows}      # one fp32 add per element
        h_ds = pair.delta_s.cpu().numpy().copy()
        h_x = pair.x.cpu().numpy().copy()
        pair.gpu_step(t, g)
        gpu_pw, gpu_ps = pair.pw.to_numpy(), pair.ps.to_numpy()
        one = O.Config(comp, n=1, d=d, seed=wl.seed, clip_bits=wl.clip_bits, keep_prob=keep_prob_24(wl.keep_prob))
        for r in rows:
            ref = O.encode(one, t, r, v[r])                              # stream = worker index
            got = {k: a[r:r + 1] for k, a in gpu_pw.items()}
            assert_payload_equal(got, ref, f"{which} worker row {r}")
            assert_close_rows(pair.delta[r].cpu().numpy(), v[r] - O.decode(one, ref), f"{which} delta row {r}")
        ref_ps = O.server_aggregate_compress(cfg, t, gpu_pw, h_ds)
        assert_payload_equal(gpu_ps, ref_ps, f"{which} server payload")
        assert_close_rows(pair.delta_s.cpu().numpy(), h_ds, f"{which} delta_s")
        O.apply_update(cfg, gpu_ps, h_x, None, wl.gamma)
        assert_close_rows(pair.x.cpu().numpy(), h_x, f"{which} x")
    finally:
        pair.close()


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
