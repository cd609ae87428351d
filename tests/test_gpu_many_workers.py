"""GPU parity at worker counts that are not the configurations' 4, 8, 16: a single worker
(the average is the message itself), counts that are no multiple of the kernels' worker
batches (8 per load for sign planes, 64 per wavefront for sparse messages), more than 64, and a
thousand."""
import dataclasses

import pytest

import ds_workloads as W
from parity_util import Pair

pytestmark = pytest.mark.gpu


def _workloads(n):
    d = 3 * 2048 + 517
    return [
        W.Workload(f"sign_whole_n{n}", "sign", n=n, d=d, scale_mode="whole", dist="normal", sigma=1e-2, gamma=0.05),
        W.Workload(f"sign_chunk_n{n}", "sign", n=n, d=d, scale_mode="chunk", chunk=1024, dist="normal", sigma=1e-2,
                   gamma=0.05, grad_dtype="bf16", beta=0.9),
        W.Workload(f"topk_n{n}", "topk", n=n, d=d, k=d // 50, dist="laplace_outliers", sigma=1e-3, gamma=0.05),
        W.Workload(f"qsgd_n{n}", "qsgd", n=n, d=d, bucket=256, levels=15, dist="normal", sigma=1e-3, gamma=0.05),
        W.Workload(f"clip_n{n}", "clip", n=n, d=d, clip_bits=16, dist="normal", sigma=1e-2, gamma=0.05),
        W.Workload(f"rsparse_n{n}", "rsparse", n=n, d=d, keep_prob=0.6, dist="normal", sigma=1e-2, gamma=0.05),
        W.Workload(f"identity_n{n}", "identity", n=n, d=d, dist="normal", sigma=1.0, gamma=0.05),
    ]


@pytest.mark.parametrize("n", [1, 5, 13, 70, 1000])
@pytest.mark.parametrize("which", range(7), ids=["sign_whole", "sign_chunk", "topk", "qsgd", "clip", "rsparse", "identity"])
def test_worker_counts(gpu_device, n, which):
    wl = _workloads(n)[which]
    pair = Pair(wl, gpu_device)
    try:
        for t in range(2):
            pair.compared_step(t, wl.gradients(t, gpu_device))
    finally:
        pair.close()


@pytest.mark.parametrize("n", [1, 13, 70, 1000])
@pytest.mark.parametrize("which", ["sign_whole", "sign_chunk", "topk", "qsgd", "clip", "ternary"])
def test_worker_counts_plain_server(gpu_device, n, which):
    """The same counts through the kernels of a server that does not compress
    (DS_FLAG_SERVER_IDENTITY; the ternary quantiser exists in that mode only)."""
    import paper_1905_05957_amd as P
    import parity_util
    names = ["sign_whole", "sign_chunk", "topk", "qsgd", "clip"]
    if which == "ternary":
        wl = W.Workload(f"ternary_n{n}", "ternary", n=n, d=3 * 2048 + 517, dist="normal", sigma=1e-3, gamma=0.05)
        flags = P.FLAG_SERVER_IDENTITY | P.FLAG_NO_ERROR_FEEDBACK
    else:
        wl, flags = _workloads(n)[names.index(which)], P.FLAG_SERVER_IDENTITY
    parity_util.CONTEXT_FLAGS = flags
    try:
        pair = Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        for t in range(2):
            pair.compared_step(t, wl.gradients(t, gpu_device))
    finally:
        pair.close()
