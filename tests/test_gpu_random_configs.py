"""GPU parity on seeded random configurations: compressor, worker count, vector length (every
residue mod 4 and mod 64, below and above one tile), groups, k, buckets, clip width, keep
probability, gradient type, momentum, step counter, row strides and the top-k route are drawn together, so
that combinations no hand-written case lists get run.  Every case is two compared steps from
identical state, to the same bar as the other parity tests."""
import os

import numpy as np
import pytest
import torch

import ds_workloads as W
import paper_1905_05957_amd as P
import parity_util
from parity_util import Pair

pytestmark = pytest.mark.gpu

CASES = int(os.environ.get("DS_RANDOM_CASES", "72"))      # a wider hunt: DS_RANDOM_CASES=2000
MAX_D = int(os.environ.get("DS_RANDOM_MAX_D", "60000"))   # and longer vectors: DS_RANDOM_MAX_D=3000000


MODE_CASES = int(os.environ.get("DS_RANDOM_MODE_CASES", "60"))
SID, NOFB = P.FLAG_SERVER_IDENTITY, P.FLAG_NO_ERROR_FEEDBACK


def _draw(case: int, modes: bool = False):
    """modes=False: Algorithm 1 itself over the six compressors; modes=True: the comparison
    algorithms of Section 5.1 (one or both mode flags set) over the compressors that have them,
    the ternary quantiser included."""
    r = np.random.default_rng((50_000 if modes else 20_000) + case)
    comp = (["sign", "topk", "qsgd", "clip", "ternary"][case % 5] if modes
            else ["sign", "topk", "qsgd", "clip", "rsparse", "identity"][case % 6])
    n = int(r.choice([1, 2, 3, 4, 7, 8, 9, 16, 17]))
    d = int(np.exp(r.uniform(np.log(1), np.log(MAX_D)))) + int(r.integers(0, 4))
    kw = dict(n=n, d=d, gamma=float(r.choice([0.05, 0.1, 1.0])), dist="normal", sigma=float(10.0 ** r.uniform(-4, 0)))
    if r.random() < 0.4:
        kw["grad_dtype"] = "bf16"
    if r.random() < 0.4:
        kw["beta"] = float(r.choice([0.5, 0.9]))
    flags = 0
    if comp == "sign":
        mode = ["whole", "chunk", "segments"][(case // 6) % 3]
        kw["scale_mode"] = mode
        if mode == "chunk":
            kw["chunk"] = int(r.choice([7, 64, 100, 128, 320, 512, 640, 1024, 1920, 2048, 4096, 5000]))
        elif mode == "segments":
            n_seg = int(r.integers(1, min(d, 40) + 1))
            cuts = np.sort(r.choice(np.arange(1, d), size=n_seg - 1, replace=False)) if n_seg > 1 else np.array([], np.int64)
            kw["seg_offsets"] = np.concatenate([[0], cuts, [d]]).astype(np.int64)
            kw["seg_sigma"] = 10.0 ** r.uniform(-4, -1, n_seg)
            kw["dist"] = "segment_normal"
        if r.random() < 0.3:
            kw["sign_rms"] = True
    elif comp == "topk":
        kw["k"] = int(r.choice([1, max(1, d // 100), max(1, d // 7), d]))
        kw["dist"] = str(r.choice(["laplace_outliers", "levels8", "normal"]))
        if r.random() < 0.3:
            flags |= P.FLAG_TOPK_MULTI_LAUNCH
    elif comp == "qsgd":
        kw["bucket"] = int(r.choice([64, 128, 256, 512, 1024, 2048]))
        kw["levels"] = int(r.choice([1, 2, 7, 15]))
    elif comp == "clip":
        kw["clip_bits"] = int(r.choice([1, 8, 15, 16, 17, 23, 24, 31]))
    elif comp == "rsparse":
        kw["keep_prob"] = float(r.choice([0.6, 0.75, 0.99, 1.0, 0.05]))
    if modes:
        if comp == "ternary":
            flags |= NOFB | SID
        elif comp == "topk":
            flags |= int(r.choice([SID, NOFB | SID]))
            if flags & NOFB:
                kw.pop("grad_dtype", None)                   # the uncompensated top-k reads fp32 gradients only
        else:
            flags |= int(r.choice([SID, NOFB, NOFB | SID]))
    first_step = int(r.choice([0, 1, 12345, (1 << 32) - 1, (1 << 40) + 3]))
    # row strides of g and of the worker errors: d (contiguous) or d plus a few elements, so
    # that rows start on 16-, 8-, 4- and (bf16) 2-byte boundaries
    pads = (int(r.choice([0, 0, 1, 2, 3, 4, 6, 9])), int(r.choice([0, 0, 1, 2, 3, 4, 6, 9])))
    return W.Workload(f"random_{case}_{comp}", comp, **kw), flags, first_step, pads


def _with_row_stride(t: torch.Tensor, pad: int) -> torch.Tensor:
    if pad == 0:
        return t
    buf = torch.zeros((t.shape[0], t.shape[1] + pad), dtype=t.dtype, device=t.device)
    buf[:, :t.shape[1]] = t
    return buf[:, :t.shape[1]]


def _run(gpu_device, wl, flags, t0, pad_g, pad_delta):
    parity_util.CONTEXT_FLAGS = flags
    try:
        pair = Pair(wl, gpu_device)
    finally:
        parity_util.CONTEXT_FLAGS = 0
    try:
        if pair.delta is not None:
            pair.delta = _with_row_stride(pair.delta, pad_delta)
        for t in range(2):
            pair.compared_step(t0 + t, _with_row_stride(wl.gradients(t, gpu_device), pad_g),
                               tag=f" flags={flags} pads={pad_g},{pad_delta}")
    finally:
        pair.close()


@pytest.mark.parametrize("case", range(CASES))
def test_random_configuration(gpu_device, case):
    wl, flags, t0, (pad_g, pad_delta) = _draw(case)
    _run(gpu_device, wl, flags, t0, pad_g, pad_delta)


@pytest.mark.parametrize("case", range(MODE_CASES))
def test_random_mode_configuration(gpu_device, case):
    wl, flags, t0, (pad_g, pad_delta) = _draw(case, modes=True)
    _run(gpu_device, wl, flags, t0, pad_g, pad_delta)
