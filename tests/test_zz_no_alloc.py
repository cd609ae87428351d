"""GPU: the allocation-free worker block (ds_worker_compress_sign_noalloc) against the existing
entry point (ds_worker_compress on a 1-bit context with one scale per row), to the parity bar
of the other tests (sign planes bit-exact, scales 1e-6 relative, errors 1e-6 of the row's
maximum), on two calls in a row, the second with a smaller input: the fixed array inside the
library keeps the first call's contents."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_1905_05957_amd as P
from parity_util import assert_close_rows

pytestmark = pytest.mark.gpu


def _both(n, d, dtype, device, seed, flags=0):
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    g = (torch.randn((n, d), device=device, generator=gen) * 1e-2).to(dtype)
    delta0 = torch.randn((n, d), device=device, generator=gen) * 1e-3
    ctx = P.Context("sign", n, d, grad_dtype="bf16" if dtype == torch.bfloat16 else "f32", scale_mode="whole",
                    flags=flags)
    try:
        ref_delta, ref_msg = delta0.clone(), ctx.alloc_payload(n, device)
        ctx.worker_compress(0, g, ref_delta, ref_msg)
        torch.cuda.synchronize()
    finally:
        ctx.close()
    delta = delta0.clone()
    words = torch.full((n, (d + 63) // 64), -1, dtype=torch.int64, device=device)
    scales = torch.full((n, 1), -1.0, dtype=torch.float32, device=device)
    P.ds_worker_compress_sign_noalloc(g, delta, words, scales, flags=flags)
    torch.cuda.synchronize()
    assert torch.equal(words, ref_msg.sign_words), f"sign planes differ (n={n}, d={d})"
    a, b = scales.cpu().numpy().astype(np.float64), ref_msg.scales.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(a - b) <= 1e-6 * np.abs(b)), (a, b)
    assert_close_rows(delta.cpu().numpy(), ref_delta.cpu().numpy(), f"delta (n={n}, d={d})")


def test_no_alloc_worker_block_matches_the_context_call_twice_in_a_row(gpu_device):
    _both(4, 1_000_003, torch.float32, gpu_device, seed=1)                       # 489 tiles per row
    _both(3, 70_001, torch.bfloat16, gpu_device, seed=2)                         # smaller, other dtype
    _both(2, 5_000, torch.float32, gpu_device, seed=3, flags=P.FLAG_SIGN_RMS)    # smaller again, l2 scale


def test_no_alloc_worker_block_rejects_what_does_not_fit(gpu_device):
    lib = P.load_library()
    n, d = 8, 25_557_032                                                         # 8 x 12479 tiles > 65536
    buf = torch.zeros(64, dtype=torch.float32, device=gpu_device)
    p = buf.data_ptr()
    rc = lib.ds_worker_compress_sign_noalloc(n, d, 0, 0, p, d, p, d, p, p, None)
    assert rc == 2                                                               # DS_ERR_SHAPE, nothing launched
    assert lib.ds_worker_compress_sign_noalloc(1, 64, 0, 1, p, 64, p, 64, p, p, None) == 3    # a flag it does not take
    assert lib.ds_worker_compress_sign_noalloc(1, 64, 0, 0, None, 64, p, 64, p, p, None) == 1
    torch.cuda.synchronize()
    assert float(buf.abs().sum()) == 0.0
