"""GPU: the Python binding hands bare pointers to the library, so it refuses buffers that do not
have the device, element type, shape or layout the library will assume -- before anything is
launched -- and the context keeps working afterwards."""
import pytest
import torch

import paper_1905_05957_amd as P

pytestmark = pytest.mark.gpu


def test_wrong_buffers_are_refused_before_any_launch(gpu_device):
    dev, n, d = gpu_device, 3, 5000
    ctx = P.Context("sign", n, d, scale_mode="chunk", chunk=1024)
    other = P.Context("topk", n, d, k=50)
    try:
        g = torch.randn(n, d, device=dev) * 1e-2
        delta = torch.zeros(n, d, device=dev)
        delta_s = torch.zeros(d, device=dev)
        x = torch.zeros(d, device=dev)
        pw, ps = ctx.alloc_payload(n, dev), ctx.alloc_payload(1, dev)
        bad = [
            lambda: ctx.worker_compress(0, g.cpu(), delta, pw),                       # host memory
            lambda: ctx.worker_compress(0, g.double(), delta, pw),                    # element type
            lambda: ctx.worker_compress(0, g.bfloat16(), delta, pw),                  # not the configured gradient type
            lambda: ctx.worker_compress(0, g[:, :-1], delta, pw),                     # shape
            lambda: ctx.worker_compress(0, g.t().contiguous().t(), delta, pw),        # element stride
            lambda: ctx.worker_compress(0, g, delta[:2], pw),                         # rows
            lambda: ctx.worker_compress(0, g, delta, ps),                             # one message where n are needed
            lambda: ctx.worker_compress(0, g, delta, other.alloc_payload(n, dev)),    # another compressor's buffers
            lambda: ctx.server_aggregate_compress(0, pw, delta_s[:-1], ps),
            lambda: ctx.server_aggregate_compress(0, ps, delta_s, ps),
            lambda: ctx.apply_update(ps, x.double(), None, 0.1),
            lambda: ctx.apply_update(ps, x, x[:-1], 0.1, 0.9),
            lambda: ctx.decompress(pw, 0, x.cpu()),
        ]
        for i, f in enumerate(bad):
            with pytest.raises(ValueError):
                f()
        assert not delta.any() and not x.any()                                        # nothing ran
        with pytest.raises(P.binding.DsError):
            ctx.decompress(pw, n, x)                                                  # the library's own check: row out of range
        ctx.worker_compress(0, g, delta, pw)
        ctx.server_aggregate_compress_update(0, pw, delta_s, ps, x, None, 0.1)
        torch.cuda.synchronize()
        assert delta.any() and x.any()
    finally:
        ctx.close()
        other.close()
