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


def test_library_error_codes_on_a_live_context(gpu_device):
    """The C-ABI's own argument checks (include/ds.h: errors are return codes, detected before
    anything is launched, every buffer untouched), called through ctypes without the binding's."""
    import ctypes as C
    from paper_1905_05957_amd import binding as B
    dev, n, d = gpu_device, 2, 4100
    L = P.load_library()
    ctx = P.Context("sign", n, d, scale_mode="chunk", chunk=1024)
    try:
        g = torch.randn(n, d + 4, device=dev)
        delta = torch.zeros(n, d + 4, device=dev)
        delta_s = torch.zeros(d + 4, device=dev)
        x = torch.zeros(d + 4, device=dev)
        pw, ps = ctx.alloc_payload(n, dev), ctx.alloc_payload(1, dev)
        sw, ss = pw.c_struct(), ps.c_struct()
        null_words = B.ds_payload_t(None, pw.scales.data_ptr(), None, None, None)
        st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        h = ctx._h
        NULL, SHAPE, ALIGN = 1, 2, 4
        assert L.ds_worker_compress(h, 0, None, d + 4, delta.data_ptr(), d + 4, C.byref(sw), st) == NULL
        assert L.ds_worker_compress(h, 0, g.data_ptr(), d + 4, None, d + 4, C.byref(sw), st) == NULL
        assert L.ds_worker_compress(h, 0, g.data_ptr(), d + 4, delta.data_ptr(), d + 4, None, st) == NULL
        assert L.ds_worker_compress(h, 0, g.data_ptr(), d + 4, delta.data_ptr(), d + 4, C.byref(null_words), st) == NULL
        assert L.ds_worker_compress(h, 0, g.data_ptr(), d - 1, delta.data_ptr(), d + 4, C.byref(sw), st) == SHAPE
        assert L.ds_worker_compress(h, 0, g.data_ptr(), d + 4, delta.data_ptr(), d - 1, C.byref(sw), st) == SHAPE
        assert L.ds_worker_compress(h, 0, g.data_ptr() + 4, d + 4, delta.data_ptr(), d + 4, C.byref(sw), st) == ALIGN
        assert L.ds_worker_compress(h, 0, g.data_ptr(), d + 4, delta.data_ptr() + 8, d + 4, C.byref(sw), st) == ALIGN
        assert L.ds_server_aggregate_compress(h, 0, C.byref(sw), None, C.byref(ss), st) == NULL
        assert L.ds_server_aggregate_compress(h, 0, C.byref(sw), delta_s.data_ptr() + 4, C.byref(ss), st) == ALIGN
        assert L.ds_apply_update(h, C.byref(ss), None, None, 0.1, 0.0, st) == NULL
        assert L.ds_apply_update(h, C.byref(ss), x.data_ptr() + 4, None, 0.1, 0.0, st) == ALIGN
        assert L.ds_decompress(h, C.byref(sw), n, n, x.data_ptr(), st) == SHAPE
        assert L.ds_decompress(h, C.byref(sw), n, -1, x.data_ptr(), st) == SHAPE
        assert L.ds_materialize_error(h, delta.data_ptr(), d - 1, None, st) == SHAPE
        torch.cuda.synchronize()
        assert not delta.any() and not delta_s.any() and not x.any()
        assert not pw.sign_words.any() and not pw.scales.any()
        # rows that start 4 elements into a padded buffer row are fine (stride d + 4)
        assert L.ds_worker_compress(h, 0, g.data_ptr(), d + 4, delta.data_ptr(), d + 4, C.byref(sw), st) == 0
        torch.cuda.synchronize()
        assert delta[:, :d].any() and not delta[:, d:].any()
    finally:
        ctx.close()


def test_probe_copy_copies_and_checks_its_arguments(gpu_device):
    """The measurement aid ds_probe_copy: a plain copy, refused for sizes and pointers it cannot take."""
    import ctypes as C
    lib = P.load_library()
    src = torch.arange(0, 1 << 20, dtype=torch.float32, device=gpu_device)
    dst = torch.zeros_like(src)
    P.ds_probe_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    tail = torch.zeros(12, dtype=torch.float32, device=gpu_device)             # 48 bytes: three 16-byte units
    P.ds_probe_copy(src[:12].contiguous(), tail)
    torch.cuda.synchronize()
    assert torch.equal(tail, src[:12])
    p, q = src.data_ptr(), dst.data_ptr()
    assert lib.ds_probe_copy(None, q, 64, None) == 1                            # DS_ERR_NULL
    assert lib.ds_probe_copy(p, q, 0, None) == 2 and lib.ds_probe_copy(p, q, 40, None) == 2    # DS_ERR_SHAPE
    assert lib.ds_probe_copy(p + 4, q, 64, None) == 4                           # DS_ERR_ALIGN


def test_status_of_contexts_that_cannot_fail_asynchronously(gpu_device):
    """ds_status: DS_OK for every compressor whose kernels wait for nothing, DS_ERR_NULL without a context."""
    lib = P.load_library()
    assert lib.ds_status(None) == 1
    for kw in (dict(comp="sign", n=2, d=5000, scale_mode="chunk", chunk=1024), dict(comp="qsgd", n=2, d=5000),
               dict(comp="topk", n=2, d=5000, k=50, flags=P.FLAG_TOPK_MULTI_LAUNCH), dict(comp="topk", n=2, d=5000, k=50)):
        ctx = P.Context(**kw)
        try:
            assert ctx.status() == 0
        finally:
            ctx.close()
