"""ctypes binding of libds_hip.so -- same names as the C-ABI in include/ds.h.

Marshalling only: tensors' device pointers and the current HIP stream are handed to the
library; nothing here computes.  There is no CPU fallback: if the library is missing the
import of a symbol fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

COMP_IDENTITY, COMP_SIGN, COMP_TOPK, COMP_QSGD, COMP_CLIP, COMP_RSPARSE, COMP_TERNARY = 0, 1, 2, 3, 4, 5, 6
SCALE_WHOLE, SCALE_SEGMENTS, SCALE_CHUNK = 0, 1, 2
F32, BF16 = 0, 1
FLAG_TOPK_MULTI_LAUNCH = 1
FLAG_DEFERRED_ERROR = 2
FLAG_SIGN_RMS = 4
FLAG_NO_ERROR_FEEDBACK = 8
FLAG_SERVER_IDENTITY = 16

_COMP = {"identity": COMP_IDENTITY, "sign": COMP_SIGN, "topk": COMP_TOPK, "qsgd": COMP_QSGD,
         "clip": COMP_CLIP, "rsparse": COMP_RSPARSE, "ternary": COMP_TERNARY}
_MODE = {"whole": SCALE_WHOLE, "segments": SCALE_SEGMENTS, "chunk": SCALE_CHUNK}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBNAME = "libds_hip.so"


class DsError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: status {code} ({_status_string(code)})")


class ds_config_t(C.Structure):
    _fields_ = [("comp", C.c_int32), ("n", C.c_int32), ("d", C.c_int64), ("grad_dtype", C.c_int32),
                ("scale_mode", C.c_int32), ("chunk", C.c_int64),
                ("seg_offsets", C.POINTER(C.c_int64)), ("n_seg", C.c_int32), ("levels", C.c_int32),
                ("k", C.c_int64), ("bucket", C.c_int32), ("flags", C.c_int32),
                ("seed", C.c_uint64), ("topk_max_workgroups", C.c_int32), ("topk_spin_limit", C.c_int32)]


class ds_payload_t(C.Structure):
    _fields_ = [("sign_words", C.c_void_p), ("scales", C.c_void_p), ("levels", C.c_void_p),
                ("pairs", C.c_void_p), ("dense", C.c_void_p)]


EXPORTS = ["ds_create", "ds_destroy", "ds_payload_sizes", "ds_worker_compress",
           "ds_server_aggregate_compress", "ds_apply_update", "ds_decompress", "ds_materialize_error",
           "ds_server_aggregate_compress_update", "ds_worker_compress_sign_noalloc", "ds_status", "ds_probe_copy",
           "ds_status_string", "ds_version"]

_lib = None


def library_path() -> str:
    return os.path.join(_HERE, _LIBNAME)


def load_library():
    """Loads libds_hip.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_1905_05957_amd.build` "
            "(there is no fallback path)")
    L = C.CDLL(path)
    vp, i64, i32, u64, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_float
    L.ds_create.argtypes = [C.POINTER(ds_config_t), C.POINTER(vp)]
    L.ds_destroy.argtypes = [vp]
    L.ds_payload_sizes.argtypes = [vp, i32, C.POINTER(C.c_size_t)]
    L.ds_worker_compress.argtypes = [vp, u64, vp, i64, vp, i64, C.POINTER(ds_payload_t), vp]
    L.ds_server_aggregate_compress.argtypes = [vp, u64, C.POINTER(ds_payload_t), vp,
                                               C.POINTER(ds_payload_t), vp]
    L.ds_apply_update.argtypes = [vp, C.POINTER(ds_payload_t), vp, vp, f32, f32, vp]
    L.ds_decompress.argtypes = [vp, C.POINTER(ds_payload_t), i32, i32, vp, vp]
    L.ds_materialize_error.argtypes = [vp, vp, i64, vp, vp]
    L.ds_server_aggregate_compress_update.argtypes = [vp, u64, C.POINTER(ds_payload_t), vp, C.POINTER(ds_payload_t),
                                                      vp, vp, f32, f32, vp]
    L.ds_status.argtypes = [vp]
    L.ds_probe_copy.argtypes = [vp, vp, C.c_size_t, vp]
    L.ds_worker_compress_sign_noalloc.argtypes = [i32, i64, i32, i32, vp, i64, vp, i64, vp, vp, vp]
    for name in EXPORTS:
        if name not in ("ds_status_string", "ds_version"):
            getattr(L, name).restype = C.c_int
    L.ds_status_string.argtypes = [C.c_int]
    L.ds_status_string.restype = C.c_char_p
    L.ds_version.argtypes = []
    L.ds_version.restype = C.c_char_p
    _lib = L
    return L


def _status_string(code: int) -> str:
    try:
        return load_library().ds_status_string(code).decode()
    except Exception:  # pragma: no cover
        return "?"


def _check(code: int, what: str):
    if code != 0:
        raise DsError(code, what)


def _need(t: torch.Tensor, what: str, dtype, shape) -> torch.Tensor:
    """A tensor is handed over as a bare pointer, so what the library assumes about it is checked
    here: device memory of the right element type, rows of the right length laid out densely
    (any row stride).  A wrong buffer would otherwise be a memory fault on the device."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError(f"{what}: a CUDA/HIP device tensor is required")
    if t.dtype != dtype:
        raise ValueError(f"{what}: dtype {t.dtype}, expected {dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{what}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if t.stride(-1) != 1 or (t.dim() == 2 and t.shape[0] > 1 and t.stride(0) < t.shape[1]):
        raise ValueError(f"{what}: rows must be dense (element stride 1, row stride >= row length)")
    return t


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


class Payload:
    """Device buffers of a batch of compressed messages (torch tensors, caller-owned)."""

    def __init__(self, comp: int, rows: int, d: int, W: int, S: int, k: int, device, sizes=None):
        self.comp, self.rows, self.d, self.k = comp, rows, d, k
        self.sign_words = self.scales = self.levels = self.pairs = self.dense = None
        if comp == COMP_IDENTITY:
            self.dense = torch.zeros((rows, d), dtype=torch.float32, device=device)
        elif comp == COMP_SIGN:
            self.sign_words = torch.zeros((rows, W), dtype=torch.int64, device=device)
            self.scales = torch.zeros((rows, S), dtype=torch.float32, device=device)
        elif comp == COMP_TOPK:
            self.pairs = torch.zeros((rows, k, 2), dtype=torch.int32, device=device)
        elif comp == COMP_QSGD:
            self.sign_words = torch.zeros((rows, W), dtype=torch.int64, device=device)
            self.scales = torch.zeros((rows, S), dtype=torch.float32, device=device)
            self.levels = torch.zeros((rows, (d + 1) // 2), dtype=torch.uint8, device=device)
        elif comp == COMP_CLIP:
            self.levels = torch.zeros((rows, sizes[2] // rows), dtype=torch.uint8, device=device)
        elif comp == COMP_RSPARSE:
            self.sign_words = torch.zeros((rows, W), dtype=torch.int64, device=device)
            self.dense = torch.zeros((rows, d), dtype=torch.float32, device=device)
        elif comp == COMP_TERNARY:
            self.sign_words = torch.zeros((rows, W), dtype=torch.int64, device=device)
            self.levels = torch.zeros((rows, 8 * W), dtype=torch.uint8, device=device)
            self.scales = torch.zeros((rows, 1), dtype=torch.float32, device=device)

    def check(self, ctx: "Context", rows: int, what: str, server: bool = False) -> "Payload":
        want = COMP_IDENTITY if (server and ctx.server_identity) else ctx.comp
        if self.comp != want or self.d != ctx.d or (self.comp != COMP_IDENTITY and self.k != ctx.k) or self.rows != rows:
            raise ValueError(f"{what}: a payload of {rows} message(s) allocated by this context is required")
        for t in self.tensors().values():
            if not t.is_cuda or not t.is_contiguous():
                raise ValueError(f"{what}: payload buffers must be contiguous device tensors")
        return self

    def c_struct(self) -> ds_payload_t:
        def p(t):
            return None if t is None else t.data_ptr()
        return ds_payload_t(p(self.sign_words), p(self.scales), p(self.levels), p(self.pairs),
                            p(self.dense))

    def tensors(self):
        return {k: v for k, v in (("sign_words", self.sign_words), ("scales", self.scales),
                                  ("levels", self.levels), ("pairs", self.pairs),
                                  ("dense", self.dense)) if v is not None}

    def to_numpy(self) -> dict:
        """Host copy in the layout the tests compare (top-k pairs split into idx / val)."""
        out = {}
        if self.sign_words is not None:
            out["sign_words"] = self.sign_words.cpu().numpy().view(np.uint64)
        if self.scales is not None:
            out["scales"] = self.scales.cpu().numpy()
        if self.levels is not None:
            out["levels"] = self.levels.cpu().numpy()
        if self.pairs is not None:
            pr = self.pairs.cpu().numpy()
            out["idx"] = np.ascontiguousarray(pr[:, :, 0])
            out["val"] = np.ascontiguousarray(pr[:, :, 1]).view(np.float32)
        if self.dense is not None:
            # randomised sparsification keeps its packed values in `dense`
            out["val" if self.comp == COMP_RSPARSE else "dense"] = self.dense.cpu().numpy()
        return out

    def load_numpy(self, host: dict) -> None:
        """Uploads a host message batch (same layout as to_numpy) into these buffers."""
        if self.sign_words is not None:
            self.sign_words.copy_(torch.from_numpy(host["sign_words"].view(np.int64)))
        if self.scales is not None:
            self.scales.copy_(torch.from_numpy(host["scales"]))
        if self.levels is not None:
            self.levels.copy_(torch.from_numpy(host["levels"]))
        if self.pairs is not None:
            pr = np.stack([host["idx"], host["val"].view(np.int32)], axis=-1)
            self.pairs.copy_(torch.from_numpy(np.ascontiguousarray(pr)))
        if self.dense is not None:
            self.dense.copy_(torch.from_numpy(host["val" if self.comp == COMP_RSPARSE else "dense"]))


class Context:
    """One configured DoubleSqueeze context (ds_ctx_t) on the current device."""

    def __init__(self, comp, n: int, d: int, grad_dtype: str = "f32", scale_mode="whole",
                 chunk: int = 0, seg_offsets=None, k: int = 0, bucket: int = 512, levels: int = 15,
                 seed: int = 0, flags: int = 0, keep_prob: Optional[float] = None,
                 topk_max_workgroups: int = 0, topk_spin_limit: int = 0):
        L = load_library()
        self.comp = _COMP[comp] if isinstance(comp, str) else int(comp)
        if keep_prob is not None:       # RSPARSE: the probability as a 24-bit threshold
            k = max(1, min(1 << 24, int(round(float(keep_prob) * (1 << 24)))))
        self.n, self.d, self.k = int(n), int(d), int(k)
        self.grad_dtype = BF16 if grad_dtype in ("bf16", BF16, torch.bfloat16) else F32
        mode = _MODE[scale_mode] if isinstance(scale_mode, str) else int(scale_mode)
        cfg = ds_config_t()
        cfg.comp, cfg.n, cfg.d, cfg.grad_dtype = self.comp, self.n, self.d, self.grad_dtype
        cfg.scale_mode, cfg.chunk = mode, int(chunk)
        self._seg = None
        if seg_offsets is not None:
            self._seg = np.ascontiguousarray(seg_offsets, dtype=np.int64)
            cfg.seg_offsets = self._seg.ctypes.data_as(C.POINTER(C.c_int64))
            cfg.n_seg = len(self._seg) - 1
        cfg.k, cfg.bucket, cfg.levels, cfg.seed = self.k, int(bucket), int(levels), int(seed)
        cfg.flags = int(flags)
        cfg.topk_max_workgroups, cfg.topk_spin_limit = int(topk_max_workgroups), int(topk_spin_limit)
        self._h = C.c_void_p()
        _check(L.ds_create(C.byref(cfg), C.byref(self._h)), "ds_create")
        sizes = self.payload_sizes(1)
        self.W = (self.d + 63) // 64
        self.S = sizes[1] // 4
        self.no_error_feedback = bool(int(flags) & FLAG_NO_ERROR_FEEDBACK)
        self.server_identity = bool(int(flags) & FLAG_SERVER_IDENTITY)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            torch.cuda.synchronize()
            load_library().ds_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass

    def status(self) -> int:
        """ds_status: 0, or the code of an asynchronous failure that no call has reported yet."""
        return int(load_library().ds_status(self._h))

    def payload_sizes(self, rows: int):
        out = (C.c_size_t * 5)()
        _check(load_library().ds_payload_sizes(self._h, rows, out), "ds_payload_sizes")
        return list(out)

    def alloc_payload(self, rows: int, device="cuda") -> Payload:
        return Payload(self.comp, rows, self.d, self.W, self.S, self.k, device, self.payload_sizes(rows))

    def alloc_server_payload(self, device="cuda") -> Payload:
        """The server's message: the compressor's, or the dense average under FLAG_SERVER_IDENTITY."""
        if self.server_identity:
            return Payload(COMP_IDENTITY, 1, self.d, self.W, self.S, 0, device)
        return self.alloc_payload(1, device)

    def worker_compress(self, step: int, g: torch.Tensor, delta: torch.Tensor, out: Payload,
                        stream=None):
        _need(g, "g", torch.bfloat16 if self.grad_dtype == BF16 else torch.float32, (self.n, self.d))
        if delta is not None or not self.no_error_feedback:
            _need(delta, "delta", torch.float32, (self.n, self.d))
        s = out.check(self, self.n, "out").c_struct()
        # a single row has no meaningful row stride (torch may report anything for it)
        gs = g.stride(0) if self.n > 1 else max(g.stride(0), self.d)
        ds_ = self.d if delta is None else (delta.stride(0) if self.n > 1 else max(delta.stride(0), self.d))
        _check(load_library().ds_worker_compress(self._h, step, g.data_ptr(), gs,
                                                 None if delta is None else delta.data_ptr(), ds_, C.byref(s),
                                                 _stream_ptr(stream)), "ds_worker_compress")

    def server_aggregate_compress(self, step: int, inp: Payload, delta_s: torch.Tensor,
                                  out: Payload, stream=None):
        if delta_s is not None or not (self.no_error_feedback or self.server_identity):
            _need(delta_s, "delta_s", torch.float32, (self.d,))
        a, b = inp.check(self, self.n, "in").c_struct(), out.check(self, 1, "out", server=True).c_struct()
        _check(load_library().ds_server_aggregate_compress(self._h, step, C.byref(a),
                                                           None if delta_s is None else delta_s.data_ptr(), C.byref(b),
                                                           _stream_ptr(stream)),
               "ds_server_aggregate_compress")

    def server_aggregate_compress_update(self, step: int, inp: Payload, delta_s: torch.Tensor, out: Payload,
                                         x: torch.Tensor, m: Optional[torch.Tensor], gamma: float,
                                         beta: float = 0.0, stream=None):
        if delta_s is not None or not (self.no_error_feedback or self.server_identity):
            _need(delta_s, "delta_s", torch.float32, (self.d,))
        _need(x, "x", torch.float32, (self.d,))
        if m is not None:
            _need(m, "m", torch.float32, (self.d,))
        a = inp.check(self, self.n, "in").c_struct()
        b = ds_payload_t() if (out is None and self.server_identity) else out.check(self, 1, "out", server=True).c_struct()
        _check(load_library().ds_server_aggregate_compress_update(
            self._h, step, C.byref(a), None if delta_s is None else delta_s.data_ptr(), C.byref(b), x.data_ptr(),
            None if m is None else m.data_ptr(), gamma, beta, _stream_ptr(stream)),
            "ds_server_aggregate_compress_update")

    def apply_update(self, srv: Payload, x: torch.Tensor, m: Optional[torch.Tensor], gamma: float,
                     beta: float = 0.0, stream=None):
        _need(x, "x", torch.float32, (self.d,))
        if m is not None:
            _need(m, "m", torch.float32, (self.d,))
        s = srv.check(self, 1, "srv", server=True).c_struct()
        _check(load_library().ds_apply_update(self._h, C.byref(s), x.data_ptr(),
                                              None if m is None else m.data_ptr(), gamma, beta,
                                              _stream_ptr(stream)), "ds_apply_update")

    def materialize_error(self, delta: Optional[torch.Tensor], delta_s: Optional[torch.Tensor],
                          stream=None):
        if delta is not None:
            _need(delta, "delta", torch.float32, (self.n, self.d))
        if delta_s is not None:
            _need(delta_s, "delta_s", torch.float32, (self.d,))
        _check(load_library().ds_materialize_error(
            self._h, None if delta is None else delta.data_ptr(),
            0 if delta is None else (delta.stride(0) if self.n > 1 else max(delta.stride(0), self.d)),
            None if delta_s is None else delta_s.data_ptr(), _stream_ptr(stream)),
            "ds_materialize_error")

    def decompress(self, p: Payload, row: int, out: torch.Tensor, stream=None):
        _need(out, "dense_out", torch.float32, (self.d,))
        s = p.check(self, p.rows, "p", server=(self.server_identity and p.comp == COMP_IDENTITY)).c_struct()
        _check(load_library().ds_decompress(self._h, C.byref(s), p.rows, row, out.data_ptr(),
                                            _stream_ptr(stream)), "ds_decompress")


# -- the C names, as plain functions ------------------------------------------------------
def ds_create(**kw) -> Context:
    return Context(**kw)


def ds_destroy(ctx: Context) -> None:
    ctx.close()


def ds_payload_sizes(ctx: Context, rows: int):
    return ctx.payload_sizes(rows)


def ds_worker_compress(ctx: Context, step, g, delta, out, stream=None):
    ctx.worker_compress(step, g, delta, out, stream)


def ds_server_aggregate_compress_update(ctx: Context, step, inp, delta_s, out, x, m, gamma, beta=0.0, stream=None):
    ctx.server_aggregate_compress_update(step, inp, delta_s, out, x, m, gamma, beta, stream)


def ds_materialize_error(ctx: Context, delta, delta_s, stream=None):
    ctx.materialize_error(delta, delta_s, stream)


def ds_server_aggregate_compress(ctx: Context, step, inp, delta_s, out, stream=None):
    ctx.server_aggregate_compress(step, inp, delta_s, out, stream)


def ds_apply_update(ctx: Context, srv, x, m, gamma, beta=0.0, stream=None):
    ctx.apply_update(srv, x, m, gamma, beta, stream)


def ds_decompress(ctx: Context, p, row, out, stream=None):
    ctx.decompress(p, row, out, stream)


def ds_probe_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    """The library's plain streaming copy kernel (measurement aid)."""
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("contiguous device tensors are required")
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise ValueError("source and destination differ in size")
    _check(load_library().ds_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream_ptr(stream)), "ds_probe_copy")


def ds_worker_compress_sign_noalloc(g: torch.Tensor, delta: torch.Tensor, sign_words: torch.Tensor,
                                    scales: torch.Tensor, flags: int = 0, stream=None) -> None:
    """The context-free, allocation-free worker block (1-bit, one scale per row)."""
    if g.dim() != 2:
        raise ValueError("g: [n, d] required")
    n, d = g.shape
    if g.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError(f"g: dtype {g.dtype}")
    _need(g, "g", g.dtype, (n, d))
    _need(delta, "delta", torch.float32, (n, d))
    _need(sign_words, "sign_words", torch.int64, (n, (d + 63) // 64))
    _need(scales, "scales", torch.float32, (n, 1))
    if not (sign_words.is_contiguous() and scales.is_contiguous()):
        raise ValueError("message buffers must be contiguous")
    gs = g.stride(0) if n > 1 else max(g.stride(0), d)
    ds_ = delta.stride(0) if n > 1 else max(delta.stride(0), d)
    _check(load_library().ds_worker_compress_sign_noalloc(
        n, d, BF16 if g.dtype == torch.bfloat16 else F32, int(flags), g.data_ptr(), gs, delta.data_ptr(), ds_,
        sign_words.data_ptr(), scales.data_ptr(), _stream_ptr(stream)), "ds_worker_compress_sign_noalloc")
