"""Shared helpers of the GPU parity tests: build both sides from one Workload, run one
DoubleSqueeze step on each from identical state, compare to the stated bar.

Bar (per call, on identical inputs):
  sign planes, level codes, top-k indices ........ bit-exact (pad bits included)
  scales / bucket norms ........................... |a-b| <= 1e-6 |b|
  delta, delta_s, x, m ............................ max|a-b| <= 1e-6 max|b| per row
  top-k values .................................... equal as floats
"""
from __future__ import annotations

import numpy as np
import torch

import oracle as O
import paper_1905_05957_amd as P

REL = 1e-6


def keep_prob_24(p: float) -> float:
    """p rounded to a multiple of 2^-24 (exact in fp32): what a 24-bit uniform can resolve and
    what the library's integer threshold stands for."""
    return float(np.float32(max(1, min(1 << 24, int(round(p * (1 << 24))))) / np.float32(1 << 24)))


def oracle_config(wl) -> O.Config:
    comp = {"identity": O.IDENTITY, "sign": O.SIGN, "topk": O.TOPK, "qsgd": O.QSGD, "clip": O.CLIP,
            "rsparse": O.RSPARSE, "ternary": O.TERNARY}[wl.comp]
    return O.Config(comp, n=wl.n, d=wl.d, grad_bf16=(wl.grad_dtype == "bf16"),
                    group_off=wl.group_offsets() if wl.comp == "sign" else None,
                    k=wl.k, bucket=wl.bucket, levels=wl.levels, seed=wl.seed, sign_rms=wl.sign_rms,
                    clip_bits=wl.clip_bits, keep_prob=keep_prob_24(wl.keep_prob))


# ds_config_t::flags of the contexts that gpu_context builds; tests that cover both top-k
# refinement routes set it through the `topk_route` fixture of their module.
CONTEXT_FLAGS = 0
# further keyword arguments of P.Context for those contexts (top-k launch limits)
CONTEXT_KW: dict = {}


def gpu_context(wl) -> P.Context:
    return P.Context(wl.comp, wl.n, wl.d, grad_dtype=wl.grad_dtype, scale_mode=wl.scale_mode,
                     chunk=wl.chunk,
                     seg_offsets=wl.seg_offsets if wl.scale_mode == "segments" else None,
                     k=wl.k, bucket=wl.bucket, levels=wl.clip_bits if wl.comp == "clip" else wl.levels,
                     seed=wl.seed, keep_prob=wl.keep_prob if wl.comp == "rsparse" else None, flags=CONTEXT_FLAGS | (P.FLAG_SIGN_RMS if wl.sign_rms else 0), **CONTEXT_KW)


def host_grad(g: torch.Tensor) -> np.ndarray:
    """Contiguous host copy in the oracle's input format (bf16 -> uint16 bit patterns)."""
    g = g.contiguous()
    if g.dtype == torch.bfloat16:
        return g.view(torch.int16).cpu().numpy().view(np.uint16)
    return g.cpu().numpy()


def assert_close_rows(a: np.ndarray, b: np.ndarray, what: str, rel: float = REL):
    a2 = a.reshape(-1, a.shape[-1]) if a.ndim > 1 else a[None]
    b2 = b.reshape(-1, b.shape[-1]) if b.ndim > 1 else b[None]
    assert a2.shape == b2.shape, (what, a2.shape, b2.shape)
    for r in range(a2.shape[0]):
        ref = np.abs(b2[r]).max() if b2.shape[1] else 0.0
        err = np.abs(a2[r].astype(np.float64) - b2[r].astype(np.float64)).max() if b2.shape[1] else 0.0
        assert err <= rel * ref, f"{what} row {r}: max err {err:.3e} > {rel:g} * {ref:.3e}"


def assert_payload_equal(gpu: dict, ref: dict, what: str):
    assert set(gpu) == set(ref), (what, set(gpu), set(ref))
    if set(ref) == {"sign_words", "val"}:
        # randomised sparsification: the packed values count as far as the kept bits say;
        # what follows them is unspecified on the GPU side
        a, b = gpu["sign_words"], ref["sign_words"]
        assert np.array_equal(a, b), f"{what}.sign_words (kept bits) differ"
        for r in range(b.shape[0]):
            cnt = int(np.unpackbits(b[r].view(np.uint8)).sum())
            assert np.array_equal(gpu["val"][r, :cnt], ref["val"][r, :cnt]), f"{what}.val row {r} differs"
        return True
    for key in ref:
        a, b = gpu[key], ref[key]
        assert a.shape == b.shape, (what, key, a.shape, b.shape)
        if key in ("sign_words", "levels", "idx"):
            if not np.array_equal(a, b):
                bad = np.argwhere(a != b)
                raise AssertionError(f"{what}.{key}: {len(bad)} mismatches, first at {bad[0]}: "
                                     f"gpu {a[tuple(bad[0])]} ref {b[tuple(bad[0])]}")
        elif key == "scales":
            err = np.abs(a.astype(np.float64) - b.astype(np.float64))
            assert np.all(err <= REL * np.abs(b)), f"{what}.scales: max rel err {np.max(err / np.maximum(np.abs(b), 1e-300)):.3e}"
        elif key == "val":
            assert np.array_equal(a, b), f"{what}.val differs"      # by value: -0 == +0
        elif key == "dense":
            assert_close_rows(a, b, f"{what}.dense")
    return True


class Pair:
    """GPU state + the means to run one compared step.

    The library's two mode flags have no counterpart in the oracle, which stays a composition of
    its plain functions: without compensation the oracle's worker and server start from zero
    error buffers that are thrown away; a server that does not compress is the oracle's identity
    compressor fed with the decoded worker messages."""

    def __init__(self, wl, device):
        self.wl, self.dev = wl, device
        self.ctx = gpu_context(wl)
        self.cfg = oracle_config(wl)
        self.nofb, self.sid = self.ctx.no_error_feedback, self.ctx.server_identity
        self.ident = O.Config(O.IDENTITY, n=wl.n, d=wl.d)
        self.delta = None if self.nofb else wl.initial_delta(device)
        self.delta_s = None if (self.nofb or self.sid) else torch.zeros(wl.d, dtype=torch.float32, device=device)
        self.x = wl.initial_x(device)
        self.m = torch.zeros(wl.d, dtype=torch.float32, device=device) if wl.beta is not None else None
        self.pw = self.ctx.alloc_payload(wl.n, device)
        self.ps = self.ctx.alloc_server_payload(device)

    def gpu_step(self, t: int, g: torch.Tensor):
        self.ctx.worker_compress(t, g, self.delta, self.pw)
        self.ctx.server_aggregate_compress(t, self.pw, self.delta_s, self.ps)
        self.ctx.apply_update(self.ps, self.x, self.m, self.wl.gamma,
                              0.0 if self.wl.beta is None else self.wl.beta)

    def oracle_server(self, t: int, pw: dict, h_ds: np.ndarray) -> dict:
        """The oracle's parameter-server block for this pair's mode; h_ds is updated in place."""
        if self.sid:
            dense = {"dense": np.stack([O.decode(self.cfg, pw, i) for i in range(self.wl.n)])}
            return O.server_aggregate_compress(self.ident, t, dense, np.zeros(self.wl.d, np.float32))
        return O.server_aggregate_compress(self.cfg, t, pw, h_ds)

    def compared_step(self, t: int, g: torch.Tensor, tag: str = ""):
        """One step on the GPU and, call by call from the same inputs, on the oracle."""
        wl, cfg = self.wl, self.cfg
        scfg = self.ident if self.sid else cfg              # what the server's message is encoded with
        tag = f"{wl.name}{tag} t={t}"
        # ---- worker ----
        h_delta = np.zeros((wl.n, wl.d), np.float32) if self.nofb else self.delta.cpu().numpy().copy()
        h_g = host_grad(g)
        self.ctx.worker_compress(t, g, self.delta, self.pw)
        ref_pw = O.worker_compress(cfg, t, h_g, h_delta)
        gpu_pw = self.pw.to_numpy()
        assert_payload_equal(gpu_pw, ref_pw, tag + " worker payload")
        if not self.nofb:
            assert_close_rows(self.delta.cpu().numpy(), h_delta, tag + " delta")
        # ---- server (the oracle is fed the GPU's worker messages) ----
        h_ds = np.zeros(wl.d, np.float32) if self.delta_s is None else self.delta_s.cpu().numpy().copy()
        self.ctx.server_aggregate_compress(t, self.pw, self.delta_s, self.ps)
        ref_ps = self.oracle_server(t, gpu_pw, h_ds)
        gpu_ps = self.ps.to_numpy()
        assert_payload_equal(gpu_ps, ref_ps, tag + " server payload")
        if self.delta_s is not None:
            assert_close_rows(self.delta_s.cpu().numpy(), h_ds, tag + " delta_s")
        # ---- update (the oracle is fed the GPU's server message) ----
        h_x = self.x.cpu().numpy().copy()
        h_m = None if self.m is None else self.m.cpu().numpy().copy()
        beta = 0.0 if wl.beta is None else wl.beta
        self.ctx.apply_update(self.ps, self.x, self.m, wl.gamma, beta)
        O.apply_update(scfg, gpu_ps, h_x, h_m, wl.gamma, beta)
        assert_close_rows(self.x.cpu().numpy(), h_x, tag + " x")
        if h_m is not None:
            assert_close_rows(self.m.cpu().numpy(), h_m, tag + " m")
        # ---- the decoder the server uses ----
        dec = torch.empty(wl.d, dtype=torch.float32, device=self.dev)
        self.ctx.decompress(self.ps, 0, dec)
        assert_close_rows(dec.cpu().numpy(), O.decode(scfg, gpu_ps, 0), tag + " decode(server)")
        row = wl.n - 1
        self.ctx.decompress(self.pw, row, dec)
        assert_close_rows(dec.cpu().numpy(), O.decode(cfg, gpu_pw, row), tag + " decode(worker)")

    def close(self):
        self.ctx.close()
