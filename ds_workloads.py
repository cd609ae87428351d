"""Seeded synthetic inputs for the five DoubleSqueeze workloads.

This module is the ONLY code shared by the CPU oracle's tests and the GPU path's tests and
bench: it draws gradients, initial error buffers and the least-squares toy problem, and
describes each workload's shape.  It holds none of the method's arithmetic (no
compensation, no compression, no update) and imports neither side.

The paper's own workload is ResNet-18 gradients on CIFAR-10 (Section 5.1, a model of about
44 MB, 8 workers + 1 server); no real gradients exist here, so these draws stand in for
them with the stated shapes, value distributions and segment structure.

Everything is generated with torch on the requested device from explicit seeds and handed
byte-identically to both sides (the GPU side keeps the tensor, the oracle gets
``.cpu().numpy()``).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

DATA_SEED = 1905
RNG_SEED = 0x5957


# --------------------------------------------------------------------------------------
# segment layout: n_seg log-uniform sizes in [lo, hi] that sum to d, unaligned boundaries
# --------------------------------------------------------------------------------------
def segment_offsets(d: int, n_seg: int, lo: int, hi: int, seed: int) -> np.ndarray:
    """Offsets [n_seg+1] of segments with log-uniform sizes in [lo, hi] summing to d."""
    assert n_seg * lo <= d <= n_seg * hi, (d, n_seg, lo, hi)
    rng = np.random.default_rng(seed)
    u = np.exp(rng.uniform(math.log(lo), math.log(hi), size=n_seg))
    sizes = np.floor(u * (d / u.sum())).astype(np.int64)
    sizes = np.clip(sizes, lo, hi)
    order = np.argsort(-sizes, kind="stable")
    rem = d - int(sizes.sum())
    # hand the remainder (either sign) to segments in descending-size order within bounds
    while rem != 0:
        moved = False
        for s in order:
            if rem == 0:
                break
            room = (hi - sizes[s]) if rem > 0 else (sizes[s] - lo)
            step = min(abs(rem), int(room))
            if step > 0:
                sizes[s] += step if rem > 0 else -step
                rem += -step if rem > 0 else step
                moved = True
        assert moved, "segment bounds cannot absorb the remainder"
    off = np.zeros(n_seg + 1, dtype=np.int64)
    off[1:] = np.cumsum(sizes)
    assert off[-1] == d and sizes.min() >= lo and sizes.max() <= hi
    return off


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _per_element(seg_off: np.ndarray, per_seg: np.ndarray, device) -> torch.Tensor:
    sizes = torch.from_numpy(np.diff(seg_off)).to(device)
    return torch.repeat_interleave(torch.from_numpy(per_seg.astype(np.float32)).to(device), sizes)


@dataclass
class Workload:
    """Shape and data recipe of one configuration."""
    name: str
    comp: str                      # 'identity' | 'sign' | 'topk' | 'qsgd' | 'clip' | 'rsparse' | 'ternary'
    n: int
    d: int
    grad_dtype: str = "f32"        # 'f32' | 'bf16'
    scale_mode: str = "whole"      # sign: 'whole' | 'segments' | 'chunk'
    chunk: int = 0
    seg_offsets: Optional[np.ndarray] = None   # data-shaping segments (and scale groups if 'segments')
    seg_sigma: Optional[np.ndarray] = None
    k: int = 0
    bucket: int = 512
    levels: int = 15
    seed: int = RNG_SEED           # Philox seed of the stochastic quantiser / sparsifier
    sign_rms: bool = False         # sign: root-mean-square scale instead of mean |v|
    clip_bits: int = 16            # clip: low bits set to zero
    keep_prob: float = 1.0         # rsparse: probability of keeping an element
    gamma: float = 0.05
    beta: Optional[float] = None   # momentum coefficient, None = plain SGD
    dist: str = "normal"           # 'normal' | 'student_t3' | 'laplace_outliers' | 'segment_normal'
    sigma: float = 1e-3
    data_seed: int = DATA_SEED
    delta_init_rel: float = 0.0    # initial worker error ~ N(0, (rel * sigma_seg)^2)
    extra: dict = field(default_factory=dict)

    # ---- scale groups of the sign compressor, as offsets ----
    def group_offsets(self) -> np.ndarray:
        if self.scale_mode == "whole":
            return np.array([0, self.d], dtype=np.int64)
        if self.scale_mode == "segments":
            return np.ascontiguousarray(self.seg_offsets, dtype=np.int64)
        off = np.arange(0, self.d, self.chunk, dtype=np.int64)
        return np.concatenate([off, np.array([self.d], dtype=np.int64)])

    # ---- data ----
    def gradients(self, set_index: int = 0, device="cpu") -> torch.Tensor:
        """[n, d] gradients (fp32, or bf16 for grad_dtype 'bf16'); one independent draw per set."""
        dev = torch.device(device)
        out_dtype = torch.bfloat16 if self.grad_dtype == "bf16" else torch.float32
        out = torch.empty((self.n, self.d), dtype=out_dtype, device=dev)
        sig = None
        if self.seg_sigma is not None:
            sig = _per_element(self.seg_offsets, self.seg_sigma, dev)
        for i in range(self.n):
            gen = _gen(dev, self.data_seed * 1000003 + set_index * 1009 + i)
            z = torch.randn(self.d, generator=gen, device=dev, dtype=torch.float32)
            if self.dist == "normal":
                row = z * self.sigma
            elif self.dist == "segment_normal":
                row = z * sig
            elif self.dist == "student_t3":
                w = torch.randn(3, self.d, generator=gen, device=dev, dtype=torch.float32)
                chi2 = (w * w).sum(0)
                row = z / torch.sqrt(chi2 / 3.0) * sig
            elif self.dist == "laplace_outliers":
                u = torch.rand(self.d, generator=gen, device=dev, dtype=torch.float32) - 0.5
                # |u| < 1/2 strictly, so the draw stays finite
                a2 = (2.0 * u.abs()).clamp_(max=1.0 - 2.0 ** -24)
                lap = -self.sigma * torch.sign(u) * torch.log1p(-a2)
                hit = torch.rand(self.d, generator=gen, device=dev, dtype=torch.float32) < 1e-3
                row = torch.where(hit, lap * 100.0, lap)
            elif self.dist == "levels8":
                # tie-heavy: magnitudes from only 8 distinct values, random signs
                q = torch.randint(0, 8, (self.d,), generator=gen, device=dev)
                sgn = torch.randint(0, 2, (self.d,), generator=gen, device=dev) * 2 - 1
                row = (q.float() + 1.0) * self.sigma * sgn.float()
            else:
                raise ValueError(self.dist)
            out[i] = row.to(out_dtype)
        return out

    def initial_delta(self, device="cpu") -> torch.Tensor:
        dev = torch.device(device)
        delta = torch.zeros((self.n, self.d), dtype=torch.float32, device=dev)
        if self.delta_init_rel > 0.0:
            sig = (_per_element(self.seg_offsets, self.seg_sigma, dev)
                   if self.seg_sigma is not None else self.sigma)
            for i in range(self.n):
                gen = _gen(dev, self.data_seed * 7919 + 31 * i + 5)
                delta[i] = torch.randn(self.d, generator=gen, device=dev) * sig * self.delta_init_rel
        return delta

    def initial_x(self, device="cpu") -> torch.Tensor:
        gen = _gen(torch.device(device), self.data_seed + 77)
        return torch.randn(self.d, generator=gen, device=device, dtype=torch.float32) * 0.02


def _loguniform(rng, lo, hi, size):
    return np.exp(rng.uniform(math.log(lo), math.log(hi), size=size))


# --------------------------------------------------------------------------------------
# the five configurations; `d` (and what scales with it) can be shrunk for parity tests
# --------------------------------------------------------------------------------------
def c1() -> Workload:
    return Workload("C1_least_squares_sign_whole", "sign", n=4, d=1024, scale_mode="whole",
                    gamma=0.05)


def c2(d: int = 11_173_962, n: int = 8, n_seg: int = 62, lo: int = 64,
       hi: Optional[int] = None) -> Workload:
    if hi is None:
        hi = 2_400_000 if d == 11_173_962 else max(4 * lo, (3 * d) // n_seg)
    off = segment_offsets(d, n_seg, lo, hi, DATA_SEED + 2)
    rng = np.random.default_rng(DATA_SEED + 20)
    sig = _loguniform(rng, 1e-4, 1e-1, n_seg)
    return Workload("C2_sign_segments_fp32", "sign", n=n, d=d, scale_mode="segments",
                    seg_offsets=off, seg_sigma=sig, dist="student_t3", delta_init_rel=0.1,
                    gamma=0.05)


def c3(d: int = 25_557_032, n: int = 8, k: Optional[int] = None) -> Workload:
    return Workload("C3_topk_1pct_fp32", "topk", n=n, d=d, k=(d // 100 if k is None else k),
                    dist="laplace_outliers", sigma=1e-3, gamma=0.05)


def c3_ties(d: int = 1 << 20, n: int = 4, k: Optional[int] = None) -> Workload:
    return Workload("C3_topk_ties", "topk", n=n, d=d, k=(d // 100 if k is None else k),
                    dist="levels8", sigma=1e-3, gamma=0.05)


def c4(d: int = 25_557_032, n: int = 16) -> Workload:
    return Workload("C4_qsgd_b512_s15", "qsgd", n=n, d=d, bucket=512, levels=15, dist="normal",
                    sigma=1e-3, gamma=0.05)


def c5(d: int = 124_439_808, n: int = 8, n_seg: int = 148, lo: int = 768,
       hi: Optional[int] = None) -> Workload:
    if hi is None:
        hi = 38_600_000 if d == 124_439_808 else max(4 * lo, (8 * d) // n_seg)
    off = segment_offsets(d, n_seg, lo, hi, DATA_SEED + 5)
    rng = np.random.default_rng(DATA_SEED + 50)
    sig = _loguniform(rng, 1e-5, 1e-2, n_seg)
    return Workload("C5_sign_chunk2048_bf16_momentum", "sign", n=n, d=d, grad_dtype="bf16",
                    scale_mode="chunk", chunk=2048, seg_offsets=off, seg_sigma=sig,
                    dist="segment_normal", gamma=0.1, beta=0.9)


def clip16(d: int = 25_557_032, n: int = 8) -> Workload:
    """Not one of the five configurations: the clipping compressor at the shape of C3/C4."""
    return Workload("X1_clip16_fp32", "clip", n=n, d=d, clip_bits=16, dist="normal", sigma=1e-3, gamma=0.05)


def rsparse60(d: int = 25_557_032, n: int = 8) -> Workload:
    """Not one of the five configurations: randomised sparsification, p = 0.6 (with error
    feedback the loop is stable only for p > 1/2), at the shape of C3/C4."""
    return Workload("X2_rsparse_p60_fp32", "rsparse", n=n, d=d, keep_prob=0.6, dist="normal", sigma=1e-3,
                    gamma=0.05)


# --------------------------------------------------------------------------------------
# C1: the distributed least-squares toy (problem data and minibatch gradients only)
# --------------------------------------------------------------------------------------
@dataclass
class LeastSquares:
    A: np.ndarray       # [n, rows, d] float64
    b: np.ndarray       # [n, rows]    float64
    x_star: np.ndarray  # [d]
    seed: int

    @property
    def n(self):
        return self.A.shape[0]

    def batch_rows(self, t: int, i: int, batch: int = 32) -> np.ndarray:
        rng = np.random.default_rng([self.seed, 424242, t, i])
        return np.sort(rng.choice(self.A.shape[1], size=batch, replace=False))

    def gradients(self, x: np.ndarray, t: int, batch: int = 32) -> np.ndarray:
        """g_i = A_B^T (A_B x - b_B) (loss = half the SUM of squared residuals over the
        minibatch), evaluated in fp64 at the caller's current x and rounded to fp32."""
        xx = x.astype(np.float64)
        g = np.empty((self.n, self.A.shape[2]), dtype=np.float32)
        for i in range(self.n):
            rows = self.batch_rows(t, i, batch)
            Ab, bb = self.A[i, rows], self.b[i, rows]
            g[i] = (Ab.T @ (Ab @ xx - bb)).astype(np.float32)
        return g

    def loss(self, x: np.ndarray) -> float:
        """f(x) = (1/n) sum_i (1/2)||A_i x - b_i||^2 / rows_i * 32 -- the expectation of the
        minibatch loss above (32 rows), so that it is the function SGD descends."""
        xx = x.astype(np.float64)
        tot = 0.0
        for i in range(self.n):
            r = self.A[i] @ xx - self.b[i]
            tot += 0.5 * float(r @ r) * (32.0 / self.A.shape[1])
        return tot / self.n


def least_squares(seed: int = DATA_SEED, n: int = 4, rows: int = 256, d: int = 1024) -> LeastSquares:
    rng = np.random.default_rng(seed)
    x_star = rng.standard_normal(d)
    A = rng.standard_normal((n, rows, d)) / math.sqrt(d)
    b = np.einsum("nrd,d->nr", A, x_star) + 0.01 * rng.standard_normal((n, rows))
    return LeastSquares(A=A, b=b, x_star=x_star, seed=seed)
