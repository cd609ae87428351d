"""Pins of the oracle's further compressors of Section 3.2 of the paper (Tang et al.,
"DoubleSqueeze", ICML 2019): the l2 reading of the 1-bit scale, clipping of low bits,
randomised sparsification.  CPU only.  Expected values are a hand-worked fixture, closed
forms, an independent arithmetic definition, invariants and special cases that reduce to the
identity -- never a second call of the routine under test."""
import os

import numpy as np
import pytest

import oracle as O
from test_oracle_pins import _read_rows, _rng, unpack_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------------------
# 1-bit compressor, scale = root mean square (Section 3.2 "1-Bit Quantization", l2 reading)
# ----------------------------------------------------------------------------------------
def test_sign_rms_hand_example():
    rows = _read_rows(os.path.join(GOLD, "sign_rms_hand_example.txt"))
    v = np.array([float(t) for t in rows["v"]], np.float32)[None]
    cfg = O.Config(O.SIGN, n=1, d=4, sign_rms=True)
    delta = np.zeros((1, 4), np.float32)
    p = O.worker_compress(cfg, 0, v, delta)
    assert p["scales"][0, 0] == np.float32(float(rows["scale"][0]))
    assert int(p["sign_words"][0, 0]) == int(rows["word"][0])
    assert O.decode(cfg, p, 0).tolist() == [float(t) for t in rows["q"]]
    assert delta[0].tolist() == [float(t) for t in rows["delta"]]


@pytest.mark.parametrize("groups", [None, [0, 1, 65, 130, 700, 1000]])
def test_sign_rms_closed_forms(groups):
    """Per group G with s = sqrt(mean v^2):  ||Q[v]||_2 = ||v||_2  (the recovered vector has
    the magnitude of the compensated one, Section 5.1, in the l2 sense), and
    ||v - Q[v]||^2 = ||v||^2 - 2 s ||v||_1 + |G| s^2 = 2 ||v||^2 - 2 s ||v||_1.
    The rms is never below the mean absolute value (Cauchy-Schwarz), with equality when all
    magnitudes are equal."""
    d = 1000
    off = np.array([0, d] if groups is None else groups, dtype=np.int64)
    r = _rng(31)
    v = (r.standard_normal(d) * 3e-2).astype(np.float32)
    v[5] = 0.0
    words = np.zeros((d + 63) // 64, np.uint64)
    s_rms = np.zeros(len(off) - 1, np.float32)
    s_l1 = np.zeros(len(off) - 1, np.float32)
    O.lib().dso_sign_encode_kind(v.ctypes.data, d, off.ctypes.data, len(off) - 1, 1, words.ctypes.data, s_rms.ctypes.data)
    O.lib().dso_sign_encode_kind(v.ctypes.data, d, off.ctypes.data, len(off) - 1, 0, words.ctypes.data, s_l1.ctypes.data)
    assert np.array_equal(unpack_bits(words, d), v < 0)
    v64 = v.astype(np.float64)
    for g in range(len(off) - 1):
        lo, hi = off[g], off[g + 1]
        seg = v64[lo:hi]
        s = float(s_rms[g])
        assert abs(s * np.sqrt(hi - lo) - np.linalg.norm(seg)) <= 1e-6 * np.linalg.norm(seg) + 1e-30
        q = np.where(seg < 0, -s, s)
        lhs = np.sum((seg - q) ** 2)
        rhs = 2 * np.sum(seg ** 2) - 2 * s * np.abs(seg).sum()
        assert abs(lhs - rhs) <= 1e-5 * np.sum(seg ** 2) + 1e-30
        assert s_rms[g] >= s_l1[g] * (1 - 1e-6)
        assert abs(float(s_l1[g]) - np.abs(seg).mean()) <= 1e-6 * np.abs(seg).mean() + 1e-30
    same = np.full(d, 0.375, np.float32) * np.where(r.random(d) < 0.5, -1, 1).astype(np.float32)
    O.lib().dso_sign_encode_kind(same.ctypes.data, d, off.ctypes.data, len(off) - 1, 1, words.ctypes.data, s_rms.ctypes.data)
    assert np.all(s_rms == np.float32(0.375))


# ----------------------------------------------------------------------------------------
# Clipping (Section 3.2 "Clipping": the lower b bits of a number are set to zero)
# ----------------------------------------------------------------------------------------
def clip_by_arithmetic(v, b):
    """The same operation stated on values instead of bit patterns, in fp64 (exact): a
    normal fp32 number with exponent e has spacing 2^(e-23); zeroing b <= 23 low bits rounds
    its magnitude down to a multiple of 2^(e-23+b).  Denormals have the fixed spacing 2^-149."""
    a = np.abs(v.astype(np.float64))
    _, ex = np.frexp(a)                       # a = m * 2^ex, m in [0.5, 1)
    e = np.maximum(ex - 1, -126)              # denormals share the exponent of the smallest normal
    ulp = np.ldexp(1.0, e - 23 + b)
    q = np.floor(a / ulp) * ulp
    return np.copysign(q, v.astype(np.float64))


@pytest.mark.parametrize("b", [1, 8, 16, 23])
def test_clip_equals_rounding_the_magnitude_down(b):
    r = _rng(b)
    v = (r.standard_normal(4000) * np.exp(r.uniform(-30, 30, 4000))).astype(np.float32)
    v[:4] = [0.0, -0.0, 1e-40, -3e-42]        # zeros and denormals
    v[4:6] = [np.float32(2.0) ** -126, np.float32(3.4e38)]
    nb = O.lib().dso_clip_bytes(b)
    assert nb == (2 if b >= 16 else 4)
    out = np.zeros(v.size * nb, np.uint8)
    O.lib().dso_clip_encode(v.ctypes.data, v.size, b, out.ctypes.data)
    q = np.zeros_like(v)
    O.lib().dso_clip_decode(out.ctypes.data, v.size, b, q.ctypes.data)
    assert np.array_equal(q.astype(np.float64), clip_by_arithmetic(v, b))
    assert np.array_equal(np.signbit(q), np.signbit(v))
    # the error is exact: v - q is representable, so the stored fp32 difference loses nothing
    assert np.array_equal((v - q).astype(np.float64), v.astype(np.float64) - q.astype(np.float64))
    # idempotent
    out2 = np.zeros_like(out)
    O.lib().dso_clip_encode(q.ctypes.data, v.size, b, out2.ctypes.data)
    assert np.array_equal(out, out2)


def test_clip_message_layout_and_wide_clips():
    """b = 16: the message is the upper half of every fp32 word (the bf16 grid, truncated);
    b >= 24 eats into the exponent: one byte per element, magnitudes only shrink, signs stay."""
    r = _rng(77)
    v = (r.standard_normal(1000) * 10).astype(np.float32)
    out = np.zeros(2000, np.uint8)
    O.lib().dso_clip_encode(v.ctypes.data, 1000, 16, out.ctypes.data)
    assert np.array_equal(out.view("<u2"), (v.view("<u4") >> 16).astype(np.uint16))
    for b in (24, 27, 31):
        assert O.lib().dso_clip_bytes(b) == 1
        o1 = np.zeros(1000, np.uint8)
        O.lib().dso_clip_encode(v.ctypes.data, 1000, b, o1.ctypes.data)
        q = np.zeros_like(v)
        O.lib().dso_clip_decode(o1.ctypes.data, 1000, b, q.ctypes.data)
        assert np.all(np.abs(q) <= np.abs(v)) and np.array_equal(np.signbit(q), np.signbit(v))
        assert np.all((q.view(np.uint32) & np.uint32((1 << b) - 1)) == 0)
    cfg = O.Config(O.CLIP, n=1, d=1000, clip_bits=31)          # only the sign survives: Q[v] = +-0
    delta = np.zeros((1, 1000), np.float32)
    O.worker_compress(cfg, 0, v[None].copy(), delta)
    assert np.array_equal(delta[0], v)


# ----------------------------------------------------------------------------------------
# Randomised sparsification (Section 3.2 "Randomized Sparsification": z/p with probability
# p, otherwise 0; unbiased)
# ----------------------------------------------------------------------------------------
def _rsparse(v, p, seed, step, stream):
    d = v.size
    words = np.zeros((d + 63) // 64, np.uint64)
    vals = np.zeros(d, np.float32)
    O.lib().dso_rsparse_encode(v.ctypes.data, d, np.float32(p), seed, step, stream, words.ctypes.data, vals.ctypes.data)
    q = np.zeros(d, np.float32)
    O.lib().dso_rsparse_decode(words.ctypes.data, vals.ctypes.data, d, q.ctypes.data)
    return unpack_bits(words, d), vals, q


def test_rsparse_outcomes_and_layout():
    r = _rng(5)
    d, p = 5000, 0.25
    v = (r.standard_normal(d)).astype(np.float32)
    v[v == 0] = 1.0
    keep, vals, q = _rsparse(v, p, 9, 4, 2)
    # the two outcomes of the section, nothing else
    assert np.array_equal(q[keep], v[keep] / np.float32(p)) and not q[~keep].any()
    # message: kept values in index order, then zeros
    cnt = int(keep.sum())
    assert np.array_equal(vals[:cnt], q[keep]) and not vals[cnt:].any()
    # the count is Binomial(d, p): within 6 standard deviations
    assert abs(cnt - d * p) <= 6 * np.sqrt(d * p * (1 - p))
    # deterministic in (seed, step, stream), different across them
    keep2, _, _ = _rsparse(v, p, 9, 4, 2)
    assert np.array_equal(keep, keep2)
    for other in ((10, 4, 2), (9, 5, 2), (9, 4, 3), (9, 4, O.SERVER_STREAM)):
        k3, _, _ = _rsparse(v, p, *other)
        assert 0.1 < np.mean(k3 != keep) < 0.6           # independent draws differ on 2p(1-p) = 37.5 %


def test_rsparse_is_unbiased_and_reduces_to_identity():
    """E Q[z] = p * z/p = z (Section 3.2: "an unbiased compression operator"); with p = 1
    every element is kept and divided by one: the identity."""
    r = _rng(6)
    d, p, T = 400, 0.3, 3000
    v = (r.standard_normal(d)).astype(np.float32)
    acc = np.zeros(d, np.float64)
    for t in range(T):
        acc += _rsparse(v, p, 1234, t, 0)[2]
    mean = acc / T
    sd = np.abs(v) * np.sqrt((1 - p) / p / T)             # std of the mean of T draws of z/p * Bernoulli(p)
    assert np.all(np.abs(mean - v) <= 5 * sd + 1e-7)
    keep, vals, q = _rsparse(v, 1.0, 1, 0, 0)
    assert keep.all() and np.array_equal(q, v) and np.array_equal(vals, v)


# ----------------------------------------------------------------------------------------
# Algorithm 1 with these compressors
# ----------------------------------------------------------------------------------------
def _cfgs(n, d):
    return {
        "sign_rms": O.Config(O.SIGN, n=n, d=d, group_off=O.chunk_offsets(d, 192), sign_rms=True),
        "clip16": O.Config(O.CLIP, n=n, d=d, clip_bits=16),
        "clip20": O.Config(O.CLIP, n=n, d=d, clip_bits=20),
        # with error feedback the error of this operator has energy (1-p)/p times that of v per
        # pass, so the loop is stable only for p > 1/2
        "rsparse": O.Config(O.RSPARSE, n=n, d=d, keep_prob=0.6, seed=7),
    }


@pytest.mark.parametrize("name", ["sign_rms", "clip16", "clip20", "rsparse"])
def test_error_is_v_minus_decoded_message(name):
    """delta_i = v_i - Q[v_i] and delta = v - Q[v] bit for bit (Section 3.1, the two
    error-update equations), and the server's v is delta + (1/n) sum_i Q[v_i]."""
    n, d = 4, 1000
    cfg = _cfgs(n, d)[name]
    r = _rng(21)
    g = (r.standard_normal((n, d)) * 1e-2).astype(np.float32)
    delta = (r.standard_normal((n, d)) * 1e-3).astype(np.float32)
    delta_s = (r.standard_normal(d) * 1e-3).astype(np.float32)
    v = g + delta
    pw = O.worker_compress(cfg, 3, g, delta)
    inv_n = np.float32(1.0) / np.float32(n)
    acc = delta_s.astype(np.float64)
    for i in range(n):
        qi = O.decode(cfg, pw, i)
        assert np.array_equal(delta[i], v[i] - qi)
        acc += qi.astype(np.float64) * float(inv_n)
    ps = O.server_aggregate_compress(cfg, 3, pw, delta_s)
    qs = O.decode(cfg, ps)
    vs = delta_s.astype(np.float64) + qs
    assert np.allclose(vs, acc, rtol=0, atol=2e-7 * np.abs(acc).max())


@pytest.mark.parametrize("name", ["sign_rms", "clip16", "clip20", "rsparse"])
def test_conservation_no_information_is_dropped(name):
    """Telescoped global view (Section 3.3 / proof of Theorem 1):
    sum_t Q[v_t] + Omega_T = sum_t mean_i g_t^(i),  Omega = delta + mean_i delta_i."""
    n, d, T, gamma = 4, 768, 25, 0.05
    cfg = _cfgs(n, d)[name]
    r = _rng(13)
    x = r.standard_normal(d).astype(np.float32)
    x0 = x.astype(np.float64)
    delta = np.zeros((n, d), np.float32)
    delta_s = np.zeros(d, np.float32)
    sum_gbar = np.zeros(d, np.float64)
    sum_q = np.zeros(d, np.float64)
    for t in range(T):
        g = (r.standard_normal((n, d)) * 1e-2).astype(np.float32)
        sum_gbar += g.astype(np.float64).mean(0)
        pw = O.worker_compress(cfg, t, g, delta)
        ps = O.server_aggregate_compress(cfg, t, pw, delta_s)
        sum_q += O.decode(cfg, ps)
        O.apply_update(cfg, ps, x, None, gamma)
    omega = delta_s.astype(np.float64) + delta.astype(np.float64).mean(0)
    scale = np.abs(sum_gbar).max()
    assert np.abs(sum_q + omega - sum_gbar).max() <= 1e-5 * scale
    assert np.abs(x - (x0 - gamma * (sum_gbar - omega))).max() <= 1e-5 * np.abs(x0).max()
    assert np.abs(omega).max() > 1e-4 * scale


# ----------------------------------------------------------------------------------------
# Ternary quantiser (Section 5.1, compressor of the paper's QSGD comparison system)
# ----------------------------------------------------------------------------------------
def _ternary_planes(p, d, row=0):
    nz = unpack_bits(np.ascontiguousarray(p["levels"][row]).view(np.uint64), d)
    neg = unpack_bits(p["sign_words"][row], d)
    return nz, neg


def test_ternary_hand_example():
    rows = _read_rows(os.path.join(GOLD, "ternary_hand_example.txt"))
    v = np.array([float(t) for t in rows["v"]], np.float32)
    cfg = O.Config(O.TERNARY, n=1, d=len(v), seed=77)
    for step in (0, 1, 12345):                                   # no draw matters here
        p = O.encode(cfg, step, 0, v)
        assert int(np.ascontiguousarray(p["levels"][0]).view(np.uint64)[0]) == int(rows["nz"][0])
        assert int(p["sign_words"][0, 0]) == int(rows["neg"][0])
        assert p["scales"][0, 0] == np.float32(float(rows["scale"][0]))
        assert O.decode(cfg, p, 0).tolist() == [float(t) for t in rows["q"]]


def test_ternary_codes_draws_and_scale():
    """Codes are -1, 0 or +1 with the sign of the element; element j is kept exactly when its
    draw (the counter-based uniform, pinned by its own known answers) is below |v_j| / m in
    fp32; the largest element is always kept, zeros never; count * scale = sum |v| (the decoded
    vector has the l1 magnitude of v)."""
    d = 3000
    r = _rng(5)
    v = (r.standard_normal(d) * 1e-2).astype(np.float32)
    v[17] = 0.0
    v[1234] = -0.2                                               # the largest magnitude, negative
    m = np.float32(0.2)
    cfg = O.Config(O.TERNARY, n=1, d=d, seed=0xABCDEF)
    for step, stream in ((0, 0), (3, 5), (2 ** 32 + 1, O.SERVER_STREAM)):
        p = O.encode(cfg, step, stream, v)
        nz, neg = _ternary_planes(p, d)
        assert not np.any(neg & ~nz)                             # a code of -1 is a non-zero code
        assert np.array_equal(neg, nz & (v < 0))                 # the code carries the element's sign
        u = np.array([O.uniform24(cfg.seed, step, stream, j) for j in range(d)], np.float32)
        prob = np.abs(v) / m                                     # fp32 division
        assert prob.dtype == np.float32
        assert np.array_equal(nz, u < prob)
        assert nz[1234] and not nz[17]
        scale = float(p["scales"][0, 0])
        total = np.abs(v.astype(np.float64)).sum()
        assert abs(nz.sum() * scale - total) <= 1e-6 * total
        q = O.decode(cfg, p, 0)
        assert np.array_equal(q, np.where(nz, np.where(neg, -np.float32(scale), np.float32(scale)), np.float32(0)))


def test_ternary_is_unbiased_before_the_rescale():
    """E[m * code_j] = v_j (probability |v_j|/m of sign(v_j)); the variance of m * code_j is
    m |v_j| - v_j^2 <= m^2 / 4, so the mean over S steps lies within 5 m / (2 sqrt S)."""
    d, S = 400, 3000
    r = _rng(9)
    v = (r.standard_normal(d) * 0.3).astype(np.float32)
    m = np.abs(v).max()
    cfg = O.Config(O.TERNARY, n=1, d=d, seed=2024)
    acc = np.zeros(d)
    kept_max = 0
    for step in range(S):
        p = O.encode(cfg, step, 1, v)
        nz, neg = _ternary_planes(p, d)
        acc += np.where(nz, np.where(neg, -1.0, 1.0), 0.0) * float(m)
        kept_max += int(nz[np.abs(v).argmax()])
    assert kept_max == S
    assert np.abs(acc / S - v).max() <= 5 * float(m) / (2 * np.sqrt(S))
    # a small element is mostly dropped: the quantiser is not the sign compressor
    small = np.abs(v).argmin()
    assert abs(acc[small] / S) < 0.2 * float(m)


def test_ternary_zero_vector_and_step_identity():
    d, n = 130, 3
    cfg = O.Config(O.TERNARY, n=n, d=d, seed=1)
    p = O.encode(O.Config(O.TERNARY, n=1, d=d, seed=1), 4, 0, np.zeros(d, np.float32))
    assert not p["levels"].any() and not p["sign_words"].any() and p["scales"][0, 0] == 0.0
    assert not O.decode(cfg, p, 0).any()
    # in the step: worker i draws from stream i, and delta = v - decode(message) bit for bit
    r = _rng(2)
    g = (r.standard_normal((n, d)) * 1e-2).astype(np.float32)
    g[1] = g[0]
    delta = (r.standard_normal((n, d)) * 1e-3).astype(np.float32)
    delta[1] = delta[0]
    v = g + delta
    pw = O.worker_compress(cfg, 7, g, delta)
    one = O.Config(O.TERNARY, n=1, d=d, seed=1)
    for i in range(n):
        ref = O.encode(one, 7, i, v[i])
        for key in ref:
            assert np.array_equal(pw[key][i], ref[key][0]), (key, i)
        assert np.array_equal(delta[i], v[i] - O.decode(one, ref, 0))
    assert not np.array_equal(pw["levels"][0], pw["levels"][1])   # same input, different streams


def test_ternary_decision_is_a_strict_comparison():
    """Probability |e|/m realised by a 24-bit uniform means u < |e|/m: an element of size zero
    is never kept, not even by the draw U = 0; an element at 2^-24 of the maximum is kept by
    U = 0 and dropped by U = 1.  (seed 7, stream 0: U = 0 at step 5837, element 66; U = 1 at
    step 4875, element 140.)"""
    seed, d = 7, 1024
    (t0, j0), (t1, j1) = (5837, 66), (4875, 140)
    assert O.uniform24(seed, t0, 0, j0) == 0.0 and O.uniform24(seed, t1, 0, j1) == 2.0 ** -24
    cfg = O.Config(O.TERNARY, n=1, d=d, seed=seed)

    def kept(t, j, size):
        v = np.zeros(d, np.float32)
        v[(j + 1) % d] = 1.0                         # the maximum
        v[j] = np.float32(size)
        return bool(_ternary_planes(O.encode(cfg, t, 0, v), d)[0][j])

    assert not kept(t0, j0, 0.0)                     # U = 0 is not below 0
    assert kept(t0, j0, 2.0 ** -24)                  # U = 0 < 1
    assert not kept(t1, j1, 2.0 ** -24)              # U = 1 is not below 1
    assert kept(t1, j1, 2.0 ** -23)
