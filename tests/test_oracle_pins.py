"""Pins of the CPU oracle against what the paper and the mathematics fix (CPU only).

Each test cites the passage of the paper (Tang et al., "DoubleSqueeze", ICML 2019) that
fixes the expected behaviour.  Expected values are hand-worked fixtures, closed forms,
invariants, brute force written independently here, or textbook special cases -- never a
second call of the oracle's own routine.
"""
import math
import os

import numpy as np
import pytest

import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _read_rows(path):
    rows = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            rows[parts[0]] = parts[1:]
    return rows


def unpack_bits(words, d):
    """bit j&63 of word j>>6, LSB first -- written with numpy, independent of the C decoder."""
    b = np.unpackbits(words.view(np.uint8), bitorder="little")
    return b[:d].astype(bool)


# ----------------------------------------------------------------------------------------
# Philox4x32-10 known answers (generator named by the workload definition, not the paper)
# ----------------------------------------------------------------------------------------
def test_philox_known_answers():
    n = 0
    with open(os.path.join(GOLD, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(t, 16) for t in line.replace("->", " ").split()]
            out = O.philox4x32_10(w[0:4], w[4:6])
            assert [int(v) for v in out] == w[6:10]
            n += 1
    assert n == 3


def test_uniform24_layout():
    # element j uses output word j&3 of the block with counter (j>>2, stream, step)
    seed, step, stream = 0x0123456789ABCDEF, 7, 3
    for j in (0, 1, 2, 3, 4, 1023, (1 << 34) + 5):
        blk = j >> 2
        out = O.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, stream, step & 0xFFFFFFFF],
                              [seed & 0xFFFFFFFF, (seed >> 32) ^ (step >> 32)])
        assert O.uniform24(seed, step, stream, j) == float(out[j & 3] >> 8) / 2 ** 24
    # the high word of the step reaches the key: step and step + 2^32 give different streams
    a = [O.uniform24(seed, 1, 0, j) for j in range(16)]
    b = [O.uniform24(seed, (1 << 32) + 1, 0, j) for j in range(16)]
    assert a != b
    assert all(0.0 <= u < 1.0 for u in a + b)


# ----------------------------------------------------------------------------------------
# 1-bit compressor: Section 5.1 "1-bit compression" (same magnitude after recovery)
# ----------------------------------------------------------------------------------------
def test_sign_hand_example():
    rows = _read_rows(os.path.join(GOLD, "sign_hand_example.txt"))
    v = np.array([float(t) for t in rows["v"]], np.float32)
    cfg = O.Config(O.SIGN, n=1, d=4)
    delta = np.zeros((1, 4), np.float32)
    p = O.worker_compress(cfg, 0, v[None, :].copy(), delta)
    assert p["scales"][0, 0] == float(rows["scale"][0])
    assert int(p["sign_words"][0, 0]) == int(rows["word"][0])
    assert list(O.decode(cfg, p)) == [float(t) for t in rows["q"]]
    assert list(delta[0]) == [float(t) for t in rows["delta"]]


@pytest.mark.parametrize("d,groups", [(1000, None), (1000, [0, 1, 65, 130, 700, 1000]),
                                      (4096 + 37, "chunk256")])
def test_sign_closed_forms(d, groups):
    r = _rng(11)
    v = (r.standard_t(3, d) * 1e-2).astype(np.float32)
    v[::97] = 0.0
    v[5] = -0.0
    if groups == "chunk256":
        off = O.chunk_offsets(d, 256)
    elif groups is None:
        off = np.array([0, d], np.int64)
    else:
        off = np.array(groups, np.int64)
    cfg = O.Config(O.SIGN, n=1, d=d, group_off=off)
    p = O.encode(cfg, 0, 0, v)
    q = O.decode(cfg, p)
    bits = unpack_bits(p["sign_words"][0], d)
    # bit = (v < 0): zeros and negative zero map to the positive code
    assert np.array_equal(bits, v < 0)
    # pad bits of the last word are zero
    allb = np.unpackbits(p["sign_words"][0].view(np.uint8), bitorder="little")
    assert not allb[d:].any()
    v64 = v.astype(np.float64)
    for s in range(len(off) - 1):
        lo, hi = off[s], off[s + 1]
        l1 = np.abs(v64[lo:hi]).sum()
        scale = p["scales"][0, s]
        # scale = mean |v| rounded once to fp32
        assert scale == np.float32(l1 / (hi - lo))
        # recovered group has the same l1 magnitude as the compensated one (Section 5.1)
        assert math.isclose(np.abs(q[lo:hi].astype(np.float64)).sum(), l1, rel_tol=1e-6)
        # contraction closed form (Section 4, assumption before Theorem 1):
        # ||v - Q[v]||^2 = ||v||^2 - ||v||_1^2/|G|  < ||v||^2
        err = ((v64[lo:hi] - q[lo:hi].astype(np.float64)) ** 2).sum()
        closed = (v64[lo:hi] ** 2).sum() - l1 * l1 / (hi - lo)
        assert math.isclose(err, closed, rel_tol=1e-5, abs_tol=1e-18)
        assert err <= (v64[lo:hi] ** 2).sum() * (1 + 1e-6)
        # every decoded element is +-scale with the sign of v
        assert np.array_equal(q[lo:hi], np.where(v[lo:hi] < 0, -scale, scale).astype(np.float32))


# ----------------------------------------------------------------------------------------
# top-k: Section 3.2 "Top-k sparsification", Section 5.1 "Top-k compression"
# ----------------------------------------------------------------------------------------
def brute_topk(v, k):
    """k largest |v| by repeated argmax, ties to the lower index; O(d k), tiny inputs only."""
    mag = np.abs(v.astype(np.float64))
    mag = np.where(np.isnan(mag), np.inf, mag)
    taken = np.zeros(len(v), bool)
    for _ in range(k):
        cand = np.where(taken, -1.0, mag)
        j = int(np.argmax(cand))          # argmax returns the first (lowest index) maximum
        taken[j] = True
    return np.nonzero(taken)[0].astype(np.int32)


@pytest.mark.parametrize("case", ["random", "all_equal", "all_zero", "pm_pairs", "levels"])
@pytest.mark.parametrize("k", [1, 7, 64, 300])
def test_topk_bruteforce(case, k):
    d = 300
    r = _rng(5)
    if case == "random":
        v = r.laplace(0, 1e-3, d)
    elif case == "all_equal":
        v = np.full(d, -0.5)
    elif case == "all_zero":
        v = np.zeros(d)
        v[::3] = -0.0
    elif case == "pm_pairs":
        v = np.repeat(r.standard_normal(d // 2), 2) * np.tile([1.0, -1.0], d // 2)
    else:
        v = r.integers(-3, 4, d).astype(np.float64) * 0.25
    v = v.astype(np.float32)
    cfg = O.Config(O.TOPK, n=1, d=d, k=k)
    p = O.encode(cfg, 0, 0, v)
    idx, val = p["idx"][0], p["val"][0]
    assert len(idx) == k
    assert np.all(np.diff(idx) > 0)                 # strictly ascending, hence k distinct
    assert np.array_equal(idx, brute_topk(v, k))
    assert np.array_equal(val.view(np.uint32), v[idx].view(np.uint32))
    q = O.decode(cfg, p)
    assert np.count_nonzero(q) <= k
    keep = np.zeros(d, bool)
    keep[idx] = True
    assert np.array_equal(q[keep].view(np.uint32), v[keep].view(np.uint32))
    assert not q[~keep].any()
    # error closed form: ||v - Q[v]||^2 = ||v||^2 - sum_kept v^2 <= (1 - k/d) ||v||^2
    v64 = v.astype(np.float64)
    err = ((v64 - q) ** 2).sum()
    assert math.isclose(err, (v64 ** 2).sum() - (v64[keep] ** 2).sum(), rel_tol=1e-9, abs_tol=1e-30)
    assert err <= (1 - k / d) * (v64 ** 2).sum() * (1 + 1e-9) + 1e-30


def test_topk_all_zero_takes_first_indices():
    cfg = O.Config(O.TOPK, n=1, d=100, k=10)
    p = O.encode(cfg, 0, 0, np.zeros(100, np.float32))
    assert list(p["idx"][0]) == list(range(10))


def test_topk_matches_partition_on_larger_input():
    # independent route: numpy's partition finds the k-th magnitude; no ties in this draw
    d, k = 200_000, 2_000
    v = _rng(9).laplace(0, 1e-3, d).astype(np.float32)
    cfg = O.Config(O.TOPK, n=1, d=d, k=k)
    p = O.encode(cfg, 0, 0, v)
    mag = np.abs(v)
    thr = np.partition(mag, d - k)[d - k]
    want = np.nonzero(mag >= thr)[0]
    assert len(want) == k
    assert np.array_equal(p["idx"][0], want.astype(np.int32))


# ----------------------------------------------------------------------------------------
# randomised quantisation: Section 3.2 "Randomized Quantization" (two-point, unbiased)
# ----------------------------------------------------------------------------------------
def nibbles(levels, d):
    lo = levels & 15
    hi = levels >> 4
    return np.stack([lo, hi], -1).reshape(-1)[:d].astype(np.int64)


def test_qsgd_two_point_and_bounds():
    d, bucket, s = 3 * 512 + 40, 512, 15
    v = (_rng(3).standard_normal(d) * 1e-3).astype(np.float32)
    v[700] = 0.0
    cfg = O.Config(O.QSGD, n=1, d=d, bucket=bucket, levels=s, seed=99)
    p = O.encode(cfg, 4, 2, v)
    q = O.decode(cfg, p)
    codes = nibbles(p["levels"][0], d)
    assert codes.max() <= s and codes.min() >= 0
    assert np.array_equal(unpack_bits(p["sign_words"][0], d), v < 0)
    nb = cfg.n_buckets
    assert nb == 4
    for B in range(nb):
        lo, hi = B * bucket, min(d, (B + 1) * bucket)
        norm = p["scales"][0, B]
        want = math.sqrt((v[lo:hi].astype(np.float64) ** 2).sum())
        assert norm == np.float32(want)
        pos = np.abs(v[lo:hi].astype(np.float64)) * s / float(norm)   # exact position
        c = codes[lo:hi]
        # the code is one of the two neighbouring levels of the exact position
        assert np.all(c >= np.floor(pos - 1e-4)) and np.all(c <= np.ceil(pos + 1e-4))
        # decoded magnitude never exceeds the norm, sign is preserved
        assert np.all(np.abs(q[lo:hi]) <= norm * (1 + 1e-6))
        nz = q[lo:hi] != 0
        assert np.array_equal(np.signbit(q[lo:hi][nz]), (v[lo:hi] < 0)[nz])
        # decoded value = code * norm / s
        assert np.allclose(np.abs(q[lo:hi]), c * (norm / np.float32(s)), rtol=1e-6, atol=0)
    # deterministic for a fixed (seed, step, stream); changes with each of them
    p2 = O.encode(cfg, 4, 2, v)
    assert np.array_equal(p["levels"], p2["levels"])
    assert not np.array_equal(p["levels"], O.encode(cfg, 5, 2, v)["levels"])
    assert not np.array_equal(p["levels"], O.encode(cfg, 4, 3, v)["levels"])
    cfg2 = O.Config(O.QSGD, n=1, d=d, bucket=bucket, levels=s, seed=100)
    assert not np.array_equal(p["levels"], O.encode(cfg2, 4, 2, v)["levels"])


def test_qsgd_unbiased_over_steps():
    # E_omega Q_omega[v] = v  (Section 3.2: "This compression operator is unbiased")
    d, bucket, s, S = 1024, 512, 15, 4000
    v = (_rng(8).standard_normal(d) * 1e-3).astype(np.float32)
    cfg = O.Config(O.QSGD, n=1, d=d, bucket=bucket, levels=s, seed=1234)
    acc = np.zeros(d, np.float64)
    for t in range(S):
        acc += O.decode(cfg, O.encode(cfg, t, 0, v))
    mean = acc / S
    norm = np.repeat([math.sqrt((v[:512].astype(np.float64) ** 2).sum()),
                      math.sqrt((v[512:].astype(np.float64) ** 2).sum())], 512)
    # per element the two-point variable has std <= unit/2; allow 5 sigma of the mean
    tol = 5.0 * (norm / s) / 2.0 / math.sqrt(S)
    assert np.all(np.abs(mean - v) <= tol)
    # and it is not trivially exact: rounding really is random
    assert np.abs(mean - v).max() > 0


def test_qsgd_rounding_probability():
    # a value at position l + p between levels goes up with probability p (Section 3.2)
    bucket, s = 512, 15
    v = np.zeros(bucket, np.float32)
    v[0] = 1.0                      # dominates the norm
    v[1:] = 0.02                    # position 15*0.02/norm ~ 0.27
    cfg = O.Config(O.QSGD, n=1, d=bucket, bucket=bucket, levels=s, seed=7)
    p = O.encode(cfg, 0, 0, v)
    norm = float(p["scales"][0, 0])
    pos = 15 * 0.02 / norm
    codes = nibbles(p["levels"][0], bucket)[1:]
    ups = 0
    T = 40
    for t in range(T):
        codes = nibbles(O.encode(cfg, t, 0, v)["levels"][0], bucket)[1:]
        assert set(np.unique(codes)) <= {0, 1}
        ups += int(codes.sum())
    frac = ups / (T * (bucket - 1))
    sd = math.sqrt(pos * (1 - pos) / (T * (bucket - 1)))
    assert abs(frac - pos) < 5 * sd


def test_qsgd_special_buckets():
    bucket, s = 512, 15
    d = 3 * bucket
    v = np.zeros(d, np.float32)
    v[bucket + 17] = -2.0 ** -9     # lone power of two: norm = |v|, position exactly s
    v[2 * bucket:] = 0.0            # all-zero bucket
    v[3] = 0.75
    cfg = O.Config(O.QSGD, n=1, d=d, bucket=bucket, levels=s, seed=5)
    for t in range(20):
        p = O.encode(cfg, t, 1, v)
        codes = nibbles(p["levels"][0], d)
        assert codes[bucket + 17] == s
        assert codes[2 * bucket:].sum() == 0 and p["scales"][0, 2] == 0.0
        q = O.decode(cfg, p)
        assert q[bucket + 17] == v[bucket + 17]
        assert not q[2 * bucket:].any()
        assert codes[3] == s and q[3] == 0.75


# ----------------------------------------------------------------------------------------
# Algorithm 1 as a whole
# ----------------------------------------------------------------------------------------
def _cfgs(n, d):
    return {
        "identity": O.Config(O.IDENTITY, n=n, d=d),
        "sign_whole": O.Config(O.SIGN, n=n, d=d),
        "sign_chunk": O.Config(O.SIGN, n=n, d=d, group_off=O.chunk_offsets(d, 192)),
        "topk": O.Config(O.TOPK, n=n, d=d, k=max(1, d // 20)),
        "qsgd": O.Config(O.QSGD, n=n, d=d, bucket=128, levels=15, seed=42),
    }


@pytest.mark.parametrize("name", ["identity", "sign_whole", "sign_chunk", "topk", "qsgd"])
def test_error_is_v_minus_decoded_message(name):
    """delta_i = v_i - Q[v_i] and delta = v - Q[v] hold bit for bit (Section 3.1, the two
    error-update equations), with Q[.] decoded by the decoder the server uses."""
    n, d = 4, 1000
    cfg = _cfgs(n, d)[name]
    r = _rng(21)
    g = (r.standard_normal((n, d)) * 1e-2).astype(np.float32)
    delta = (r.standard_normal((n, d)) * 1e-3).astype(np.float32)
    delta_s = (r.standard_normal(d) * 1e-3).astype(np.float32)
    v = g + delta                                   # Section 3.1, definition of v_t^(i)
    pw = O.worker_compress(cfg, 3, g, delta)
    inv_n = np.float32(1.0) / np.float32(n)
    acc = delta_s.astype(np.float64)
    for i in range(n):
        qi = O.decode(cfg, pw, i)
        assert np.array_equal(delta[i], v[i] - qi)
        acc += qi.astype(np.float64) * float(inv_n)
    d_s_before = delta_s.copy()
    ps = O.server_aggregate_compress(cfg, 3, pw, delta_s)
    qs = O.decode(cfg, ps)
    vs = delta_s.astype(np.float64) + qs            # reconstruct v = delta_new + Q[v]
    # v = delta_old + (1/n) sum_i Q[v_i]   (Section 3.1, parameter-server equation)
    assert np.allclose(vs, acc, rtol=0, atol=2e-7 * np.abs(acc).max())
    assert not np.array_equal(d_s_before, delta_s) or name == "identity"
    x = (r.standard_normal(d)).astype(np.float32)
    x0 = x.copy()
    O.apply_update(cfg, ps, x, None, 0.05)
    # x <- x - gamma Q[v]
    assert np.allclose(x, x0.astype(np.float64) - 0.05 * qs, rtol=0, atol=1e-7 * np.abs(x0).max())


def plain_parallel_sgd(x0, grads, gamma):
    """Textbook synchronous parallel SGD (Section 1): x <- x - gamma * (1/n) sum_i g_i,
    with the sum taken worker by worker."""
    x = x0.copy()
    n = grads.shape[1]
    inv_n = np.float32(1.0) / np.float32(n)
    for t in range(grads.shape[0]):
        avg = np.zeros_like(x)
        for i in range(n):
            avg = (avg.astype(np.float64) + grads[t, i].astype(np.float64) * float(inv_n)).astype(np.float32)
        x = (x.astype(np.float64) - float(np.float32(gamma)) * avg.astype(np.float64)).astype(np.float32)
    return x


@pytest.mark.parametrize("n", [4, 8])
def test_identity_compressor_is_plain_parallel_sgd(n):
    """With Q = identity the step is vanilla parallel SGD (Section 5.1 "Vanilla SGD") and
    every error buffer stays exactly zero.  n is a power of two, so each product with 1/n
    is exact and the fp64-then-round reference equals the fmaf chain bit for bit."""
    d, T, gamma = 512, 6, 0.05
    r = _rng(2)
    grads = (r.standard_normal((T, n, d))).astype(np.float32)
    x0 = r.standard_normal(d).astype(np.float32)
    cfg = O.Config(O.IDENTITY, n=n, d=d)
    x = x0.copy()
    delta = np.zeros((n, d), np.float32)
    delta_s = np.zeros(d, np.float32)
    for t in range(T):
        pw = O.worker_compress(cfg, t, grads[t].copy(), delta)
        ps = O.server_aggregate_compress(cfg, t, pw, delta_s)
        O.apply_update(cfg, ps, x, None, gamma)
        assert not delta.any() and not delta_s.any()
    assert np.array_equal(x, plain_parallel_sgd(x0, grads, gamma))


@pytest.mark.parametrize("name", ["sign_whole", "sign_chunk", "topk", "qsgd"])
def test_conservation_no_information_is_dropped(name):
    """Telescoped form of the global-view update rule (Section 3.3 and the auxiliary
    sequence y_t of the proof of Theorem 1):
        sum_t Q[v_t] + Omega_T = sum_t (1/n) sum_i g_t^(i),  Omega = delta + (1/n) sum_i delta_i
    and, with plain SGD, x_T - gamma*Omega_T... i.e. x_T = x_0 - gamma (sum gbar - Omega_T)."""
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
    # the error really is in use (the run is not trivially exact)
    assert np.abs(omega).max() > 1e-3 * scale


def test_momentum_update():
    n, d = 2, 300
    cfg = O.Config(O.SIGN, n=n, d=d, group_off=O.chunk_offsets(d, 64))
    r = _rng(4)
    g = r.standard_normal((n, d)).astype(np.float32)
    delta = np.zeros((n, d), np.float32)
    delta_s = np.zeros(d, np.float32)
    ps = O.server_aggregate_compress(cfg, 0, O.worker_compress(cfg, 0, g, delta), delta_s)
    q = O.decode(cfg, ps).astype(np.float64)
    x0 = r.standard_normal(d).astype(np.float32)
    # beta = 0 and a zero buffer: the momentum form equals the plain update
    xa, xb, m = x0.copy(), x0.copy(), np.zeros(d, np.float32)
    O.apply_update(cfg, ps, xa, None, 0.1)
    O.apply_update(cfg, ps, xb, m, 0.1, 0.0)
    assert np.array_equal(xa, xb) and np.array_equal(m, q.astype(np.float32))
    # two steps of heavy ball by hand: m1 = q, m2 = beta q + q ; x2 = x0 - gamma (m1 + m2)
    x, m = x0.copy(), np.zeros(d, np.float32)
    O.apply_update(cfg, ps, x, m, 0.1, 0.9)
    O.apply_update(cfg, ps, x, m, 0.1, 0.9)
    assert np.allclose(m, 1.9 * q, rtol=1e-6)
    assert np.allclose(x, x0 - 0.1 * (q + 1.9 * q), rtol=0, atol=1e-6 * np.abs(x0).max())


def test_bf16_gradients_are_widened_exactly():
    n, d = 2, 256
    r = _rng(6)
    g32 = (r.standard_normal((n, d)) * 1e-3).astype(np.float32)
    g16 = (g32.view(np.uint32) >> 16).astype(np.uint16)           # truncation is fine here
    gw = (g16.astype(np.uint32) << 16).view(np.float32)
    cfg16 = O.Config(O.SIGN, n=n, d=d, grad_bf16=True)
    cfg32 = O.Config(O.SIGN, n=n, d=d)
    da = (r.standard_normal((n, d)) * 1e-4).astype(np.float32)
    db = da.copy()
    pa = O.worker_compress(cfg16, 0, g16, da)
    pb = O.worker_compress(cfg32, 0, gw.copy(), db)
    assert np.array_equal(da, db)
    assert np.array_equal(pa["sign_words"], pb["sign_words"]) and np.array_equal(pa["scales"], pb["scales"])


def test_server_average_uses_every_worker_once():
    # distinct per-worker messages: a transposed or repeated operand changes the average
    n, d = 4, 64
    cfg = O.Config(O.IDENTITY, n=n, d=d)
    msgs = {"dense": np.arange(n * d, dtype=np.float32).reshape(n, d)}
    delta_s = np.full(d, 0.5, np.float32)
    ps = O.server_aggregate_compress(cfg, 0, msgs, delta_s)
    want = 0.5 + msgs["dense"].astype(np.float64).mean(0)
    assert np.array_equal(ps["dense"][0], want.astype(np.float32))
    assert not delta_s.any()


# ----------------------------------------------------------------------------------------
# Section 3.1: the compression randomness omega_t^(i) is drawn independently on every worker
# and on the server
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["qsgd", "rsparse"])
def test_every_worker_and_the_server_draw_from_their_own_stream(name):
    n, d, seed, t = 3, 4096, 11, 5
    if name == "qsgd":
        cfg = O.Config(O.QSGD, n=n, d=d, bucket=512, levels=15, seed=seed)
        plane = "levels"
    else:
        cfg = O.Config(O.RSPARSE, n=n, d=d, seed=seed, keep_prob=0.5)
        plane = "sign_words"
    one = O.Config(cfg.comp, n=1, d=d, bucket=512, levels=15, seed=seed, keep_prob=0.5)
    r = _rng(3)
    row = (r.standard_normal(d) * 1e-2).astype(np.float32)
    g = np.tile(row, (n, 1))                         # the same vector on every worker
    delta = np.zeros((n, d), np.float32)
    pw = O.worker_compress(cfg, t, g, delta)
    # identical inputs, different draws: the messages of two workers differ ...
    for i in range(n):
        for k in range(i + 1, n):
            assert not np.array_equal(pw[plane][i], pw[plane][k]), (i, k)
    # ... and worker i's message is what the compressor gives on stream i (counter word 2)
    for i in range(n):
        ref = O.encode(one, t, i, row)
        assert np.array_equal(pw[plane][i], ref[plane][0])
    # the server compresses its own vector on the stream 0xFFFFFFFF, not on a worker's
    v_s = np.zeros(d, np.float64)
    for i in range(n):
        v_s += O.decode(cfg, pw, i).astype(np.float64) / n
    delta_s = np.zeros(d, np.float32)
    ps = O.server_aggregate_compress(cfg, t, pw, delta_s)
    v32 = v_s.astype(np.float32)
    if name == "rsparse":                            # the keep decisions do not depend on the data
        assert np.array_equal(ps[plane][0], O.encode(one, t, 0xFFFFFFFF, v32)[plane][0])
        for i in range(n):
            assert not np.array_equal(ps[plane][0], O.encode(one, t, i, v32)[plane][0])
    else:
        # codes depend on v as well: redo the two-point rule on the first bucket with the
        # uniforms of a stream and count how many codes it explains (v_s here is the fp64
        # average, the oracle's is the fp32 chain, so a few codes may differ either way)
        lev = ps["levels"][0]
        codes = np.where(np.arange(512) % 2 == 0, lev[np.arange(512) // 2] & 15, lev[np.arange(512) // 2] >> 4)
        norm = float(ps["scales"][0, 0])
        rr = np.abs(v_s[:512]) * 15 / norm

        def explained(stream):
            u = np.array([O.uniform24(seed, t, stream, j) for j in range(512)])
            return np.mean(np.minimum(np.floor(rr) + (u < rr - np.floor(rr)), 15) == codes)

        assert explained(0xFFFFFFFF) > 0.98
        for i in range(n):
            assert explained(i) < 0.9


# ----------------------------------------------------------------------------------------
# Algorithm 1, "Average": v = delta + (1/n) sum_i Q[v_i], evaluated as one correctly rounded
# multiply-add per worker in ascending order (1/n rounded once) -- checked against exact
# rational arithmetic
# ----------------------------------------------------------------------------------------
def test_server_chain_is_one_rounding_per_worker():
    from fractions import Fraction
    n, d = 3, 400
    cfg = O.Config(O.IDENTITY, n=n, d=d)
    r = _rng(17)
    msgs = {"dense": (r.standard_normal((n, d)) * np.exp(r.uniform(-3, 3, (n, d)))).astype(np.float32)}
    delta_s = (r.standard_normal(d) * 0.3).astype(np.float32)
    start = delta_s.copy()
    ps = O.server_aggregate_compress(cfg, 0, msgs, delta_s)
    inv_n = Fraction(float(np.float32(1.0) / np.float32(n)))

    def round32(x: Fraction) -> float:
        # nearest fp32, ties to even, from the exact value: bracket it between neighbouring floats
        f = np.float32(float(x))                      # close; then fix up by comparing exactly
        lo, hi = np.nextafter(f, np.float32(-np.inf)), np.nextafter(f, np.float32(np.inf))
        best = min((lo, f, hi), key=lambda c: (abs(Fraction(float(c)) - x), int(np.float32(c).view(np.uint32)) & 1))
        return float(best)

    differs_from_two_roundings = 0
    for j in range(d):
        acc = Fraction(float(start[j]))
        acc2 = np.float32(start[j])
        for i in range(n):
            q = Fraction(float(msgs["dense"][i, j]))
            acc = Fraction(round32(q * inv_n + acc))
            acc2 = np.float32(acc2 + np.float32(msgs["dense"][i, j] * (np.float32(1.0) / np.float32(n))))
        assert float(ps["dense"][0, j]) == float(acc), j
        differs_from_two_roundings += float(acc2) != float(acc)
    assert differs_from_two_roundings > 0                # the inputs do tell the two evaluations apart


# ----------------------------------------------------------------------------------------
# Section 3.2: "b with probability (z - a)/(b - a)", "z/p with probability p".  A 24-bit
# uniform u = U 2^-24 realises a probability P 2^-24 exactly iff the event is u < P 2^-24
# (U in {0, .., P-1}); with <= it would be (P + 1) 2^-24.  The two draws below sit on that
# edge: seed 7, stream 0, U = 0 at (step 5837, element 66) and U = 1 at (step 4875, element 140).
# ----------------------------------------------------------------------------------------
def test_the_random_decisions_are_strict_comparisons():
    seed, d = 7, 1024
    (t0, j0), (t1, j1) = (5837, 66), (4875, 140)
    assert O.uniform24(seed, t0, 0, j0) == 0.0 and O.uniform24(seed, t1, 0, j1) == 2.0 ** -24
    ones = np.ones(d, np.float32)

    def kept(p, t, j):
        cfg = O.Config(O.RSPARSE, n=1, d=d, seed=seed, keep_prob=float(np.float32(p)))
        return bool(unpack_bits(O.encode(cfg, t, 0, ones)["sign_words"][0], d)[j])

    assert kept(2.0 ** -24, t0, j0)                  # U = 0 < 1
    assert not kept(2.0 ** -24, t1, j1)              # U = 1 is not below 1
    assert kept(2.0 ** -23, t1, j1)                  # but below 2

    # the quantiser on the same edge: one element of size 1 makes the bucket norm 1, the element
    # under test sits at 2^-24 of a level (s = 1), so it goes up iff u < 2^-24
    def code(t, j):
        v = np.zeros(d, np.float32)
        v[(j + 1) % d] = 1.0
        v[j] = np.float32(2.0 ** -24)
        cfg = O.Config(O.QSGD, n=1, d=d, bucket=d, levels=1, seed=seed)
        m = O.encode(cfg, t, 0, v)
        assert m["scales"][0, 0] == 1.0
        return int(m["levels"][0, j >> 1] >> ((j & 1) * 4)) & 15

    assert code(t0, j0) == 1
    assert code(t1, j1) == 0


def test_qsgd_position_a_hair_above_the_top_level_stays_at_the_top_level():
    """A lone element x in its bucket sits at r = |x| fl(s/|x|), which fp32 can round to just
    above s; the two representable neighbours of |x| = norm are s-1 and s (Section 3.2), so
    the code is s whatever the draw.  Here the draw is the U = 0 one (it would go "up")."""
    seed, d, s = 7, 1024, 15
    t0, j0 = 5837, 66
    x = np.float32(float.fromhex("0x1.4ea5a4p+0"))
    assert np.float32(x * np.float32(np.float32(s) / x)) > s       # the premise, in fp32
    assert O.uniform24(seed, t0, 0, j0) == 0.0
    v = np.zeros(d, np.float32)
    v[j0] = -x
    cfg = O.Config(O.QSGD, n=1, d=d, bucket=d, levels=s, seed=seed)
    m = O.encode(cfg, t0, 0, v)
    lev = m["levels"][0]
    codes = np.where(np.arange(d) % 2 == 0, lev[np.arange(d) // 2] & 15, lev[np.arange(d) // 2] >> 4)
    assert codes[j0] == s and codes.sum() == s
    q = O.decode(cfg, m, 0)
    assert q[j0] == -x and np.count_nonzero(q) == 1
