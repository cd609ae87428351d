"""The pins must notice mistakes: every entry below plants one plausible mistake in a private
copy of oracle/ds_oracle.c (a dropped term, a wrong sign or index, a swapped operand, an
off-by-one, a relaxed comparison), rebuilds that copy and runs the pin tests against it in a
subprocess.  A mutant that passes them all is a gap in the pins.  CPU only; nothing in the
repository is modified.
"""
import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_oracle_c1_toy.py", "tests/test_oracle_more_compressors.py"]

# (what is planted, text in ds_oracle.c, replacement)
MISTAKES = [
 ("sign bit for zero", "if (v[j] < 0.0f) words[j >> 6] |= (uint64_t)1 << (j & 63);\n    for (int32_t s = 0; s < n_groups; ++s) {\n        double sum = 0.0, len", "if (v[j] <= 0.0f) words[j >> 6] |= (uint64_t)1 << (j & 63);\n    for (int32_t s = 0; s < n_groups; ++s) {\n        double sum = 0.0, len"),
 ("sign scale len+1", "(float)(sum / len)", "(float)(sum / (len + 1.0))"),
 ("sign scale sum of v not |v|", ": (double)fabsf(v[j]);", ": (double)v[j];"),
 ("sign rms no sqrt", "(float)sqrt(sum / len)", "(float)(sum / len)"),
 ("sign decode swapped", "q[j] = neg ? -scales[s] : scales[s];", "q[j] = neg ? scales[s] : -scales[s];"),
 ("sign decode bit index", "int neg = (int)((words[j >> 6] >> (j & 63)) & 1u);\n            q[j] = neg ? -scales", "int neg = (int)((words[j >> 6] >> (63 - (j & 63))) & 1u);\n            q[j] = neg ? -scales"),
 ("sign decode wrong group scale", "q[j] = neg ? -scales[s] : scales[s];", "q[j] = neg ? -scales[0] : scales[0];"),
 ("topk tie to higher index", "(uint64_t)(0xFFFFFFFFu - (uint32_t)j);", "(uint64_t)((uint32_t)j);"),
 ("topk signed compare", "f32_bits(v[j]) & 0x7FFFFFFFu;", "f32_bits(v[j]);"),
 ("topk val abs", "val[r] = v[idx[r]];", "val[r] = fabsf(v[idx[r]]);"),
 ("topk k-1 entries", "for (int64_t r = 0; r < k; ++r) idx[r] = (int32_t)(0xFFFFFFFFu - (uint32_t)order[r]);", "for (int64_t r = 0; r < k; ++r) idx[r] = (int32_t)(0xFFFFFFFFu - (uint32_t)order[r < k - 1 ? r : r + 1 < d ? r + 1 : r]);"),
 ("topk smallest", "return (x < y) - (x > y);", "return (x > y) - (x < y);"),
 ("topk decode accumulate", "q[idx[r]] = val[r];", "q[idx[r]] = -val[r];"),
 ("qsgd norm no sqrt", "float norm = (float)sqrt(ss);", "float norm = (float)ss;"),
 ("qsgd norm l1", "ss += (double)v[j] * (double)v[j];", "ss += fabs((double)v[j]);"),
 ("qsgd inv s+1", "float inv = (float)s / norm;", "float inv = (float)(s + 1) / norm;"),
 ("qsgd u<=p", "(u < p ? 1 : 0)", "(u <= p ? 1 : 0)"),
 ("qsgd p inverted", "float p = r - fl; ", "float p = 1.0f - (r - fl); "),
 ("qsgd round to nearest", "(u < p ? 1 : 0)", "(0.5f < p ? 1 : 0)"),
 ("qsgd nibble order", "levels[j >> 1] |= (uint8_t)(code << ((j & 1) * 4));", "levels[j >> 1] |= (uint8_t)(code << ((1 - (j & 1)) * 4));"),
 ("qsgd decode unit s+1", "float unit = norms[B] / (float)s; ", "float unit = norms[B] / (float)(s + 1); "),
 ("qsgd decode no sign", "q[j] = neg ? -mag : mag;", "q[j] = mag;"),
 ("uniform word order", "return (float)(r[j & 3] >> 8) * 0x1p-24f;", "return (float)(r[3 - (j & 3)] >> 8) * 0x1p-24f;"),
 ("uniform low bits", "(r[j & 3] >> 8)", "(r[j & 3] & 0xFFFFFFu)"),
 ("uniform 2^-23", "* 0x1p-24f", "* 0x1p-23f"),
 ("uniform stream/step swapped", "(uint32_t)(block >> 32), stream, (uint32_t)step }", "(uint32_t)(block >> 32), (uint32_t)step, stream }"),
 ("uniform key hi no step", "(uint32_t)(seed >> 32) ^ (uint32_t)(step >> 32) }", "(uint32_t)(seed >> 32) }"),
 ("uniform block j>>1", "uint64_t block = (uint64_t)j >> 2;", "uint64_t block = (uint64_t)j >> 1;"),
 ("philox 9 rounds", "round < 10", "round < 9"),
 ("philox constants swapped", "(uint64_t)0xD2511F53u * (uint64_t)c0;\n        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;", "(uint64_t)0xCD9E8D57u * (uint64_t)c0;\n        uint64_t p1 = (uint64_t)0xD2511F53u * (uint64_t)c2;"),
 ("philox key bump swapped", "k0 += 0x9E3779B9u;\n        k1 += 0xBB67AE85u;", "k0 += 0xBB67AE85u;\n        k1 += 0x9E3779B9u;"),
 ("clip mask b-1", "~(uint32_t)(((uint64_t)1 << b) - 1u);", "~(uint32_t)(((uint64_t)1 << (b - 1)) - 1u);"),
 ("clip byte order", "out[j * nb + t] = (uint8_t)(top >> (8 * t));", "out[j * nb + t] = (uint8_t)(top >> (8 * (nb - 1 - t)));"),
 ("clip rounds to nearest", "uint32_t top = (f32_bits(v[j]) & mask) >> (32 - 8 * nb);", "uint32_t top = ((f32_bits(v[j]) + (b > 0 ? ((uint32_t)1 << (b - 1)) : 0)) & mask) >> (32 - 8 * nb);"),
 ("clip bytes threshold", "return b >= 24 ? 1 : b >= 16 ? 2 : 4;", "return b >= 24 ? 1 : b > 16 ? 2 : 4;"),
 ("rsparse <=", "dso_uniform24(seed, step, stream, j) < p)", "dso_uniform24(seed, step, stream, j) <= p)"),
 ("rsparse times p", "vals[r++] = v[j] / p;", "vals[r++] = v[j] * p;"),
 ("rsparse no scale", "vals[r++] = v[j] / p;", "vals[r++] = v[j];"),
 ("rsparse keep w.p. 1-p", "dso_uniform24(seed, step, stream, j) < p)", "dso_uniform24(seed, step, stream, j) >= p)"),
 ("rsparse decode order", "? vals[r++] : 0.0f;", "? vals[j] : 0.0f;"),
 ("worker v = g - delta", "v[j] = gij + delta_i[j];", "v[j] = gij - delta_i[j];"),
 ("worker error sign", "delta_i[j] = v[j] - q[j];", "delta_i[j] = q[j] - v[j];"),
 ("worker error dropped", "delta_i[j] = v[j] - q[j];", "delta_i[j] = 0.0f;"),
 ("worker stream 0", "rc = dso_encode(c, step, (uint32_t)i, v, &msgs[i]);", "rc = dso_encode(c, step, 0u, v, &msgs[i]);"),
 ("worker bf16 shift", "uint32_t u = (uint32_t)h << 16;", "uint32_t u = (uint32_t)h << 15;"),
 ("server forgets delta_s", "for (int64_t j = 0; j < d; ++j) v[j] = delta_s[j];", "for (int64_t j = 0; j < d; ++j) v[j] = 0.0f;"),
 ("server sum not mean", "float inv_n = 1.0f / (float)c->n;", "float inv_n = 1.0f;"),
 ("server 1/(n+1)", "float inv_n = 1.0f / (float)c->n;", "float inv_n = 1.0f / (float)(c->n + 1);"),
 ("server skips last worker", "for (int32_t i = 0; i < c->n && rc == 0; ++i) {\n        rc = dso_decode(c, &msgs[i], q);", "for (int32_t i = 0; i + 1 < c->n && rc == 0; ++i) {\n        rc = dso_decode(c, &msgs[i], q);"),
 ("server unfused mul add", "v[j] = fmaf(q[j], inv_n, v[j]);", "v[j] = v[j] + q[j] * inv_n;"),
 ("server error sign", "delta_s[j] = v[j] - q[j];", "delta_s[j] = q[j] - v[j];"),
 ("server uses worker stream", "dso_encode(c, step, DSO_SERVER_STREAM, v, out);", "dso_encode(c, step, 0u, v, out);"),
 ("update plus gamma", "x[j] = fmaf(-gamma, q[j], x[j]);", "x[j] = fmaf(gamma, q[j], x[j]);"),
 ("momentum x uses q", "x[j] = fmaf(-gamma, m[j], x[j]);", "x[j] = fmaf(-gamma, q[j], x[j]);"),
 ("momentum beta on q", "m[j] = fmaf(beta, m[j], q[j]);", "m[j] = fmaf(beta, q[j], m[j]);"),
 ("momentum dampened", "m[j] = fmaf(beta, m[j], q[j]);", "m[j] = fmaf(beta, m[j], (1.0f - beta) * q[j]);"),
 ("worker same delta row", "float *delta_i = delta + (int64_t)i * delta_stride;", "float *delta_i = delta;"),
 ("worker g row", "((const float *)g)[(int64_t)i * g_stride + j];", "((const float *)g)[j];"),
 ("server decodes msgs[0]", "rc = dso_decode(c, &msgs[i], q);\n        for (int64_t j = 0; j < d; ++j) v[j] = fmaf", "rc = dso_decode(c, &msgs[0], q);\n        for (int64_t j = 0; j < d; ++j) v[j] = fmaf"),
 ("topk message unsorted", "qsort(idx, (size_t)k, sizeof *idx, cmp_i32_asc);", ""),
 ("qsgd last bucket full", "hi = lo + bucket < d ? lo + bucket : d;\n        double ss", "hi = lo + bucket < d ? lo + bucket : d - 1;\n        double ss"),
 ("qsgd code clamp missing", "if (code > s) code = s; ", ""),
 ("clip decode shift", "uint32_t u = top << (32 - 8 * nb);", "uint32_t u = top << (24 - 8 * nb + 8 * (nb == 4));"),
 ("sign rms uses l1 flag ignored", "dso_sign_encode_kind(v, c->d, c->group_off, c->n_groups, c->sign_rms,", "dso_sign_encode_kind(v, c->d, c->group_off, c->n_groups, 0,"),
 ("update applies server error not message", "int rc = dso_decode(c, srv, q);", "int rc = dso_decode(c, srv, q); for (int64_t j = 0; j < d; ++j) q[j] = 0.5f * q[j];"),
 ("server error uses undecoded v", "delta_s[j] = v[j] - q[j];", "delta_s[j] = v[j] - 0.0f * q[j];"),
 ("ternary u<=p", "if (u < p) {\n                nz[", "if (u <= p) {\n                nz["),
 ("ternary keeps w.p. 1-p", "float p = fabsf(v[j]) / m; ", "float p = 1.0f - fabsf(v[j]) / m; "),
 ("ternary norm is the sum not the max", "if (a > m) m = a;", "m += a;"),
 ("ternary negative plane of all negatives", "                if (v[j] < 0.0f) neg[j >> 6] |= (uint64_t)1 << (j & 63);\n                ++kept;", "                ++kept;\n            }\n            if (v[j] < 0.0f) { neg[j >> 6] |= (uint64_t)1 << (j & 63);"),
 ("ternary sign dropped", "if (v[j] < 0.0f) neg[j >> 6] |= (uint64_t)1 << (j & 63);\n                ++kept;", "++kept;"),
 ("ternary scale is the max", "*scale = kept > 0 ? (float)(sum_abs / (double)kept) : 0.0f;", "*scale = kept > 0 ? m : 0.0f;"),
 ("ternary scale over d", "*scale = kept > 0 ? (float)(sum_abs / (double)kept) : 0.0f;", "*scale = kept > 0 ? (float)(sum_abs / (double)d) : 0.0f;"),
 ("ternary decode sign swapped", "q[j] = kept ? (minus ? -scale : scale) : 0.0f;", "q[j] = kept ? (minus ? scale : -scale) : 0.0f;"),
 ("ternary decode ignores the non-zero plane", "q[j] = kept ? (minus ? -scale : scale) : 0.0f;", "q[j] = minus ? -scale : scale;"),
 ("ternary draws from the server stream", "float u = dso_uniform24(seed, step, stream, j);\n            if (u < p) {\n                nz[", "float u = dso_uniform24(seed, step, DSO_SERVER_STREAM, j);\n            if (u < p) {\n                nz["),
]


def _run_mutant(args):
    name, old, new, source = args
    tmp = tempfile.mkdtemp(prefix="oracle_mutant_")
    try:
        for sub in ("oracle", "tests"):
            shutil.copytree(os.path.join(ROOT, sub), os.path.join(tmp, sub),
                            ignore=shutil.ignore_patterns("__pycache__", "*.so", "*.tmp*"))
        shutil.copy(os.path.join(ROOT, "ds_workloads.py"), tmp)
        with open(os.path.join(tmp, "oracle", "ds_oracle.c"), "w") as f:
            f.write(source.replace(old, new, 1))
        env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1")
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *PIN_FILES],
                           cwd=tmp, capture_output=True, text=True, env=env, timeout=600)
        return name, r.returncode
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def test_every_planted_mistake_fails_a_pin():
    with open(os.path.join(ROOT, "oracle", "ds_oracle.c")) as f:
        source = f.read()
    missing = [name for name, old, _ in MISTAKES if old not in source]
    assert not missing, f"the oracle's text changed; update these entries: {missing}"
    workers = max(1, min(8, (os.cpu_count() or 2) - 1))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        results = list(ex.map(_run_mutant, [(n, o, w, source) for n, o, w in MISTAKES]))
    survivors = [name for name, rc in results if rc == 0]
    broken = [name for name, rc in results if rc not in (0, 1)]        # 1 = tests failed; others: the mutant did not even run
    assert not broken, f"mutants that did not run (pytest exit code not 0/1): {broken}"
    assert not survivors, f"mistakes no pin noticed: {survivors}"
