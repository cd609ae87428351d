/*
 * ds_oracle.c -- plain, slow, single-threaded CPU oracle of the DoubleSqueeze step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the parity reference and the timed CPU
 * baseline.  Nothing in the product path (the HIP library and its Python binding)
 * includes, links, imports or calls it, and it includes nothing of theirs.
 *
 * What it computes (DoubleSqueeze, Tang et al., ICML 2019):
 *   Algorithm 1 / Section 3.1, one iteration t, n workers, one parameter server:
 *     worker i : v_i = g_i + delta_i ;  send Q[v_i] ;  delta_i <- v_i - Q[v_i]
 *     server   : v   = delta + (1/n) sum_i Q[v_i] ; send Q[v] ; delta <- v - Q[v]
 *     workers  : x  <- x - gamma * Q[v]
 *   Section 3.2 / Section 5.1 give the compressors Q: 1-bit (sign + scale so that the
 *   recovered vector has the magnitude of the compensated one), top-k by absolute
 *   value, two-point unbiased randomised quantisation, clipping of low bits and
 *   randomised sparsification; Section 5.1 adds the ternary quantiser of its QSGD comparison
 *   system.
 *
 * Every function follows the algorithm's steps in the paper's order: form v, encode,
 * decode, subtract.  The error buffers are always computed as "v minus the decoded
 * message" with the same decoder the server uses, never by a shortcut.
 *
 * Arithmetic: fp32 state, one rounding per stated operation (compile with
 * -ffp-contract=off; every fused multiply-add is an explicit fmaf).  Group sums for
 * scales and norms are accumulated in fp64 in index order and rounded once.
 *
 * Readings where the paper is silent (all restated in the repository's design notes):
 *   - 1-bit scale = mean |v| over the scale group (the l1 reading of "same magnitude",
 *     Section 5.1); bit = (v < 0); zero decodes to +scale.
 *   - top-k order: larger |v| bit pattern first, equal magnitudes by lower index;
 *     the message lists (index, value) by ascending index.
 *   - server sum order: start from delta, add worker 0..n-1 with fmaf(q_i, 1/n, acc).
 *   - randomised quantisation: buckets with an L2 norm, s uniform levels, the two
 *     neighbouring levels chosen with the probabilities of Section 3.2, random
 *     numbers from Philox4x32-10 (Salmon et al., SC'11) keyed on
 *     (seed, step, stream, index).
 *   - momentum (not in the paper, which uses none): m <- beta m + q ; x <- x - gamma m.
 *   - ternary quantiser: "magnitude" in its scale factor read as the l1 norm, as for the 1-bit
 *     compressor; probability |e|/m as one fp32 division.
 *
 * Parity pins live in tests/test_oracle_*.py; no function here is unpinned except the
 * conventions listed above (sum order, counter layout), which no text fixes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define DSO_IDENTITY 0
#define DSO_SIGN 1
#define DSO_TOPK 2
#define DSO_QSGD 3
#define DSO_CLIP 4
#define DSO_RSPARSE 5
#define DSO_TERNARY 6

#define DSO_SERVER_STREAM 0xFFFFFFFFu

typedef struct {
    int32_t comp;           /* DSO_* */
    int32_t n;              /* workers */
    int64_t d;              /* elements per vector */
    int32_t grad_bf16;      /* 1: g holds bf16 bit patterns (uint16), widened exactly */
    int32_t n_groups;       /* SIGN: number of scale groups */
    const int64_t *group_off; /* SIGN: n_groups+1 offsets, [0]=0, [n_groups]=d */
    int64_t k;              /* TOPK */
    int32_t bucket;         /* QSGD: elements per bucket */
    int32_t levels;         /* QSGD: s, 1..15 */
    uint64_t seed;          /* QSGD, RSPARSE */
    int32_t sign_rms;       /* SIGN: 1 = scale is the root mean square of the group (l2 reading) */
    int32_t clip_bits;      /* CLIP: b, the number of low bits set to zero, 1..31 */
    float keep_prob;        /* RSPARSE: p in (0, 1] */
} dso_config;

/* One message (one row).  Unused members are NULL. */
typedef struct {
    uint64_t *sign_words;   /* [ceil(d/64)]  bit (j&63) of word j>>6 = (v_j < 0), pad bits 0;
                               RSPARSE: the same plane holds "element j is kept" */
    float *scales;          /* SIGN: [n_groups] ; QSGD: [ceil(d/bucket)] bucket norms */
    uint8_t *levels;        /* QSGD: [ceil(d/2)], element j in byte j>>1, low nibble if j even;
                               CLIP: [d * nb] the kept upper bits, nb = 1, 2 or 4 bytes per element;
                               TERNARY: [8 * ceil(d/64)] a second bit plane (bytes of little-endian
                               64-bit words), bit j = (code_j != 0) */
    int32_t *idx;           /* TOPK: [k] ascending */
    float *val;             /* TOPK: [k] ; RSPARSE: [d] kept values z/p packed in index order, then zeros */
    float *dense;           /* IDENTITY: [d] */
} dso_msg;

/* ------------------------------------------------------------------------------------
 * Philox4x32-10, the public counter-based generator of Salmon, Moraes, Dror and Shaw
 * (SC'11).  Ten rounds; each round multiplies counter words 0 and 2 by two fixed
 * constants and mixes the high halves with words 1, 3 and the key; the key is bumped by
 * two Weyl constants between rounds.
 * ---------------------------------------------------------------------------------- */
void dso_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The uniform in [0,1) with 24 bits that decides the rounding of element j of a
 * vector, for iteration `step` and stream `stream` (worker index, or
 * DSO_SERVER_STREAM).  One Philox block serves four consecutive elements. */
float dso_uniform24(uint64_t seed, uint64_t step, uint32_t stream, int64_t j)
{
    uint64_t block = (uint64_t)j >> 2;
    uint32_t ctr[4] = { (uint32_t)block, (uint32_t)(block >> 32), stream, (uint32_t)step };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) ^ (uint32_t)(step >> 32) };
    uint32_t r[4];
    dso_philox4x32_10(ctr, key, r);
    return (float)(r[j & 3] >> 8) * 0x1p-24f;
}

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static uint32_t f32_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return u;
}

/* ------------------------------------------------------------------------------------
 * 1-bit compressor (Section 3.2 "1-Bit Quantization", Section 5.1 "1-bit compression").
 * One scale per group so that the decoded group has the same l1 magnitude as v.
 * ---------------------------------------------------------------------------------- */
/* rms = 0: scale = mean |v| (the l1 reading of "same magnitude", used everywhere by default).
 * rms = 1: scale = sqrt(mean v^2), the l2 reading: the decoded group then has the l2 norm of
 * v, which is what Section 3.2's "||x|| sign(x)" gives once it is normalised by sqrt(|G|). */
void dso_sign_encode_kind(const float *v, int64_t d, const int64_t *group_off, int32_t n_groups,
                          int32_t rms, uint64_t *words, float *scales)
{
    int64_t n_words = (d + 63) / 64;
    for (int64_t w = 0; w < n_words; ++w) words[w] = 0;
    for (int64_t j = 0; j < d; ++j)
        if (v[j] < 0.0f) words[j >> 6] |= (uint64_t)1 << (j & 63);
    for (int32_t s = 0; s < n_groups; ++s) {
        double sum = 0.0, len = (double)(group_off[s + 1] - group_off[s]);
        for (int64_t j = group_off[s]; j < group_off[s + 1]; ++j)
            sum += rms ? (double)v[j] * (double)v[j] : (double)fabsf(v[j]);
        scales[s] = rms ? (float)sqrt(sum / len) : (float)(sum / len);
    }
}

void dso_sign_decode(const uint64_t *words, const float *scales, int64_t d,
                     const int64_t *group_off, int32_t n_groups, float *q)
{
    (void)d;
    for (int32_t s = 0; s < n_groups; ++s)
        for (int64_t j = group_off[s]; j < group_off[s + 1]; ++j) {
            int neg = (int)((words[j >> 6] >> (j & 63)) & 1u);
            q[j] = neg ? -scales[s] : scales[s];
        }
}

/* ------------------------------------------------------------------------------------
 * Top-k compressor (Section 3.2 "Top-k sparsification", Section 5.1 "Top-k
 * compression"): keep the k entries of largest absolute value, zero the rest.
 * Written as its definition: order all entries, take the first k.
 * ---------------------------------------------------------------------------------- */
static int cmp_u64_desc(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x < y) - (x > y);
}

static int cmp_i32_asc(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int dso_topk_encode(const float *v, int64_t d, int64_t k, int32_t *idx, float *val)
{
    if (d > 0x7FFFFFFF || k < 0 || k > d) return 1;
    /* order key: magnitude bit pattern in the high half (larger first), and the
     * complement of the index in the low half so that equal magnitudes put the lower
     * index first when sorted in descending order. */
    uint64_t *order = (uint64_t *)malloc((size_t)(d > 0 ? d : 1) * sizeof *order);
    if (!order) return 2;
    for (int64_t j = 0; j < d; ++j) {
        uint64_t mag = f32_bits(v[j]) & 0x7FFFFFFFu;
        order[j] = (mag << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)j);
    }
    qsort(order, (size_t)d, sizeof *order, cmp_u64_desc);
    for (int64_t r = 0; r < k; ++r) idx[r] = (int32_t)(0xFFFFFFFFu - (uint32_t)order[r]);
    free(order);
    qsort(idx, (size_t)k, sizeof *idx, cmp_i32_asc);
    for (int64_t r = 0; r < k; ++r) val[r] = v[idx[r]];
    return 0;
}

void dso_topk_decode(const int32_t *idx, const float *val, int64_t k, int64_t d, float *q)
{
    for (int64_t j = 0; j < d; ++j) q[j] = 0.0f;
    for (int64_t r = 0; r < k; ++r) q[idx[r]] = val[r];
}

/* ------------------------------------------------------------------------------------
 * Randomised quantisation (Section 3.2 "Randomized Quantization"): a value z between
 * two neighbouring representable points a < b becomes b with probability
 * (z-a)/(b-a) and a otherwise, which is unbiased.  The representable points of a bucket
 * are {0, 1, ..., s} * norm/s with norm the bucket's l2 norm (the QSGD family); the
 * sign travels separately.
 * ---------------------------------------------------------------------------------- */
void dso_qsgd_encode(const float *v, int64_t d, int32_t bucket, int32_t s, uint64_t seed,
                     uint64_t step, uint32_t stream, uint8_t *levels, uint64_t *words,
                     float *norms)
{
    int64_t n_words = (d + 63) / 64, n_bytes = (d + 1) / 2;
    for (int64_t w = 0; w < n_words; ++w) words[w] = 0;
    for (int64_t b = 0; b < n_bytes; ++b) levels[b] = 0;
    int64_t n_buckets = (d + bucket - 1) / bucket;
    for (int64_t B = 0; B < n_buckets; ++B) {
        int64_t lo = B * bucket, hi = lo + bucket < d ? lo + bucket : d;
        double ss = 0.0;
        for (int64_t j = lo; j < hi; ++j) ss += (double)v[j] * (double)v[j];
        float norm = (float)sqrt(ss);
        norms[B] = norm;
        for (int64_t j = lo; j < hi; ++j)
            if (v[j] < 0.0f) words[j >> 6] |= (uint64_t)1 << (j & 63);
        if (!(norm > 0.0f)) continue;            /* all-zero bucket: every code 0 */
        float inv = (float)s / norm;             /* one fp32 divide */
        for (int64_t j = lo; j < hi; ++j) {
            float r = fabsf(v[j]) * inv;         /* position in units of norm/s */
            float fl = floorf(r);
            float p = r - fl;                    /* probability of the upper neighbour */
            float u = dso_uniform24(seed, step, stream, j);
            int code = (int)fl + (u < p ? 1 : 0);
            if (code > s) code = s;              /* r can round a hair above s */
            if (!(code >= 0)) code = 0;
            levels[j >> 1] |= (uint8_t)(code << ((j & 1) * 4));
        }
    }
}

void dso_qsgd_decode(const uint8_t *levels, const uint64_t *words, const float *norms,
                     int64_t d, int32_t bucket, int32_t s, float *q)
{
    int64_t n_buckets = (d + bucket - 1) / bucket;
    for (int64_t B = 0; B < n_buckets; ++B) {
        int64_t lo = B * bucket, hi = lo + bucket < d ? lo + bucket : d;
        float unit = norms[B] / (float)s;        /* one fp32 divide per bucket */
        for (int64_t j = lo; j < hi; ++j) {
            int code = (levels[j >> 1] >> ((j & 1) * 4)) & 15;
            float mag = (float)code * unit;
            int neg = (int)((words[j >> 6] >> (j & 63)) & 1u);
            q[j] = neg ? -mag : mag;
        }
    }
}

/* ------------------------------------------------------------------------------------
 * Clipping (Section 3.2 "Clipping"): the lower b bits of the number's binary
 * representation are set to zero.  The message keeps the remaining upper 32-b bits of every
 * element, in the smallest of 1, 2 or 4 bytes that holds them (b >= 24, b >= 16, otherwise),
 * little endian.  b = 16 is the truncation of fp32 to the bf16 grid.
 * ---------------------------------------------------------------------------------- */
int dso_clip_bytes(int32_t b) { return b >= 24 ? 1 : b >= 16 ? 2 : 4; }

void dso_clip_encode(const float *v, int64_t d, int32_t b, uint8_t *out)
{
    int nb = dso_clip_bytes(b);
    uint32_t mask = ~(uint32_t)(((uint64_t)1 << b) - 1u);
    for (int64_t j = 0; j < d; ++j) {
        uint32_t top = (f32_bits(v[j]) & mask) >> (32 - 8 * nb);
        for (int t = 0; t < nb; ++t) out[j * nb + t] = (uint8_t)(top >> (8 * t));
    }
}

void dso_clip_decode(const uint8_t *in, int64_t d, int32_t b, float *q)
{
    int nb = dso_clip_bytes(b);
    for (int64_t j = 0; j < d; ++j) {
        uint32_t top = 0;
        for (int t = 0; t < nb; ++t) top |= (uint32_t)in[j * nb + t] << (8 * t);
        uint32_t u = top << (32 - 8 * nb);
        float f;
        memcpy(&f, &u, sizeof f);
        q[j] = f;
    }
}

/* ------------------------------------------------------------------------------------
 * Randomised sparsification (Section 3.2 "Randomized Sparsification"): every element is
 * kept with probability p and then scaled to z/p, and set to zero otherwise, which makes the
 * operator unbiased.  (The section's sentence gives p for both outcomes; the zero outcome
 * has probability 1 - p.)  Element j is kept iff its uniform (the same counter-based stream
 * as the quantiser's) is below p.  The message is the plane of "kept" bits and the kept
 * values z/p (one fp32 division) packed in index order.
 * ---------------------------------------------------------------------------------- */
void dso_rsparse_encode(const float *v, int64_t d, float p, uint64_t seed, uint64_t step, uint32_t stream,
                        uint64_t *keep_words, float *vals)
{
    int64_t n_words = (d + 63) / 64, r = 0;
    for (int64_t w = 0; w < n_words; ++w) keep_words[w] = 0;
    for (int64_t j = 0; j < d; ++j) vals[j] = 0.0f;
    for (int64_t j = 0; j < d; ++j) {
        if (dso_uniform24(seed, step, stream, j) < p) {
            keep_words[j >> 6] |= (uint64_t)1 << (j & 63);
            vals[r++] = v[j] / p;
        }
    }
}

void dso_rsparse_decode(const uint64_t *keep_words, const float *vals, int64_t d, float *q)
{
    int64_t r = 0;
    for (int64_t j = 0; j < d; ++j)
        q[j] = ((keep_words[j >> 6] >> (j & 63)) & 1u) ? vals[r++] : 0.0f;
}

/* ------------------------------------------------------------------------------------
 * Ternary quantiser (Section 5.1, the compressor of the paper's QSGD comparison system):
 * every element becomes a code in {-1, 0, +1}.  With m the largest absolute value of the
 * vector, element e becomes sign(e) with probability |e| / m and 0 otherwise (so the largest
 * element is always kept, and m * code is an unbiased estimate of e).  One scale factor per
 * vector, "magnitude of original gradient over magnitude of compressed gradient", in the same
 * l1 reading as the 1-bit compressor: scale = sum |v_j| / #(non-zero codes), so that the
 * decoded vector code * scale has the l1 magnitude of v.  The draw for element j is the
 * counter-based uniform of the quantiser above; an all-zero vector gives all-zero codes and
 * scale 0.
 * Message: plane `neg` (bit j = code_j is -1), plane `nz` (bit j = code_j is not 0), scale.
 * ---------------------------------------------------------------------------------- */
void dso_ternary_encode(const float *v, int64_t d, uint64_t seed, uint64_t step, uint32_t stream,
                        uint64_t *neg, uint64_t *nz, float *scale)
{
    int64_t n_words = (d + 63) / 64;
    for (int64_t w = 0; w < n_words; ++w) { neg[w] = 0; nz[w] = 0; }
    float m = 0.0f;
    double sum_abs = 0.0;
    for (int64_t j = 0; j < d; ++j) {
        float a = fabsf(v[j]);
        if (a > m) m = a;
        sum_abs += (double)a;
    }
    int64_t kept = 0;
    if (m > 0.0f) {
        for (int64_t j = 0; j < d; ++j) {
            float p = fabsf(v[j]) / m;               /* one fp32 divide; 1 for the largest element */
            float u = dso_uniform24(seed, step, stream, j);
            if (u < p) {
                nz[j >> 6] |= (uint64_t)1 << (j & 63);
                if (v[j] < 0.0f) neg[j >> 6] |= (uint64_t)1 << (j & 63);
                ++kept;
            }
        }
    }
    *scale = kept > 0 ? (float)(sum_abs / (double)kept) : 0.0f;
}

void dso_ternary_decode(const uint64_t *neg, const uint64_t *nz, float scale, int64_t d, float *q)
{
    for (int64_t j = 0; j < d; ++j) {
        int kept = (int)((nz[j >> 6] >> (j & 63)) & 1u);
        int minus = (int)((neg[j >> 6] >> (j & 63)) & 1u);
        q[j] = kept ? (minus ? -scale : scale) : 0.0f;
    }
}

/* ------------------------------------------------------------------------------------
 * Q[.] and its decoder, selected by the configuration.
 * ---------------------------------------------------------------------------------- */
int dso_encode(const dso_config *c, uint64_t step, uint32_t stream, const float *v, dso_msg *m)
{
    switch (c->comp) {
    case DSO_IDENTITY:
        for (int64_t j = 0; j < c->d; ++j) m->dense[j] = v[j];
        return 0;
    case DSO_SIGN:
        dso_sign_encode_kind(v, c->d, c->group_off, c->n_groups, c->sign_rms, m->sign_words, m->scales);
        return 0;
    case DSO_TOPK:
        return dso_topk_encode(v, c->d, c->k, m->idx, m->val);
    case DSO_QSGD:
        dso_qsgd_encode(v, c->d, c->bucket, c->levels, c->seed, step, stream, m->levels,
                        m->sign_words, m->scales);
        return 0;
    case DSO_CLIP:
        if (c->clip_bits < 1 || c->clip_bits > 31) return 3;
        dso_clip_encode(v, c->d, c->clip_bits, m->levels);
        return 0;
    case DSO_RSPARSE:
        if (!(c->keep_prob > 0.0f && c->keep_prob <= 1.0f)) return 3;
        dso_rsparse_encode(v, c->d, c->keep_prob, c->seed, step, stream, m->sign_words, m->val);
        return 0;
    case DSO_TERNARY:
        dso_ternary_encode(v, c->d, c->seed, step, stream, m->sign_words, (uint64_t *)m->levels, m->scales);
        return 0;
    }
    return 3;
}

int dso_decode(const dso_config *c, const dso_msg *m, float *q)
{
    switch (c->comp) {
    case DSO_IDENTITY:
        for (int64_t j = 0; j < c->d; ++j) q[j] = m->dense[j];
        return 0;
    case DSO_SIGN:
        dso_sign_decode(m->sign_words, m->scales, c->d, c->group_off, c->n_groups, q);
        return 0;
    case DSO_TOPK:
        dso_topk_decode(m->idx, m->val, c->k, c->d, q);
        return 0;
    case DSO_QSGD:
        dso_qsgd_decode(m->levels, m->sign_words, m->scales, c->d, c->bucket, c->levels, q);
        return 0;
    case DSO_CLIP:
        dso_clip_decode(m->levels, c->d, c->clip_bits, q);
        return 0;
    case DSO_RSPARSE:
        dso_rsparse_decode(m->sign_words, m->val, c->d, q);
        return 0;
    case DSO_TERNARY:
        dso_ternary_decode(m->sign_words, (const uint64_t *)m->levels, m->scales[0], c->d, q);
        return 0;
    }
    return 3;
}

/* ------------------------------------------------------------------------------------
 * Algorithm 1, "On worker" (first block): for every worker i,
 *   v_i = g_i + delta_i ;  msg_i = Q[v_i] ;  delta_i <- v_i - decode(msg_i).
 * g: [n, g_stride] (float, or uint16 bf16 patterns), delta: [n, delta_stride] in place,
 * msgs: n messages.
 * ---------------------------------------------------------------------------------- */
int dso_worker_compress(const dso_config *c, uint64_t step, const void *g, int64_t g_stride,
                        float *delta, int64_t delta_stride, dso_msg *msgs)
{
    int64_t d = c->d;
    float *v = (float *)malloc((size_t)(d > 0 ? d : 1) * sizeof *v);
    float *q = (float *)malloc((size_t)(d > 0 ? d : 1) * sizeof *q);
    if (!v || !q) { free(v); free(q); return 2; }
    int rc = 0;
    for (int32_t i = 0; i < c->n && rc == 0; ++i) {
        float *delta_i = delta + (int64_t)i * delta_stride;
        for (int64_t j = 0; j < d; ++j) {
            float gij = c->grad_bf16 ? bf16_to_f32(((const uint16_t *)g)[(int64_t)i * g_stride + j])
                                     : ((const float *)g)[(int64_t)i * g_stride + j];
            v[j] = gij + delta_i[j];
        }
        rc = dso_encode(c, step, (uint32_t)i, v, &msgs[i]);
        if (rc) break;
        rc = dso_decode(c, &msgs[i], q);
        for (int64_t j = 0; j < d; ++j) delta_i[j] = v[j] - q[j];
    }
    free(v); free(q);
    return rc;
}

/* ------------------------------------------------------------------------------------
 * Algorithm 1, "On parameter server":
 *   v = delta + (1/n) sum_i decode(msg_i) ;  out = Q[v] ;  delta <- v - decode(out).
 * ---------------------------------------------------------------------------------- */
int dso_server_aggregate_compress(const dso_config *c, uint64_t step, const dso_msg *msgs,
                                  float *delta_s, dso_msg *out)
{
    int64_t d = c->d;
    float *v = (float *)malloc((size_t)(d > 0 ? d : 1) * sizeof *v);
    float *q = (float *)malloc((size_t)(d > 0 ? d : 1) * sizeof *q);
    if (!v || !q) { free(v); free(q); return 2; }
    float inv_n = 1.0f / (float)c->n;
    int rc = 0;
    for (int64_t j = 0; j < d; ++j) v[j] = delta_s[j];
    for (int32_t i = 0; i < c->n && rc == 0; ++i) {
        rc = dso_decode(c, &msgs[i], q);
        for (int64_t j = 0; j < d; ++j) v[j] = fmaf(q[j], inv_n, v[j]);
    }
    if (rc == 0) rc = dso_encode(c, step, DSO_SERVER_STREAM, v, out);
    if (rc == 0) rc = dso_decode(c, out, q);
    if (rc == 0)
        for (int64_t j = 0; j < d; ++j) delta_s[j] = v[j] - q[j];
    free(v); free(q);
    return rc;
}

/* ------------------------------------------------------------------------------------
 * Algorithm 1, "On worker" (second block): x <- x - gamma * decode(msg).
 * With a momentum buffer m (an extension; the paper trains without momentum):
 *   m <- beta m + q ;  x <- x - gamma m.
 * ---------------------------------------------------------------------------------- */
int dso_apply_update(const dso_config *c, const dso_msg *srv, float *x, float *m, float gamma,
                     float beta)
{
    int64_t d = c->d;
    float *q = (float *)malloc((size_t)(d > 0 ? d : 1) * sizeof *q);
    if (!q) return 2;
    int rc = dso_decode(c, srv, q);
    if (rc == 0) {
        for (int64_t j = 0; j < d; ++j) {
            if (m) {
                m[j] = fmaf(beta, m[j], q[j]);
                x[j] = fmaf(-gamma, m[j], x[j]);
            } else {
                x[j] = fmaf(-gamma, q[j], x[j]);
            }
        }
    }
    free(q);
    return rc;
}
