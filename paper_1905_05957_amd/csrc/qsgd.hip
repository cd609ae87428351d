// Randomised quantisation kernels (Section 3.2 "Randomized Quantization" of the
// DoubleSqueeze paper: a value between two neighbouring representable points goes to the
// upper one with probability proportional to its distance from the lower one, which is
// unbiased), in the bucketed QSGD form: per bucket an L2 norm, s uniform levels
// {0..s} * norm/s as 4-bit codes, the sign in a separate bit plane.
//
// Rounding draws come from Philox4x32-10 with counter (j >> 2, 0, stream, lo32(step)) and
// key (lo32(seed), hi32(seed) ^ hi32(step)): one block serves the four consecutive elements
// a thread owns, word c for element 4*(j>>2) + c.  stream = worker index, 0xFFFFFFFF on
// the server.
//
// Buckets are powers of two from 64 to 2048 elements, so a 2048-element tile holds whole
// buckets and a bucket is a fixed group of lanes: sum v^2 (fp64, exact products) by a
// segmented butterfly inside a wavefront and, for buckets above 256 elements, a fixed-order
// combine of wavefront sums through LDS.  One pass over HBM: v = g + delta, norm, codes,
// sign bits and delta' = v - Q[v] all from registers.
#include "ds_device.h"
#include "ds_internal.h"

using namespace ds;

namespace {

constexpr uint32_t kServerStream = 0xFFFFFFFFu;
constexpr int kUnitGroup = 64;  // workers whose decode units are staged in LDS at a time

struct QParams {
    int64_t d;
    int32_t bucket;       // elements per bucket, power of two in [64, 2048]
    int32_t bshift;       // log2(bucket)
    int32_t s;            // levels
    uint32_t key0, key1;  // Philox key (step's high word folded in)
    uint32_t step_lo;
    int64_t W, Bq;
};

// Sum of x over the lanes of this thread's bucket (16 lanes or more, a power of two); every
// lane of the bucket returns it.  lds: kWaves doubles.
__device__ __forceinline__ double bucket_sum(double x, int lanes_per_bucket, double *lds)
{
    x = row_sum(x);
    if (lanes_per_bucket >= 32) x = pair_row_sum<16>(x);
    if (lanes_per_bucket >= 64) x = pair_row_sum<32>(x);
    if (lanes_per_bucket <= 64) return x;
    if (lane_id() == 0) lds[wave_id()] = x;
    __syncthreads();
    const int wpb = lanes_per_bucket >> 6;            // wavefronts per bucket, a power of two
    const int first = wave_id() & ~(wpb - 1);
    double t = lds[first];
    for (int i = 1; i < wpb; ++i) t += lds[first + i];
    return t;
}

// Quantise the four values a thread holds; returns the decoded values q, hands back
// err = v - q and writes codes, sign bits and the bucket norm.  Every thread of the workgroup
// calls it (cross-lane exchanges and barriers inside).
__device__ __forceinline__ f32x4 quantise4(f32x4 v, int64_t e, uint32_t stream, const QParams &P,
                                           uint8_t *__restrict__ levels_row, uint64_t *__restrict__ words_row,
                                           float *__restrict__ norms_row, double *lds, uint32_t *sw_lds, f32x4 &err)
{
    const int lpb = P.bucket >> 2;
    const double ss = ((static_cast<double>(v.x) * static_cast<double>(v.x) +
                        static_cast<double>(v.y) * static_cast<double>(v.y)) +
                       static_cast<double>(v.z) * static_cast<double>(v.z)) +
                      static_cast<double>(v.w) * static_cast<double>(v.w);
    const float norm = static_cast<float>(sqrt(bucket_sum(ss, lpb, lds)));
    const bool live = e < P.d;
    if (live && (threadIdx.x & (lpb - 1)) == 0) norms_row[e >> P.bshift] = norm;
    // The two correctly rounded divisions a bucket needs, s / norm (to quantise) and norm / s (to
    // decode), in one: even lanes form the first, odd lanes the second, and each lane then reads
    // both from its pair (a pair of lanes lies in one bucket).
    const float sf = static_cast<float>(P.s);
    const bool odd = (threadIdx.x & 1) != 0;
    const float quot = __fdiv_rn(odd ? norm : sf, odd ? sf : norm);
    const float inv = __uint_as_float(dpp_u32<0xA0>(__float_as_uint(quot)));    // quad_perm [0,0,2,2]
    const float unit = __uint_as_float(dpp_u32<0xF5>(__float_as_uint(quot)));   // quad_perm [1,1,3,3]

    uint32_t code[4] = {0u, 0u, 0u, 0u};
    if (live && norm > 0.f) {
        const uint32_t blk = static_cast<uint32_t>(e >> 2);
        const u32x4 rnd = philox4x32_10(u32x4{blk, 0u, stream, P.step_lo}, P.key0, P.key1);
        const float vv[4] = {v.x, v.y, v.z, v.w};
        const uint32_t rr[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float r = fabsf(vv[c]) * inv;
            // r >= 0: r - floor(r) is exact and is what the fraction instruction returns; the
            // conversion truncates, which is floor(r)
            const float p = __builtin_amdgcn_fractf(r);
            const float u = static_cast<float>(rr[c] >> 8) * 0x1p-24f;
            int k = static_cast<int>(r) + ((u < p) ? 1 : 0);
            k = (k > P.s) ? P.s : k;
            code[c] = static_cast<uint32_t>(k);
        }
    }
    // 4-bit codes: element j in byte j >> 1, low nibble for even j
    if (live) {
        const uint32_t packed = code[0] | (code[1] << 4) | (code[2] << 8) | (code[3] << 12);
        uint8_t *dst = levels_row + (e >> 1);
        if (e + 4 <= P.d && (reinterpret_cast<uintptr_t>(dst) & 1u) == 0) {
            *reinterpret_cast<uint16_t *>(dst) = static_cast<uint16_t>(packed);
        } else {
            dst[0] = static_cast<uint8_t>(packed);
            if (e + 2 < P.d) dst[1] = static_cast<uint8_t>(packed >> 8);
        }
    }
    stash_sign_words(sw_lds, wave_sign_word(v.x < 0.f, v.y < 0.f, v.z < 0.f, v.w < 0.f));
    __syncthreads();
    flush_sign_words(sw_lds, words_row, (e >> 11) << 11, P.W * 64);
    // decoded message q = +-(code * norm/s) with the sign of v, and v - q = +-(|v| - code * norm/s)
    // with the same sign: the magnitudes are subtracted and the sign bit of v is put back (for
    // v = -0, where q = +0, that is -0 - 0 = -0 as well)
    const float mag[4] = {static_cast<float>(code[0]) * unit, static_cast<float>(code[1]) * unit,
                          static_cast<float>(code[2]) * unit, static_cast<float>(code[3]) * unit};
    const float vv[4] = {v.x, v.y, v.z, v.w};
    float qq[4], ee[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint32_t sb = __float_as_uint(vv[c]) & 0x80000000u;
        qq[c] = (vv[c] < 0.f) ? -mag[c] : mag[c];
        ee[c] = __uint_as_float(__float_as_uint(fabsf(vv[c]) - mag[c]) ^ sb);
    }
    err = f32x4{ee[0], ee[1], ee[2], ee[3]};
    return f32x4{qq[0], qq[1], qq[2], qq[3]};
}

// The four 4-bit codes of elements e..e+3 (e a multiple of 4, e < d).
__device__ __forceinline__ uint32_t load_codes4(const uint8_t *__restrict__ levels_row, int64_t e, int64_t d)
{
    const uint8_t *src = levels_row + (e >> 1);
    if (e + 4 <= d && (reinterpret_cast<uintptr_t>(src) & 1u) == 0) return *reinterpret_cast<const uint16_t *>(src);
    uint32_t r = src[0];
    if (e + 2 < d) r |= static_cast<uint32_t>(src[1]) << 8;
    return r;
}

// +-(code * unit): the sign bit of the magnitude is flipped where the element's bit of `nib`
// is set (what "bit ? -mag : mag" does, without compare and select).
__device__ __forceinline__ f32x4 decode4(uint32_t codes, uint32_t nib, float unit)
{
    f32x4 q;
    q.x = __uint_as_float(__float_as_uint(static_cast<float>(codes & 15u) * unit) ^ ((nib << 31) & 0x80000000u));
    q.y = __uint_as_float(__float_as_uint(static_cast<float>((codes >> 4) & 15u) * unit) ^ ((nib << 30) & 0x80000000u));
    q.z = __uint_as_float(__float_as_uint(static_cast<float>((codes >> 8) & 15u) * unit) ^ ((nib << 29) & 0x80000000u));
    q.w = __uint_as_float(__float_as_uint(static_cast<float>((codes >> 12) & 15u) * unit) ^ ((nib << 28) & 0x80000000u));
    return q;
}

// Worker block of Algorithm 1 with Q = randomised quantisation.  NOFB: without compensation,
// v = g; no error buffer is touched.  TPW tiles per workgroup, all loads issued before the
// first is used.
template <bool BF16, bool NOFB, int TPW>
__global__ __launch_bounds__(kBlock) void k_qsgd_worker(const void *g, int64_t gs, float *delta, int64_t dstr,
                                                        QParams P, uint8_t *levels, uint64_t *words, float *norms)
{
    __shared__ double lds[TPW][kWaves];
    __shared__ __attribute__((aligned(16))) uint32_t sw_lds[TPW][kWaves * 8];
    const int row = blockIdx.y;
    const void *grow = BF16 ? static_cast<const void *>(static_cast<const uint16_t *>(g) + row * gs)
                            : static_cast<const void *>(static_cast<const float *>(g) + row * gs);
    float *drow = NOFB ? nullptr : delta + row * dstr;
    const bool gvec = BF16 ? aligned8(grow) : aligned16(grow);
    const bool dvec = aligned16(drow);
    f32x4 v[TPW];
#pragma unroll
    for (int c = 0; c < TPW; ++c) {
        const int64_t e = (static_cast<int64_t>(blockIdx.x) * TPW + c) * kTile + threadIdx.x * 4;
        v[c] = ld4_grad<BF16>(grow, e, P.d, gvec);
        if constexpr (!NOFB) v[c] = v[c] + ld4_stream(drow, e, P.d, dvec);
    }
#pragma unroll
    for (int c = 0; c < TPW; ++c) {
        const int64_t tile_first = (static_cast<int64_t>(blockIdx.x) * TPW + c) * kTile;
        if (tile_first >= P.d) break;                                  // uniform over the workgroup
        const int64_t e = tile_first + threadIdx.x * 4;
        f32x4 err;
        quantise4(v[c], e, static_cast<uint32_t>(row), P, levels + row * ((P.d + 1) / 2), words + row * P.W,
                  norms + row * P.Bq, lds[c], sw_lds[c], err);
        if constexpr (!NOFB)
            if (e < P.d) st4_stream(drow, e, P.d, dvec, err);
    }
}

// Parameter-server block: v = delta_s + (1/n) sum_i decode(msg_i) as the fma chain over
// workers in ascending order, then the same quantiser on the server's stream.
// UPD: 0 = that block alone; 1, 2 = followed by the model update of Algorithm 1 for the same
// elements (2: through the momentum buffer) from the decoded values the thread already holds.
// delta_s == nullptr: no server error (chain from +0, nothing stored back).
// SID: the server does not compress: the average is written to dense_out (if not null) and / or
// applied to x, m (if x is not null), and nothing else happens.
template <int UPD, bool SID>
__global__ __launch_bounds__(kBlock) void k_qsgd_server(const uint8_t *levels_in, const uint64_t *words_in,
                                                        const float *norms_in, int n, float inv_n, float *delta_s,
                                                        QParams P, uint8_t *levels_out, uint64_t *words_out,
                                                        float *norms_out, float *x, float *m, float gamma, float beta,
                                                        float *dense_out)
{
    __shared__ double lds[kWaves];
    __shared__ __attribute__((aligned(16))) uint32_t sw_lds[kWaves * 8];
    __shared__ float units[kUnitGroup * (kTile / 64)];
    const int64_t tile_base = static_cast<int64_t>(blockIdx.x) * kTile;
    const int64_t e = tile_base + threadIdx.x * 4;
    const bool dvec = aligned16(delta_s);
    const int bpt = kTile >> P.bshift;                      // buckets per tile
    const int64_t b0 = tile_base >> P.bshift;
    const int my_b = (threadIdx.x * 4) >> P.bshift;
    const int64_t lev_stride = (P.d + 1) / 2;
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    if (delta_s) a = ld4_stream(delta_s, e, P.d, dvec);
    f32x4 xv = {0.f, 0.f, 0.f, 0.f}, mv = {0.f, 0.f, 0.f, 0.f};      // fetched up front, beside the error
    if constexpr (UPD != 0) xv = ld4_stream(x, e, P.d, aligned16(x));
    if constexpr (UPD == 2) mv = ld4_stream(m, e, P.d, aligned16(m));
    for (int i0 = 0; i0 < n; i0 += kUnitGroup) {
        const int cnt = (n - i0 < kUnitGroup) ? n - i0 : kUnitGroup;
        __syncthreads();
        for (int t = threadIdx.x; t < cnt * bpt; t += kBlock) {
            const int i = t / bpt, b = t - i * bpt;
            const int64_t B = b0 + b;
            units[t] = (B < P.Bq) ? __fdiv_rn(norms_in[(i0 + i) * P.Bq + B], static_cast<float>(P.s)) : 0.f;
        }
        __syncthreads();
        // Messages of the wavefront's 256 elements: 128 bytes of codes and 32 bytes of sign
        // bits per worker.  Fast route (whole wavefront in range, 4-byte aligned code rows):
        // eight workers at a time, one 32-bit load fetches the sign words of all eight
        // (lane L: word L & 7 of worker L >> 3) and four 32-bit loads fetch the codes of two
        // workers each (lane L: word L & 31 of worker L >> 5); ds_bpermute then hands every
        // lane its own nibble and 16-bit code group.  Other wavefronts load per lane.
        const int lane = lane_id();
        const int64_t wave_first = tile_base + wave_id() * 256;
        const bool fast = (wave_first + 256 <= P.d) && ((lev_stride & 3) == 0) &&
                          ((reinterpret_cast<uintptr_t>(levels_in) & 3u) == 0);
        if (fast) {
            for (int j0 = 0; j0 < cnt; j0 += 8) {
                const int nb = (cnt - j0 < 8) ? cnt - j0 : 8;
                uint32_t sw = 0u;
                if ((lane >> 3) < nb)
                    sw = reinterpret_cast<const uint32_t *>(words_in + (i0 + j0 + (lane >> 3)) * P.W)[(wave_first >> 5) + (lane & 7)];
                uint32_t cw[4];
#pragma unroll
                for (int p2 = 0; p2 < 4; ++p2) {
                    const int wk = 2 * p2 + (lane >> 5);
                    cw[p2] = 0u;
                    if (wk < nb)
                        cw[p2] = reinterpret_cast<const uint32_t *>(levels_in + (i0 + j0 + wk) * lev_stride + (wave_first >> 1))[lane & 31];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (j >= nb) break;                      // uniform
                    const uint32_t nib = (__shfl(sw, j * 8 + (lane >> 3), 64) >> (4 * (lane & 7))) & 15u;
                    const uint32_t c32 = __shfl(cw[j >> 1], (j & 1) * 32 + (lane >> 1), 64);
                    const uint32_t codes = (c32 >> (16 * (lane & 1))) & 0xFFFFu;
                    a = fma4(inv_n, decode4(codes, nib, units[(j0 + j) * bpt + my_b]), a);
                }
            }
        } else if (e < P.d) {
            for (int i = 0; i < cnt; ++i) {
                const int64_t w = i0 + i;
                const uint32_t codes = load_codes4(levels_in + w * lev_stride, e, P.d);
                const uint32_t nib = load_sign_nibble(words_in + w * P.W, e);
                const f32x4 q = decode4(codes, nib, units[i * bpt + my_b]);
                a = fma4(inv_n, q, a);   // fma(q, 1/n, acc): the product commutes
            }
        }
    }
    a = zero_past(a, e, P.d);
    if constexpr (SID) {
        if (e < P.d) put_average4(a, e, P.d, dense_out, x, m, gamma, beta);
        return;
    }
    f32x4 err;
    f32x4 q = quantise4(a, e, kServerStream, P, levels_out, words_out, norms_out, lds, sw_lds, err);
    if (delta_s && e < P.d) st4_stream(delta_s, e, P.d, dvec, err);
    if constexpr (UPD != 0) {
        if (e < P.d) {
            q = zero_past(q, e, P.d);
            if constexpr (UPD == 2) {
                q = fma4(beta, mv, q);
                st4_stream(m, e, P.d, aligned16(m), q);
            }
            st4_stream(x, e, P.d, aligned16(x), fma4(-gamma, q, xv));
        }
    }
}

template <bool MOM, bool DECODE_ONLY>
__global__ __launch_bounds__(kBlock) void k_qsgd_update(const uint8_t *levels, const uint64_t *words,
                                                        const float *norms, QParams P, float *x, float *m,
                                                        float gamma, float beta)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * kTile + threadIdx.x * 4;
    if (e >= P.d) return;
    const float unit = __fdiv_rn(norms[e >> P.bshift], static_cast<float>(P.s));
    const f32x4 q = decode4(load_codes4(levels, e, P.d), load_sign_nibble(words, e), unit);
    apply_q4<MOM, DECODE_ONLY>(zero_past(q, e, P.d), e, P.d, x, m, gamma, beta);
}

bool bucket_ok(int32_t b) { return b >= 64 && b <= kTile && (b & (b - 1)) == 0; }

QParams make_params(const ds_ctx *c, uint64_t step)
{
    QParams P;
    P.d = c->cfg.d;
    P.bucket = c->cfg.bucket;
    P.bshift = 0;
    while ((1 << P.bshift) < P.bucket) ++P.bshift;
    P.s = c->cfg.levels;
    P.key0 = static_cast<uint32_t>(c->cfg.seed);
    P.key1 = static_cast<uint32_t>(c->cfg.seed >> 32) ^ static_cast<uint32_t>(step >> 32);
    P.step_lo = static_cast<uint32_t>(step);
    P.W = c->W;
    P.Bq = c->S;
    return P;
}

}  // namespace

ds_status_t ds_qsgd_worker(ds_ctx *c, uint64_t step, const void *g, int64_t gs, float *delta, int64_t dstr,
                           const ds_payload_t *out, hipStream_t st)
{
    if (!bucket_ok(c->cfg.bucket)) return DS_ERR_UNSUPPORTED;
    const QParams P = make_params(c, step);
    dim3 grid(static_cast<unsigned>(c->n_tiles), static_cast<unsigned>(c->cfg.n));
    // two tiles per workgroup: 1.5 % on the 16 x 25.6 M workload (fewer, longer-lived workgroups)
    constexpr int TPW = 2;
    grid.x = static_cast<unsigned>((c->n_tiles + TPW - 1) / TPW);
    const bool bf16 = c->cfg.grad_dtype == DS_BF16;
    if (bf16 && c->nofb) k_qsgd_worker<true, true, TPW><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, P, out->levels, out->sign_words, out->scales);
    else if (bf16) k_qsgd_worker<true, false, TPW><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, P, out->levels, out->sign_words, out->scales);
    else if (c->nofb) k_qsgd_worker<false, true, TPW><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, P, out->levels, out->sign_words, out->scales);
    else k_qsgd_worker<false, false, TPW><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, P, out->levels, out->sign_words, out->scales);
    return ds_launch_status();
}

// x != nullptr: the model update for the same elements in the same kernel.
ds_status_t ds_qsgd_server(ds_ctx *c, uint64_t step, const ds_payload_t *in, float *delta_s,
                           const ds_payload_t *out, hipStream_t st, float *x, float *m, float gamma, float beta)
{
    if (!bucket_ok(c->cfg.bucket)) return DS_ERR_UNSUPPORTED;
    const QParams P = make_params(c, step);
    const unsigned blocks = static_cast<unsigned>(c->n_tiles);
    if (!x)
        k_qsgd_server<0, false><<<blocks, kBlock, 0, st>>>(in->levels, in->sign_words, in->scales, c->cfg.n, c->inv_n, delta_s, P,
                                                           out->levels, out->sign_words, out->scales, x, m, gamma, beta, nullptr);
    else if (!m)
        k_qsgd_server<1, false><<<blocks, kBlock, 0, st>>>(in->levels, in->sign_words, in->scales, c->cfg.n, c->inv_n, delta_s, P,
                                                           out->levels, out->sign_words, out->scales, x, m, gamma, beta, nullptr);
    else
        k_qsgd_server<2, false><<<blocks, kBlock, 0, st>>>(in->levels, in->sign_words, in->scales, c->cfg.n, c->inv_n, delta_s, P,
                                                           out->levels, out->sign_words, out->scales, x, m, gamma, beta, nullptr);
    return ds_launch_status();
}

ds_status_t ds_qsgd_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st)
{
    if (!bucket_ok(c->cfg.bucket)) return DS_ERR_UNSUPPORTED;
    const QParams P = make_params(c, 0);
    k_qsgd_server<0, true><<<static_cast<unsigned>(c->n_tiles), kBlock, 0, st>>>(
        in->levels, in->sign_words, in->scales, c->cfg.n, c->inv_n, nullptr, P, nullptr, nullptr, nullptr, u.x, u.m, u.gamma,
        u.beta, dense_out);
    return ds_launch_status();
}

ds_status_t ds_qsgd_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma, float beta,
                           hipStream_t st)
{
    if (!bucket_ok(c->cfg.bucket)) return DS_ERR_UNSUPPORTED;
    const QParams P = make_params(c, 0);
    const unsigned blocks = static_cast<unsigned>(c->n_tiles);
    if (m)
        k_qsgd_update<true, false><<<blocks, kBlock, 0, st>>>(srv->levels, srv->sign_words, srv->scales, P, x, m, gamma, beta);
    else
        k_qsgd_update<false, false><<<blocks, kBlock, 0, st>>>(srv->levels, srv->sign_words, srv->scales, P, x, m, gamma, beta);
    return ds_launch_status();
}

ds_status_t ds_qsgd_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st)
{
    if (!bucket_ok(c->cfg.bucket)) return DS_ERR_UNSUPPORTED;
    const QParams P = make_params(c, 0);
    k_qsgd_update<false, true><<<static_cast<unsigned>(c->n_tiles), kBlock, 0, st>>>(
        p->levels + row * ((P.d + 1) / 2), p->sign_words + row * P.W, p->scales + row * P.Bq, P, out, nullptr, 0.f, 0.f);
    return ds_launch_status();
}
