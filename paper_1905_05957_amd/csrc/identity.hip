// Identity compressor (Section 5.1 "Vanilla SGD"): the message is the dense vector.  With
// it the step is plain synchronous parallel SGD and both error buffers stay zero; it is the
// test mode that ties the three calls to a textbook routine.
#include "ds_device.h"
#include "ds_internal.h"

using namespace ds;

namespace {

template <bool BF16>
__global__ __launch_bounds__(kBlock) void k_identity_worker(const void *g, int64_t gs, float *delta,
                                                            int64_t dstr, float *dense, int64_t d)
{
    const int row = blockIdx.y;
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    const void *grow = BF16 ? static_cast<const void *>(static_cast<const uint16_t *>(g) + row * gs)
                            : static_cast<const void *>(static_cast<const float *>(g) + row * gs);
    float *drow = delta + row * dstr;
    float *orow = dense + row * d;
    const bool gvec = BF16 ? aligned8(grow) : aligned16(grow);
    const bool dvec = aligned16(drow), ovec = aligned16(orow);
    const f32x4 v = ld4_grad<BF16>(grow, e, d, gvec) + ld4(drow, e, d, dvec);
    st4(orow, e, d, ovec, v);          // Q[v] = v
    st4(drow, e, d, dvec, v - v);      // delta <- v - Q[v]
}

__global__ __launch_bounds__(kBlock) void k_identity_server(const float *dense_in, int n, float inv_n,
                                                            float *delta_s, float *dense_out, int64_t d)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    const bool dvec = aligned16(delta_s), ovec = aligned16(dense_out);
    f32x4 a = ld4(delta_s, e, d, dvec);
    for (int i = 0; i < n; ++i) {
        const float *irow = dense_in + i * d;
        const f32x4 q = ld4(irow, e, d, aligned16(irow));
        a.x = __fmaf_rn(q.x, inv_n, a.x); a.y = __fmaf_rn(q.y, inv_n, a.y);
        a.z = __fmaf_rn(q.z, inv_n, a.z); a.w = __fmaf_rn(q.w, inv_n, a.w);
    }
    st4(dense_out, e, d, ovec, a);
    st4(delta_s, e, d, dvec, a - a);
}

template <bool MOM, bool DECODE_ONLY>
__global__ __launch_bounds__(kBlock) void k_identity_update(const float *q_in, float *x, float *m,
                                                            int64_t d, float gamma, float beta)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    const bool xvec = aligned16(x);
    f32x4 q = ld4(q_in, e, d, aligned16(q_in));
    if constexpr (DECODE_ONLY) {
        st4(x, e, d, xvec, q);
    } else {
        f32x4 xv = ld4(x, e, d, xvec);
        if constexpr (MOM) {
            const bool mvec = aligned16(m);
            f32x4 mv = ld4(m, e, d, mvec);
            mv.x = __fmaf_rn(beta, mv.x, q.x); mv.y = __fmaf_rn(beta, mv.y, q.y);
            mv.z = __fmaf_rn(beta, mv.z, q.z); mv.w = __fmaf_rn(beta, mv.w, q.w);
            st4(m, e, d, mvec, mv);
            q = mv;
        }
        xv.x = __fmaf_rn(-gamma, q.x, xv.x); xv.y = __fmaf_rn(-gamma, q.y, xv.y);
        xv.z = __fmaf_rn(-gamma, q.z, xv.z); xv.w = __fmaf_rn(-gamma, q.w, xv.w);
        st4(x, e, d, xvec, xv);
    }
}

unsigned blocks4(int64_t d) { return static_cast<unsigned>((d + kBlock * 4 - 1) / (kBlock * 4)); }

// Measurement aid: a plain copy in the shape of the library's dense passes (512 threads, one
// non-temporal 128-bit load and store per thread).
__global__ __launch_bounds__(kBlock) void k_probe_copy(const f32x4 *__restrict__ src, f32x4 *__restrict__ dst, int64_t n16)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace

extern "C" ds_status_t ds_probe_copy(const void *src, void *dst, size_t bytes, void *hip_stream)
{
    if (!src || !dst) return DS_ERR_NULL;
    if (bytes == 0 || (bytes & 15u) != 0 || bytes > (static_cast<size_t>(1) << 40)) return DS_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return DS_ERR_ALIGN;
    const int64_t n16 = static_cast<int64_t>(bytes / 16);
    k_probe_copy<<<static_cast<unsigned>((n16 + kBlock - 1) / kBlock), kBlock, 0, static_cast<hipStream_t>(hip_stream)>>>(
        static_cast<const f32x4 *>(src), static_cast<f32x4 *>(dst), n16);
    return ds_launch_status();
}

ds_status_t ds_identity_worker(ds_ctx *c, const void *g, int64_t gs, float *delta, int64_t dstr,
                               const ds_payload_t *out, hipStream_t st)
{
    dim3 grid(blocks4(c->cfg.d), static_cast<unsigned>(c->cfg.n));
    if (c->cfg.grad_dtype == DS_BF16)
        k_identity_worker<true><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, out->dense, c->cfg.d);
    else
        k_identity_worker<false><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, out->dense, c->cfg.d);
    return ds_launch_status();
}

ds_status_t ds_identity_server(ds_ctx *c, const ds_payload_t *in, float *delta_s, const ds_payload_t *out,
                               hipStream_t st)
{
    k_identity_server<<<blocks4(c->cfg.d), kBlock, 0, st>>>(in->dense, c->cfg.n, c->inv_n, delta_s, out->dense,
                                                            c->cfg.d);
    return ds_launch_status();
}

ds_status_t ds_identity_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma, float beta,
                               hipStream_t st)
{
    if (m)
        k_identity_update<true, false><<<blocks4(c->cfg.d), kBlock, 0, st>>>(srv->dense, x, m, c->cfg.d, gamma, beta);
    else
        k_identity_update<false, false><<<blocks4(c->cfg.d), kBlock, 0, st>>>(srv->dense, x, m, c->cfg.d, gamma, beta);
    return ds_launch_status();
}

ds_status_t ds_identity_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st)
{
    k_identity_update<false, true><<<blocks4(c->cfg.d), kBlock, 0, st>>>(p->dense + row * c->cfg.d, out, nullptr,
                                                                        c->cfg.d, 0.f, 0.f);
    return ds_launch_status();
}
