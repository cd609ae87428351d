// Clipping compressor (Section 3.2 "Clipping" of the DoubleSqueeze paper): the lower b bits
// of every number's binary representation are set to zero.  The message keeps the upper 32-b
// bits of every element in the smallest of 1, 2 or 4 bytes that holds them (b >= 24,
// b >= 16, otherwise), little endian; b = 16 is the truncation of fp32 to the bf16 grid.
// The error v - Q[v] is the value of the cleared bits and is exact in fp32.
//
// Everything is element-wise, so each of the three calls is one streaming pass with one
// 128-bit load per thread and input stream; the message leaves as one 4*NB-byte store per
// thread.
#include "ds_device.h"
#include "ds_internal.h"

using namespace ds;

namespace {

template <int NB>
__device__ __forceinline__ void store_msg4(uint8_t *__restrict__ row, int64_t e, int64_t d, const uint32_t top[4])
{
    uint8_t *p = row + e * NB;
    if (e + 4 <= d && (reinterpret_cast<uintptr_t>(p) & (4 * NB - 1)) == 0) {
        if constexpr (NB == 1) {
            *reinterpret_cast<uint32_t *>(p) = top[0] | (top[1] << 8) | (top[2] << 16) | (top[3] << 24);
        } else if constexpr (NB == 2) {
            *reinterpret_cast<u32x2 *>(p) = u32x2{top[0] | (top[1] << 16), top[2] | (top[3] << 16)};
        } else {
            *reinterpret_cast<u32x4 *>(p) = u32x4{top[0], top[1], top[2], top[3]};
        }
        return;
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (e + c >= d) break;
        if constexpr (NB == 1) p[c] = static_cast<uint8_t>(top[c]);
        else if constexpr (NB == 2) {               // rows of an odd length start on odd 2-byte boundaries at worst
            p[2 * c] = static_cast<uint8_t>(top[c]);
            p[2 * c + 1] = static_cast<uint8_t>(top[c] >> 8);
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) p[4 * c + t] = static_cast<uint8_t>(top[c] >> (8 * t));
        }
    }
}

// decoded values of four elements; elements past d decode to 0
template <int NB>
__device__ __forceinline__ f32x4 load_msg4(const uint8_t *__restrict__ row, int64_t e, int64_t d)
{
    const uint8_t *p = row + e * NB;
    uint32_t top[4] = {0u, 0u, 0u, 0u};
    if (e + 4 <= d && (reinterpret_cast<uintptr_t>(p) & (4 * NB - 1)) == 0) {
        if constexpr (NB == 1) {
            const uint32_t w = *reinterpret_cast<const uint32_t *>(p);
            top[0] = w & 255u; top[1] = (w >> 8) & 255u; top[2] = (w >> 16) & 255u; top[3] = w >> 24;
        } else if constexpr (NB == 2) {
            const u32x2 w = *reinterpret_cast<const u32x2 *>(p);
            top[0] = w.x & 0xFFFFu; top[1] = w.x >> 16; top[2] = w.y & 0xFFFFu; top[3] = w.y >> 16;
        } else {
            const u32x4 w = *reinterpret_cast<const u32x4 *>(p);
            top[0] = w.x; top[1] = w.y; top[2] = w.z; top[3] = w.w;
        }
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (e + c >= d) break;
#pragma unroll
            for (int t = 0; t < NB; ++t) top[c] |= static_cast<uint32_t>(p[NB * c + t]) << (8 * t);
        }
    }
    constexpr int sh = 32 - 8 * NB;
    return f32x4{__uint_as_float(top[0] << sh), __uint_as_float(top[1] << sh), __uint_as_float(top[2] << sh),
                 __uint_as_float(top[3] << sh)};
}

// Q[v], the message and the error for the four elements of a thread
template <int NB>
__device__ __forceinline__ void clip_store4(f32x4 v, uint32_t mask, int64_t e, int64_t d, uint8_t *__restrict__ msg_row,
                                            float *__restrict__ err_row, bool err_vec)
{
    const uint32_t u[4] = {__float_as_uint(v.x) & mask, __float_as_uint(v.y) & mask, __float_as_uint(v.z) & mask,
                           __float_as_uint(v.w) & mask};
    constexpr int sh = 32 - 8 * NB;
    const uint32_t top[4] = {u[0] >> sh, u[1] >> sh, u[2] >> sh, u[3] >> sh};
    store_msg4<NB>(msg_row, e, d, top);
    const f32x4 q = {__uint_as_float(u[0]), __uint_as_float(u[1]), __uint_as_float(u[2]), __uint_as_float(u[3])};
    if (err_row) st4_stream(err_row, e, d, err_vec, v - q);     // no buffer: no compensation
}

// Algorithm 1, worker block: v = g + delta ; message = Q[v] ; delta <- v - Q[v].
template <bool BF16, int NB>
__global__ __launch_bounds__(kBlock) void k_clip_worker(const void *g, int64_t gs, float *delta, int64_t dstr,
                                                        uint8_t *msg, int64_t d, uint32_t mask)
{
    const int row = blockIdx.y;
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    const void *grow = BF16 ? static_cast<const void *>(static_cast<const uint16_t *>(g) + row * gs)
                            : static_cast<const void *>(static_cast<const float *>(g) + row * gs);
    float *drow = delta ? delta + row * dstr : nullptr;         // null: no compensation, v = g
    const bool gvec = BF16 ? aligned8(grow) : aligned16(grow);
    const bool dvec = aligned16(drow);
    f32x4 v = ld4_grad<BF16>(grow, e, d, gvec);
    if (drow) v = v + ld4_stream(drow, e, d, dvec);
    clip_store4<NB>(v, mask, e, d, msg + static_cast<int64_t>(row) * d * NB, drow, dvec);
}

// Parameter-server block: v = delta_s + (1/n) sum_i Q[v_i] as the chain acc = fma(q_i, 1/n, acc)
// over workers in ascending order, then the same compression.
template <int NB>
__global__ __launch_bounds__(kBlock) void k_clip_server(const uint8_t *msg_in, int n, float inv_n, float *delta_s,
                                                        uint8_t *msg_out, int64_t d, uint32_t mask)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    const bool dvec = aligned16(delta_s);
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    if (delta_s) a = ld4_stream(delta_s, e, d, dvec);           // null: no server error
    for (int i = 0; i < n; ++i) a = fma4(inv_n, load_msg4<NB>(msg_in + static_cast<int64_t>(i) * d * NB, e, d), a);
    clip_store4<NB>(a, mask, e, d, msg_out, delta_s, dvec);
}

// Server that does not compress: the average is the message (written and / or applied).
template <int NB>
__global__ __launch_bounds__(kBlock) void k_clip_server_identity(const uint8_t *msg_in, int n, float inv_n, int64_t d,
                                                                 float *dense_out, ds_update_args u)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < n; ++i) a = fma4(inv_n, load_msg4<NB>(msg_in + static_cast<int64_t>(i) * d * NB, e, d), a);
    put_average4(a, e, d, dense_out, u.x, u.m, u.gamma, u.beta);
}

template <int NB, bool MOM, bool DECODE_ONLY>
__global__ __launch_bounds__(kBlock) void k_clip_update(const uint8_t *msg, float *x, float *m, int64_t d, float gamma,
                                                        float beta)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    apply_q4<MOM, DECODE_ONLY>(load_msg4<NB>(msg, e, d), e, d, x, m, gamma, beta);
}

unsigned blocks4(int64_t d) { return static_cast<unsigned>((d + kBlock * 4 - 1) / (kBlock * 4)); }

uint32_t clip_mask(int bits) { return ~static_cast<uint32_t>((1ull << bits) - 1ull); }

// f(std::integral_constant<int, NB>) for the configured width
template <class F>
void with_bytes(int bits, F f)
{
    if (bits >= 24) f(std::integral_constant<int, 1>{});
    else if (bits >= 16) f(std::integral_constant<int, 2>{});
    else f(std::integral_constant<int, 4>{});
}

}  // namespace

int ds_clip_bytes(int bits) { return bits >= 24 ? 1 : bits >= 16 ? 2 : 4; }

ds_status_t ds_clip_worker(ds_ctx *c, const void *g, int64_t gs, float *delta, int64_t dstr, const ds_payload_t *out,
                           hipStream_t st)
{
    const int bits = c->cfg.levels;
    const dim3 grid(blocks4(c->cfg.d), static_cast<unsigned>(c->cfg.n));
    with_bytes(bits, [&](auto nb) {
        constexpr int NB = decltype(nb)::value;
        if (c->cfg.grad_dtype == DS_BF16)
            k_clip_worker<true, NB><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, out->levels, c->cfg.d, clip_mask(bits));
        else
            k_clip_worker<false, NB><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, out->levels, c->cfg.d, clip_mask(bits));
    });
    return ds_launch_status();
}

ds_status_t ds_clip_server(ds_ctx *c, const ds_payload_t *in, float *delta_s, const ds_payload_t *out, hipStream_t st)
{
    const int bits = c->cfg.levels;
    with_bytes(bits, [&](auto nb) {
        constexpr int NB = decltype(nb)::value;
        k_clip_server<NB><<<blocks4(c->cfg.d), kBlock, 0, st>>>(in->levels, c->cfg.n, c->inv_n, delta_s, out->levels,
                                                               c->cfg.d, clip_mask(bits));
    });
    return ds_launch_status();
}

ds_status_t ds_clip_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st)
{
    with_bytes(c->cfg.levels, [&](auto nb) {
        constexpr int NB = decltype(nb)::value;
        k_clip_server_identity<NB><<<blocks4(c->cfg.d), kBlock, 0, st>>>(in->levels, c->cfg.n, c->inv_n, c->cfg.d, dense_out, u);
    });
    return ds_launch_status();
}

ds_status_t ds_clip_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma, float beta, hipStream_t st)
{
    with_bytes(c->cfg.levels, [&](auto nb) {
        constexpr int NB = decltype(nb)::value;
        if (m) k_clip_update<NB, true, false><<<blocks4(c->cfg.d), kBlock, 0, st>>>(srv->levels, x, m, c->cfg.d, gamma, beta);
        else k_clip_update<NB, false, false><<<blocks4(c->cfg.d), kBlock, 0, st>>>(srv->levels, x, m, c->cfg.d, gamma, beta);
    });
    return ds_launch_status();
}

ds_status_t ds_clip_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st)
{
    with_bytes(c->cfg.levels, [&](auto nb) {
        constexpr int NB = decltype(nb)::value;
        k_clip_update<NB, false, true><<<blocks4(c->cfg.d), kBlock, 0, st>>>(
            p->levels + static_cast<int64_t>(row) * c->cfg.d * NB, out, nullptr, c->cfg.d, 0.f, 0.f);
    });
    return ds_launch_status();
}
