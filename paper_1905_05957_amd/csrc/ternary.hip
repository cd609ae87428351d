// Ternary quantiser (Section 5.1 of the DoubleSqueeze paper, the compressor of its "QSGD"
// comparison system): every element becomes a code in {-1, 0, +1}.  With m the largest
// absolute value of the row, element e becomes sign(e) with probability |e| / m, decided by
// u < |e| / m with the element's 24-bit uniform (Philox4x32-10, counter (j >> 2, 0, stream,
// lo32(step)), key (lo32(seed), hi32(seed) ^ hi32(step)), word j & 3), and 0 otherwise.  One
// scale per row, sum |v| / number of non-zero codes ("magnitude of original gradient over
// magnitude of compressed gradient", read as l1), so that code * scale has the l1 magnitude of v.
//
// The comparison system runs without compensation and with a server that does not compress,
// and that is the mode built here: v = g, no error buffer.  The row-wide maximum has to be
// known before the first code, so the worker call looks at g twice:
//   stats    per 2048-element tile: max |v| and sum |v| (fp64)
//   rowstat  per row: the maximum, and the sum in a fixed order
//   encode   codes from the second look: two bit planes packed like the sign words, kept count per tile
//   scale    per row: sum / count, rounded once
// The message is 2 bits per element: plane `levels` (bit j = code_j is not 0), plane
// `sign_words` (bit j = code_j is -1), one fp32 scale.
#include "ds_device.h"
#include "ds_internal.h"

#include <new>

using namespace ds;

struct ds_tern_scratch {
    float *pmax;       // [n][n_tiles]
    double *psum;      // [n][n_tiles]
    uint32_t *pcnt;    // [n][n_tiles]
    float *rowmax;     // [n]
    double *rowsum;    // [n]
};

namespace {

template <bool BF16>
__device__ __forceinline__ const void *grad_row(const void *g, int64_t gs, int row)
{
    if constexpr (BF16) return static_cast<const uint16_t *>(g) + row * gs;
    else return static_cast<const float *>(g) + row * gs;
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void k_tern_stats(const void *g, int64_t gs, int64_t d, float *pmax, double *psum)
{
    __shared__ double lds[kWaves];
    __shared__ float mx[kWaves];
    const int row = blockIdx.y;
    const int64_t e = static_cast<int64_t>(blockIdx.x) * kTile + threadIdx.x * 4;
    const void *grow = grad_row<BF16>(g, gs, row);
    const f32x4 v = ld4_grad<BF16>(grow, e, d, BF16 ? aligned8(grow) : aligned16(grow));   // zero past d
    const float a0 = fabsf(v.x), a1 = fabsf(v.y), a2 = fabsf(v.z), a3 = fabsf(v.w);
    float m = fmaxf(fmaxf(a0, a1), fmaxf(a2, a3));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    if (lane_id() == 0) mx[wave_id()] = m;
    const double total = block_sum(((static_cast<double>(a0) + static_cast<double>(a1)) + static_cast<double>(a2)) +
                                       static_cast<double>(a3), lds, false);   // its barrier also covers mx
    if (threadIdx.x == 0) {
        float t = mx[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) t = fmaxf(t, mx[w]);
        pmax[row * gridDim.x + blockIdx.x] = t;
        psum[row * gridDim.x + blockIdx.x] = total;
    }
}

// One workgroup per row: maximum and, in a fixed order, the sum over the row's tiles.
__global__ __launch_bounds__(kBlock) void k_tern_rowstat(const float *pmax, const double *psum, int64_t n_tiles,
                                                         float *rowmax, double *rowsum)
{
    __shared__ double sm[kBlock];
    __shared__ float mm[kBlock];
    const int row = blockIdx.x;
    double acc = 0.0;
    float m = 0.f;
    for (int64_t t = threadIdx.x; t < n_tiles; t += kBlock) {
        acc += psum[row * n_tiles + t];
        m = fmaxf(m, pmax[row * n_tiles + t]);
    }
    sm[threadIdx.x] = acc;
    mm[threadIdx.x] = m;
    __syncthreads();
    for (int o = kBlock / 2; o > 0; o >>= 1) {
        if (threadIdx.x < o) {
            sm[threadIdx.x] += sm[threadIdx.x + o];
            mm[threadIdx.x] = fmaxf(mm[threadIdx.x], mm[threadIdx.x + o]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) { rowmax[row] = mm[0]; rowsum[row] = sm[0]; }
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void k_tern_encode(const void *g, int64_t gs, int64_t d, const float *rowmax,
                                                        uint32_t key0, uint32_t key1, uint32_t step_lo, uint64_t *neg,
                                                        uint64_t *nz, int64_t W, uint32_t *pcnt)
{
    __shared__ __attribute__((aligned(16))) uint32_t sw_neg[kWaves * 8], sw_nz[kWaves * 8];
    __shared__ uint32_t cnt[kWaves];
    const int row = blockIdx.y;
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kTile;
    const int64_t e = base + threadIdx.x * 4;
    const void *grow = grad_row<BF16>(g, gs, row);
    const f32x4 v = ld4_grad<BF16>(grow, e, d, BF16 ? aligned8(grow) : aligned16(grow));
    const float m = rowmax[row];
    bool keep[4] = {false, false, false, false};
    if (e < d && m > 0.f) {
        const u32x4 rnd = philox4x32_10(u32x4{static_cast<uint32_t>(e >> 2), 0u, static_cast<uint32_t>(row), step_lo}, key0, key1);
        const float vv[4] = {v.x, v.y, v.z, v.w};
        const uint32_t rr[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float p = __fdiv_rn(fabsf(vv[c]), m);
            const float u = static_cast<float>(rr[c] >> 8) * 0x1p-24f;
            keep[c] = (e + c < d) && (u < p);
        }
    }
    stash_sign_words(sw_nz, wave_sign_word(keep[0], keep[1], keep[2], keep[3]));
    stash_sign_words(sw_neg, wave_sign_word(keep[0] && v.x < 0.f, keep[1] && v.y < 0.f, keep[2] && v.z < 0.f, keep[3] && v.w < 0.f));
    const uint32_t kept = wave_sum_u32(static_cast<uint32_t>(keep[0]) + keep[1] + keep[2] + keep[3]);
    if (lane_id() == 0) cnt[wave_id()] = kept;
    __syncthreads();
    flush_sign_words(sw_nz, nz + row * W, base, W * 64);
    flush_sign_words(sw_neg, neg + row * W, base, W * 64);
    if (threadIdx.x == 0) {
        uint32_t t = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) t += cnt[w];
        pcnt[row * gridDim.x + blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(kBlock) void k_tern_scale(const uint32_t *pcnt, const double *rowsum, int64_t n_tiles, float *scales)
{
    __shared__ unsigned long long sm[kBlock];
    const int row = blockIdx.x;
    unsigned long long acc = 0;
    for (int64_t t = threadIdx.x; t < n_tiles; t += kBlock) acc += pcnt[row * n_tiles + t];
    sm[threadIdx.x] = acc;
    __syncthreads();
    for (int o = kBlock / 2; o > 0; o >>= 1) {
        if (threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) scales[row] = sm[0] ? static_cast<float>(rowsum[row] / static_cast<double>(sm[0])) : 0.f;
}

// code * scale of elements e..e+3 of one message
__device__ __forceinline__ f32x4 tern_decode4(const uint64_t *neg_row, const uint64_t *nz_row, float s, int64_t e)
{
    const uint32_t kb = load_sign_nibble(nz_row, e), nb = load_sign_nibble(neg_row, e);
    f32x4 q;
    q.x = (kb & 1u) ? ((nb & 1u) ? -s : s) : 0.f;
    q.y = (kb & 2u) ? ((nb & 2u) ? -s : s) : 0.f;
    q.z = (kb & 4u) ? ((nb & 4u) ? -s : s) : 0.f;
    q.w = (kb & 8u) ? ((nb & 8u) ? -s : s) : 0.f;
    return q;
}

// Server that does not compress: a = (1/n) sum_i Q[v_i] by the chain from +0.
__global__ __launch_bounds__(kBlock) void k_tern_server_identity(const uint64_t *neg, const uint64_t *nz, const float *scales,
                                                                 int n, float inv_n, int64_t d, int64_t W, float *dense_out,
                                                                 ds_update_args u)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < n; ++i) a = fma4(inv_n, tern_decode4(neg + i * W, nz + i * W, scales[i], e), a);
    put_average4(zero_past(a, e, d), e, d, dense_out, u.x, u.m, u.gamma, u.beta);
}

__global__ __launch_bounds__(kBlock) void k_tern_decode(const uint64_t *neg_row, const uint64_t *nz_row, const float *scale,
                                                        int64_t d, float *out)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    st4(out, e, d, aligned16(out), tern_decode4(neg_row, nz_row, scale[0], e));
}

unsigned blocks4(int64_t d) { return static_cast<unsigned>((d + kBlock * 4 - 1) / (kBlock * 4)); }

}  // namespace

ds_status_t ds_ternary_init(ds_ctx *c)
{
    ds_tern_scratch *t = new (std::nothrow) ds_tern_scratch();
    if (!t) return DS_ERR_DEVICE;
    *t = ds_tern_scratch{};
    c->tern = t;
    const size_t n = static_cast<size_t>(c->cfg.n), tiles = static_cast<size_t>(c->n_tiles);
    DS_HIP_TRY(hipMalloc(&t->pmax, n * tiles * sizeof(float)));
    DS_HIP_TRY(hipMalloc(&t->psum, n * tiles * sizeof(double)));
    DS_HIP_TRY(hipMalloc(&t->pcnt, n * tiles * sizeof(uint32_t)));
    DS_HIP_TRY(hipMalloc(&t->rowmax, n * sizeof(float)));
    DS_HIP_TRY(hipMalloc(&t->rowsum, n * sizeof(double)));
    return DS_OK;
}

void ds_ternary_fini(ds_ctx *c)
{
    ds_tern_scratch *t = c->tern;
    if (!t) return;
    void *ptrs[5] = {t->pmax, t->psum, t->pcnt, t->rowmax, t->rowsum};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    delete t;
    c->tern = nullptr;
}

ds_status_t ds_ternary_worker(ds_ctx *c, uint64_t step, const void *g, int64_t gs, const ds_payload_t *out, hipStream_t st)
{
    ds_tern_scratch *t = c->tern;
    const int64_t d = c->cfg.d, n_tiles = c->n_tiles;
    const unsigned n = static_cast<unsigned>(c->cfg.n);
    const dim3 grid(static_cast<unsigned>(n_tiles), n);
    const uint32_t key0 = static_cast<uint32_t>(c->cfg.seed);
    const uint32_t key1 = static_cast<uint32_t>(c->cfg.seed >> 32) ^ static_cast<uint32_t>(step >> 32);
    uint64_t *nz = reinterpret_cast<uint64_t *>(out->levels);
    const bool bf16 = c->cfg.grad_dtype == DS_BF16;
    if (bf16) k_tern_stats<true><<<grid, kBlock, 0, st>>>(g, gs, d, t->pmax, t->psum);
    else k_tern_stats<false><<<grid, kBlock, 0, st>>>(g, gs, d, t->pmax, t->psum);
    k_tern_rowstat<<<n, kBlock, 0, st>>>(t->pmax, t->psum, n_tiles, t->rowmax, t->rowsum);
    if (bf16)
        k_tern_encode<true><<<grid, kBlock, 0, st>>>(g, gs, d, t->rowmax, key0, key1, static_cast<uint32_t>(step),
                                                     out->sign_words, nz, c->W, t->pcnt);
    else
        k_tern_encode<false><<<grid, kBlock, 0, st>>>(g, gs, d, t->rowmax, key0, key1, static_cast<uint32_t>(step),
                                                      out->sign_words, nz, c->W, t->pcnt);
    k_tern_scale<<<n, kBlock, 0, st>>>(t->pcnt, t->rowsum, n_tiles, out->scales);
    return ds_launch_status();
}

ds_status_t ds_ternary_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st)
{
    k_tern_server_identity<<<blocks4(c->cfg.d), kBlock, 0, st>>>(in->sign_words, reinterpret_cast<const uint64_t *>(in->levels),
                                                                in->scales, c->cfg.n, c->inv_n, c->cfg.d, c->W, dense_out, u);
    return ds_launch_status();
}

ds_status_t ds_ternary_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st)
{
    k_tern_decode<<<blocks4(c->cfg.d), kBlock, 0, st>>>(p->sign_words + row * c->W,
                                                       reinterpret_cast<const uint64_t *>(p->levels) + row * c->W,
                                                       p->scales + row, c->cfg.d, out);
    return ds_launch_status();
}
