// Randomised sparsification (Section 3.2 "Randomized Sparsification" of the DoubleSqueeze
// paper): every element is kept with probability p, and then scaled to z/p, or set to zero,
// which makes the operator unbiased.  (The section prints p for both outcomes; the zero
// outcome has probability 1 - p.)
//
// Element j of stream s (worker index, 0xFFFFFFFF for the server) at iteration t is kept iff
// the upper 24 bits of word j & 3 of Philox4x32-10(counter (j >> 2, 0, s, lo32(t)), key
// (lo32(seed), hi32(seed) ^ hi32(t))) are below P24 = p * 2^24: the same draws as the
// quantiser's rounding.  The message is the plane of "kept" bits (layout of the sign plane)
// and the kept values z/p, one IEEE fp32 division each, packed in index order.
//
// Packing in index order needs every element's rank among the kept ones.  The keep decisions
// do not depend on the data, so the writer first runs the generator alone (k_rs_counts: it
// writes the kept-bit plane, which is part of the message anyway, and the number of kept
// elements per 256-element subtile), scans the counts, and the ONE dense pass then reads its
// keep bits back from the plane (1/8 byte per element instead of a second evaluation of the
// generator) and writes each kept value straight to its final slot: ballots give the rank
// inside the wavefront's subtile.  A reader gets the same offsets from the population counts
// of the plane (k_rs_popcounts), so the message carries no offsets.
//
// The generator is pure integer ALU, and as a launch of its own it overlaps with nothing
// (about 80 us for 8 x 25.6 M elements against 490 us for the dense pass).  Folding it into
// the dense pass needs the offsets inside that pass; a chained scan with decoupled look-back
// over the 2048-element tiles was tried and took 1250 us: a tile is too little work, the
// look-back of a workgroup runs over most of the thousand workgroups that are resident with it.
#include "ds_device.h"
#include "ds_internal.h"

#include <new>

using namespace ds;

namespace {

constexpr int kSub = 256;   // elements per wavefront

struct RsParams {
    uint32_t key0, key1, step_lo;
    uint32_t p24;    // keep iff 24-bit uniform < p24
    float p;         // p24 * 2^-24, exact
};

// bits of a nibble whose elements e..e+3 lie below d
__device__ __forceinline__ uint32_t valid_nibble(int64_t e, int64_t d)
{
    return (e + 4 <= d) ? 15u : (e >= d) ? 0u : ((1u << (d - e)) - 1u);
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(m >> 32), __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(m), 0u));
}

// Rank of this lane's first flagged element among the flagged elements of the wavefront's
// subtile (index order: lane-major, the four elements of a lane in order), and the 32-bit
// words of the bit plane (lane q < 8 returns word q).
struct Ranks {
    uint32_t before;
    uint32_t word;
};

__device__ __forceinline__ Ranks subtile_ranks(uint32_t nib)
{
    const uint64_t m0 = __ballot(nib & 1u), m1 = __ballot(nib & 2u), m2 = __ballot(nib & 4u), m3 = __ballot(nib & 8u);
    Ranks r;
    r.before = lanes_below(m0) + lanes_below(m1) + lanes_below(m2) + lanes_below(m3);
    const int sh = (lane_id() & 7) * 8;
    const uint32_t x0 = static_cast<uint32_t>(m0 >> sh) & 0xFFu, x1 = static_cast<uint32_t>(m1 >> sh) & 0xFFu;
    const uint32_t x2 = static_cast<uint32_t>(m2 >> sh) & 0xFFu, x3 = static_cast<uint32_t>(m3 >> sh) & 0xFFu;
    r.word = spread4(x0) | (spread4(x1) << 1) | (spread4(x2) << 2) | (spread4(x3) << 3);
    return r;
}

// ---------------------------------------------------------------------------------------
// offsets of the packed values per subtile
// ---------------------------------------------------------------------------------------
// Writer side: the kept-bit plane and the kept elements per subtile from the generator alone.
// A wavefront takes kCountSubs consecutive subtiles (one subtile per workgroup-launch slot made
// the launch overhead of 100 000 tiny workgroups the cost of this kernel).  The kernel is bound
// by integer ALU work, so everything around the ten Philox rounds is kept short: one compare
// per element ((r >> 8) < P24 as r <= 256 P24 - 1), the count from the compare masks with
// scalar instructions, and the plane's 32-bit words by three shift-and-merge steps between
// neighbouring lanes (lane 8q ends up with word q).
constexpr int kCountSubs = 8;

// x of the lane N places above this one, inside a row of 16 lanes
template <int N>
__device__ __forceinline__ uint32_t from_lane_above(uint32_t x)
{
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x100 | N, 0xF, 0xF, true));   // row_shl:N
}

// One subtile: PARTIAL for the row's last one when d cuts it (nothing at or past d is kept).
template <bool PARTIAL>
__device__ __forceinline__ uint32_t count_subtile(int64_t s, int lane, int64_t d, uint32_t stream, uint32_t thr, const RsParams &P,
                                              uint32_t *wrow, int64_t words32, uint32_t *cnt_row)
{
    const uint32_t blk = static_cast<uint32_t>(s) * (kSub / 4) + lane;        // (s * 256 + 4 * lane) >> 2
    const u32x4 r = philox4x32_10(u32x4{blk, 0u, stream, P.step_lo}, P.key0, P.key1);
    bool k0 = r.x <= thr, k1 = r.y <= thr, k2 = r.z <= thr, k3 = r.w <= thr;
    if (PARTIAL) {
        const int left = static_cast<int>(d - s * kSub) - lane * 4;            // elements of the row from this lane's first on
        k0 = k0 && left > 0; k1 = k1 && left > 1; k2 = k2 && left > 2; k3 = k3 && left > 3;
    }
    const uint32_t c = __popcll(__ballot(k0)) + __popcll(__ballot(k1)) + __popcll(__ballot(k2)) + __popcll(__ballot(k3));
    uint32_t t = (k0 ? 1u : 0u) | (k1 ? 2u : 0u) | (k2 ? 4u : 0u) | (k3 ? 8u : 0u);
    t |= from_lane_above<1>(t) << 4;
    t |= from_lane_above<2>(t) << 8;
    t |= from_lane_above<4>(t) << 16;
    const int64_t w = s * 8 + (lane >> 3);
    if ((lane & 7) == 0 && (!PARTIAL || w < words32)) wrow[w] = t;
    if (lane == 0) cnt_row[s] = c;
    return c;
}

// tot64 [row][ceil(n_sub / 64)]: kept elements per 64 consecutive subtiles (= per workgroup
// here), which spares the scan a launch.
__global__ __launch_bounds__(kBlock) void k_rs_counts(uint64_t *words, int64_t W, uint32_t *cnt, uint32_t *tot64, int64_t n_sub,
                                                      int64_t n_t64, int64_t d, bool server, RsParams P)
{
    static_assert(kWaves * kCountSubs == 64, "one workgroup = one entry of tot64");
    __shared__ uint32_t wsum[kWaves];
    const int row = blockIdx.y;
    const int lane = lane_id();
    const uint32_t stream = server ? 0xFFFFFFFFu : static_cast<uint32_t>(row);
    const uint32_t thr = static_cast<uint32_t>((static_cast<uint64_t>(P.p24) << 8) - 1u);
    uint32_t *wrow = reinterpret_cast<uint32_t *>(words + row * W);
    uint32_t *cnt_row = cnt + row * (n_sub + 1);
    const int wave = __builtin_amdgcn_readfirstlane(wave_id());               // the loop bounds are scalars
    const int64_t s0 = (static_cast<int64_t>(blockIdx.x) * kWaves + wave) * kCountSubs;
    const int64_t s1 = (s0 + kCountSubs < n_sub) ? s0 + kCountSubs : n_sub;
    const int64_t full = d / kSub;                                            // subtiles before this one are whole
    uint32_t total = 0;
    if (s0 + kCountSubs <= full) {
#pragma unroll 2
        for (int j = 0; j < kCountSubs; ++j) total += count_subtile<false>(s0 + j, lane, d, stream, thr, P, wrow, 2 * W, cnt_row);
    } else {
        // the end of the row
        const int64_t s_whole = (s1 < full) ? s1 : full;
        for (int64_t s = s0; s < s_whole; ++s) total += count_subtile<false>(s, lane, d, stream, thr, P, wrow, 2 * W, cnt_row);
        if (s0 <= full && full < s1) total += count_subtile<true>(full, lane, d, stream, thr, P, wrow, 2 * W, cnt_row);   // d % 256 != 0
    }
    if (lane == 0) wsum[wave] = total;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) t += wsum[w];
        tot64[row * n_t64 + blockIdx.x] = t;
    }
}

// Reader side: the same counts from the kept-bit plane.  One thread per subtile, so one
// wavefront per entry of tot64.
__global__ __launch_bounds__(kBlock) void k_rs_popcounts(const uint64_t *__restrict__ words, int64_t W, uint32_t *cnt,
                                                         uint32_t *tot64, int64_t n_sub, int64_t n_t64, int64_t d)
{
    const int row = blockIdx.y;
    const int64_t s = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    uint32_t c = 0;
    if (s < n_sub) {
        const uint64_t *w = words + row * W + s * 4;
        for (int q = 0; q < 4; ++q) {
            const int64_t first = (s * 4 + q) * 64;         // bits at or past d do not count, whatever they hold
            if (first >= d) break;
            const uint64_t valid = (d - first >= 64) ? ~0ull : ((1ull << (d - first)) - 1ull);
            c += __popcll(w[q] & valid);
        }
        cnt[row * (n_sub + 1) + s] = c;
    }
    const uint32_t t = wave_sum_u32(c);
    if (lane_id() == 0 && (s >> 6) < n_t64) tot64[row * n_t64 + (s >> 6)] = t;
}

// Counts [row][0 .. n_sub) -> exclusive offsets [row][0 .. n_sub], the last one the row's
// total, in place and in one launch: a workgroup scans its block of 4096 entries and gets what
// lies before the block from tot64 (64 entries per block).
constexpr int kScanPer = 8, kScanBlock = kBlock * kScanPer;

__global__ __launch_bounds__(kBlock) void k_rs_scan(uint32_t *tab, const uint32_t *__restrict__ tot64, int64_t n_sub, int64_t n_t64)
{
    __shared__ uint32_t tmp[kWaves], pre[kWaves];
    uint32_t *row = tab + static_cast<int64_t>(blockIdx.y) * (n_sub + 1);
    const uint32_t *trow = tot64 + static_cast<int64_t>(blockIdx.y) * n_t64;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kScanBlock + threadIdx.x * kScanPer;
    uint32_t c[kScanPer], s = 0;
#pragma unroll
    for (int j = 0; j < kScanPer; ++j) {
        c[j] = (t0 + j < n_sub) ? row[t0 + j] : 0u;
        s += c[j];
    }
    uint32_t b = 0;
    const int64_t n_before = static_cast<int64_t>(blockIdx.x) * (kScanBlock / 64);
    for (int64_t t = threadIdx.x; t < n_before; t += kBlock) b += trow[t];
    b = wave_sum_u32(b);
    const int lane = lane_id();
    const uint32_t p = wave_inclusive_scan_u32(s);
    if (lane == 63) tmp[wave_id()] = p;
    if (lane == 0) pre[wave_id()] = b;
    __syncthreads();
    uint32_t run = p - s;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave_id()) run += tmp[w];
        run += pre[w];
    }
#pragma unroll
    for (int j = 0; j < kScanPer; ++j) {
        if (t0 + j <= n_sub) row[t0 + j] = run;            // entry n_sub receives the running total
        run += c[j];
    }
}

// ---------------------------------------------------------------------------------------
// the three calls
// ---------------------------------------------------------------------------------------
// p0..p3: the four floats that follow a lane's position in the packed values; the kept ones
// among its four elements (flags in nib) are the first of them, in element order.  Returns
// them at their elements and 0 for the others (selects instead of a load per kept element).
__device__ __forceinline__ f32x4 place_kept4(float p0, float p1, float p2, float p3, uint32_t nib)
{
    const bool k0 = nib & 1u, k1 = nib & 2u, k2 = nib & 4u, k3 = nib & 8u;
    const float a1 = k0 ? p1 : p0, a2 = k0 ? p2 : p1, a3 = k0 ? p3 : p2;     // ranks k0, k0 + 1, k0 + 2
    const float b1 = k1 ? a2 : a1, b2 = k1 ? a3 : a2;                        // ranks k0 + k1, k0 + k1 + 1
    return f32x4{k0 ? p0 : 0.f, k1 ? a1 : 0.f, k2 ? b1 : 0.f, k3 ? (k2 ? b2 : b1) : 0.f};
}

// Q[v] of the four elements of a thread, the message and the error.
__device__ __forceinline__ void rs_store4(f32x4 v, uint32_t nib, const Ranks &rk, uint32_t base, int64_t e, int64_t d,
                                          float *__restrict__ vals_row, float *__restrict__ err_row, bool err_vec, float p)
{
    const f32x4 q = {(nib & 1u) ? v.x / p : 0.f, (nib & 2u) ? v.y / p : 0.f, (nib & 4u) ? v.z / p : 0.f,
                     (nib & 8u) ? v.w / p : 0.f};
    float *out = vals_row + base + rk.before;
    uint32_t r = 0;
    if (nib & 1u) out[r++] = q.x;
    if (nib & 2u) out[r++] = q.y;
    if (nib & 4u) out[r++] = q.z;
    if (nib & 8u) out[r++] = q.w;
    if (e < d) st4_stream(err_row, e, d, err_vec, v - q);
}

// Algorithm 1, worker block.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void k_rs_worker(const void *g, int64_t gs, float *delta, int64_t dstr, int64_t d,
                                                      const uint64_t *words, int64_t W, float *vals, const uint32_t *off,
                                                      int64_t n_sub, float p)
{
    const int row = blockIdx.y;
    const int64_t e = static_cast<int64_t>(blockIdx.x) * kTile + threadIdx.x * 4;
    const int64_t sub = e >> 8;
    if (sub >= n_sub) return;                               // whole wavefronts
    const void *grow = BF16 ? static_cast<const void *>(static_cast<const uint16_t *>(g) + row * gs)
                            : static_cast<const void *>(static_cast<const float *>(g) + row * gs);
    float *drow = delta + row * dstr;
    const bool gvec = BF16 ? aligned8(grow) : aligned16(grow);
    const bool dvec = aligned16(drow);
    const f32x4 v = ld4_grad<BF16>(grow, e, d, gvec) + ld4_stream(drow, e, d, dvec);
    const uint32_t nib = (e < d) ? load_sign_nibble(words + row * W, e) : 0u;   // written by k_rs_counts: no bits past d
    const Ranks rk = subtile_ranks(nib);
    rs_store4(v, nib, rk, off[row * (n_sub + 1) + sub], e, d, vals + static_cast<int64_t>(row) * d, drow, dvec, p);
}

// Parameter-server block: v = delta_s + (1/n) sum_i Q[v_i] as the chain acc = fma(q_i, 1/n, acc)
// over workers in ascending order (elements a worker did not keep add nothing), then the same
// compressor on the server's stream.
__global__ __launch_bounds__(kBlock) void k_rs_server(const uint64_t *words_in, const float *vals_in, const uint32_t *off_in,
                                                      int n, float inv_n, float *delta_s, int64_t d, int64_t W,
                                                      const uint64_t *words_out, float *vals_out, const uint32_t *off_out,
                                                      int64_t n_sub, float p)
{
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kTile;
    const int64_t e = base + threadIdx.x * 4;
    const int lane = lane_id();
    const int64_t wave_first = base + wave_id() * kSub;
    const int64_t sub = wave_first >> 8;
    if (sub >= n_sub) return;                               // whole wavefronts
    const bool dvec = aligned16(delta_s);
    f32x4 a = ld4_stream(delta_s, e, d, dvec);
    {
        for (int i0 = 0; i0 < n; i0 += 8) {
            const int nb = (n - i0 < 8) ? n - i0 : 8;
            // lane L: 32-bit word L & 7 of the plane of worker i0 + (L >> 3); lane i: offset of worker i0 + i
            uint32_t word = 0u;
            if ((lane >> 3) < nb && wave_first + 32 * (lane & 7) < W * 64)
                word = reinterpret_cast<const uint32_t *>(words_in + (i0 + (lane >> 3)) * W)[(wave_first >> 5) + (lane & 7)];
            const uint32_t o = (lane < nb) ? off_in[(i0 + lane) * (n_sub + 1) + sub] : 0u;
            const uint32_t vn = valid_nibble(e, d);
            if (nb == 8 && (sub + 1) * kSub + 4 <= d) {
                // A full batch away from the end of the rows: a lane's kept values start at most
                // at float (sub + 1) * 256 of a row, so four floats from there stay inside it.
                // All eight fetches are issued before the first is used.
                typedef float f32x4_unaligned __attribute__((ext_vector_type(4), aligned(4)));
                f32x4_unaligned pk[8];
                uint32_t nibs[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t w = __shfl(word, i * 8 + (lane >> 3), 64);
                    nibs[i] = (w >> (4 * (lane & 7))) & vn;
                    const Ranks rk = subtile_ranks(nibs[i]);
                    const int64_t at = static_cast<int64_t>(i0 + i) * d +
                                       static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(o), i)) + rk.before;
                    pk[i] = *reinterpret_cast<const f32x4_unaligned *>(vals_in + at);
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) a = fma4(inv_n, place_kept4(pk[i].x, pk[i].y, pk[i].z, pk[i].w, nibs[i]), a);
            } else {
                for (int i = 0; i < nb; ++i) {
                    const uint32_t w = __shfl(word, i * 8 + (lane >> 3), 64);
                    const uint32_t nib = (w >> (4 * (lane & 7))) & vn;
                    const Ranks rk = subtile_ranks(nib);
                    const float *src = vals_in + static_cast<int64_t>(i0 + i) * d +
                                       static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(o), i)) + rk.before;
                    f32x4 q = {0.f, 0.f, 0.f, 0.f};
                    uint32_t r = 0;
                    if (nib & 1u) q.x = src[r++];
                    if (nib & 2u) q.y = src[r++];
                    if (nib & 4u) q.z = src[r++];
                    if (nib & 8u) q.w = src[r++];
                    a = fma4(inv_n, q, a);                  // an element that was not kept adds nothing: fma(0, 1/n, a) = a
                }
            }
        }
    }
    const uint32_t nib = (e < d) ? load_sign_nibble(words_out, e) : 0u;         // written by k_rs_counts
    const Ranks rk = subtile_ranks(nib);
    rs_store4(a, nib, rk, off_out[sub], e, d, vals_out, delta_s, dvec, p);
}

// Model update / decoder from one message.  SPARSE (plain update, small p): only the kept
// elements are touched, x - gamma * 0 is x exactly; otherwise 128-bit accesses to all of x.
template <bool MOM, bool DECODE_ONLY, bool SPARSE>
__global__ __launch_bounds__(kBlock) void k_rs_apply(const uint64_t *__restrict__ words, const float *__restrict__ vals,
                                                     const uint32_t *__restrict__ off, float *x, float *m, int64_t d,
                                                     int64_t W, int64_t n_sub, float gamma, float beta)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    const int64_t sub = e >> 8;
    if (sub >= n_sub) return;                               // whole wavefronts
    const uint32_t nib = (e < d) ? (load_sign_nibble(words, e) & valid_nibble(e, d)) : 0u;
    const Ranks rk = subtile_ranks(nib);
    const float *src = vals + off[sub] + rk.before;
    f32x4 q = {0.f, 0.f, 0.f, 0.f};
    uint32_t r = 0;
    if (nib & 1u) q.x = src[r++];
    if (nib & 2u) q.y = src[r++];
    if (nib & 4u) q.z = src[r++];
    if (nib & 8u) q.w = src[r++];
    if (e >= d) return;
    if constexpr (SPARSE) {
        if (nib & 1u) x[e] = __fmaf_rn(-gamma, q.x, x[e]);
        if (nib & 2u) x[e + 1] = __fmaf_rn(-gamma, q.y, x[e + 1]);
        if (nib & 4u) x[e + 2] = __fmaf_rn(-gamma, q.z, x[e + 2]);
        if (nib & 8u) x[e + 3] = __fmaf_rn(-gamma, q.w, x[e + 3]);
    } else {
        apply_q4<MOM, DECODE_ONLY>(q, e, d, x, m, gamma, beta);
    }
}

unsigned blocks4(int64_t d) { return static_cast<unsigned>((d + kBlock * 4 - 1) / (kBlock * 4)); }


RsParams make_params(const ds_ctx *c, uint64_t step)
{
    RsParams P;
    P.key0 = static_cast<uint32_t>(c->cfg.seed);
    P.key1 = static_cast<uint32_t>(c->cfg.seed >> 32) ^ static_cast<uint32_t>(step >> 32);
    P.step_lo = static_cast<uint32_t>(step);
    P.p24 = static_cast<uint32_t>(c->cfg.k);
    P.p = static_cast<float>(c->cfg.k) * (1.0f / 16777216.0f);
    return P;
}

}  // namespace

struct ds_rs_scratch {
    int64_t n_sub;
    uint32_t *off_w;    // [n][n_sub + 1]  worker messages, writer side
    uint32_t *off_in;   // [n][n_sub + 1]  worker messages, as read by the server
    uint32_t *off_s;    // [n_sub + 1]     server message, writer side
    uint32_t *off_r;    // [n_sub + 1]     a message as read by the update / decoder
    uint32_t *tot64;    // [n][n_t64]      kept elements per 64 subtiles, from the count kernels for the scan
    int64_t n_t64;
};

static void scan_rows(const ds_rs_scratch *t, uint32_t *tab, unsigned rows, hipStream_t st)
{
    const unsigned n_blk = static_cast<unsigned>((t->n_sub + 1 + kScanBlock - 1) / kScanBlock);
    k_rs_scan<<<dim3(n_blk, rows), kBlock, 0, st>>>(tab, t->tot64, t->n_sub, t->n_t64);
}

ds_status_t ds_rsparse_init(ds_ctx *c)
{
    ds_rs_scratch *t = new (std::nothrow) ds_rs_scratch();
    if (!t) return DS_ERR_DEVICE;
    *t = ds_rs_scratch{};
    c->rs = t;
    t->n_sub = (c->cfg.d + kSub - 1) / kSub;
    const size_t row = static_cast<size_t>(t->n_sub + 1) * sizeof(uint32_t), n = static_cast<size_t>(c->cfg.n);
    DS_HIP_TRY(hipMalloc(&t->off_w, n * row));
    DS_HIP_TRY(hipMalloc(&t->off_in, n * row));
    DS_HIP_TRY(hipMalloc(&t->off_s, row));
    DS_HIP_TRY(hipMalloc(&t->off_r, row));
    t->n_t64 = (t->n_sub + 63) / 64;
    DS_HIP_TRY(hipMalloc(&t->tot64, n * static_cast<size_t>(t->n_t64) * sizeof(uint32_t)));
    return DS_OK;
}

void ds_rsparse_fini(ds_ctx *c)
{
    ds_rs_scratch *t = c->rs;
    if (!t) return;
    void *ptrs[5] = {t->off_w, t->off_in, t->off_s, t->off_r, t->tot64};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    delete t;
    c->rs = nullptr;
}

ds_status_t ds_rsparse_worker(ds_ctx *c, uint64_t step, const void *g, int64_t gs, float *delta, int64_t dstr,
                              const ds_payload_t *out, hipStream_t st)
{
    ds_rs_scratch *t = c->rs;
    const RsParams P = make_params(c, step);
    const unsigned n = static_cast<unsigned>(c->cfg.n);
    k_rs_counts<<<dim3(static_cast<unsigned>((t->n_sub + kWaves * kCountSubs - 1) / (kWaves * kCountSubs)), n), kBlock, 0, st>>>(
        out->sign_words, c->W, t->off_w, t->tot64, t->n_sub, t->n_t64, c->cfg.d, false, P);
    scan_rows(t, t->off_w, n, st);
    const dim3 grid(static_cast<unsigned>(c->n_tiles), n);
    if (c->cfg.grad_dtype == DS_BF16)
        k_rs_worker<true><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, c->cfg.d, out->sign_words, c->W, out->dense, t->off_w,
                                                   t->n_sub, P.p);
    else
        k_rs_worker<false><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, c->cfg.d, out->sign_words, c->W, out->dense, t->off_w,
                                                    t->n_sub, P.p);
    return ds_launch_status();
}

ds_status_t ds_rsparse_server(ds_ctx *c, uint64_t step, const ds_payload_t *in, float *delta_s, const ds_payload_t *out,
                              hipStream_t st)
{
    ds_rs_scratch *t = c->rs;
    const RsParams P = make_params(c, step);
    const unsigned n = static_cast<unsigned>(c->cfg.n);
    k_rs_popcounts<<<dim3(static_cast<unsigned>((t->n_sub + kBlock - 1) / kBlock), n), kBlock, 0, st>>>(
        in->sign_words, c->W, t->off_in, t->tot64, t->n_sub, t->n_t64, c->cfg.d);
    scan_rows(t, t->off_in, n, st);
    k_rs_counts<<<dim3(static_cast<unsigned>((t->n_sub + kWaves * kCountSubs - 1) / (kWaves * kCountSubs)), 1), kBlock, 0, st>>>(
        out->sign_words, c->W, t->off_s, t->tot64, t->n_sub, t->n_t64, c->cfg.d, true, P);
    scan_rows(t, t->off_s, 1, st);
    k_rs_server<<<static_cast<unsigned>(c->n_tiles), kBlock, 0, st>>>(in->sign_words, in->dense, t->off_in, c->cfg.n, c->inv_n,
                                                                    delta_s, c->cfg.d, c->W, out->sign_words, out->dense,
                                                                    t->off_s, t->n_sub, P.p);
    return ds_launch_status();
}

// off == nullptr: the offsets of the packed values are derived from the message's own plane.
template <bool DECODE_ONLY>
static ds_status_t rs_apply(ds_ctx *c, const uint64_t *words, const float *vals, float *x, float *m, float gamma, float beta,
                            hipStream_t st, const uint32_t *off = nullptr)
{
    ds_rs_scratch *t = c->rs;
    if (!off) {
        k_rs_popcounts<<<dim3(static_cast<unsigned>((t->n_sub + kBlock - 1) / kBlock), 1), kBlock, 0, st>>>(
            words, c->W, t->off_r, t->tot64, t->n_sub, t->n_t64, c->cfg.d);
        scan_rows(t, t->off_r, 1, st);
        off = t->off_r;
    }
    const unsigned blocks = blocks4(t->n_sub * kSub);
    if (DECODE_ONLY)
        k_rs_apply<false, true, false><<<blocks, kBlock, 0, st>>>(words, vals, off, x, nullptr, c->cfg.d, c->W, t->n_sub, 0.f, 0.f);
    else if (m)
        k_rs_apply<true, false, false><<<blocks, kBlock, 0, st>>>(words, vals, off, x, m, c->cfg.d, c->W, t->n_sub, gamma, beta);
    else if (c->cfg.k < (1 << 20))      // p < 1/16: most 64-byte lines of x hold no kept element
        k_rs_apply<false, false, true><<<blocks, kBlock, 0, st>>>(words, vals, off, x, m, c->cfg.d, c->W, t->n_sub, gamma, beta);
    else
        k_rs_apply<false, false, false><<<blocks, kBlock, 0, st>>>(words, vals, off, x, m, c->cfg.d, c->W, t->n_sub, gamma, beta);
    return ds_launch_status();
}

// The server block followed by the model update: the update reads the server's message with
// the offsets the server has just written it with, instead of deriving them from the plane again.
ds_status_t ds_rsparse_server_update(ds_ctx *c, uint64_t step, const ds_payload_t *in, float *delta_s, const ds_payload_t *out,
                                     float *x, float *m, float gamma, float beta, hipStream_t st)
{
    const ds_status_t rc = ds_rsparse_server(c, step, in, delta_s, out, st);
    if (rc != DS_OK) return rc;
    return rs_apply<false>(c, out->sign_words, out->dense, x, m, gamma, beta, st, c->rs->off_s);
}

ds_status_t ds_rsparse_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma, float beta, hipStream_t st)
{
    return rs_apply<false>(c, srv->sign_words, srv->dense, x, m, gamma, beta, st);
}

ds_status_t ds_rsparse_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st)
{
    return rs_apply<true>(c, p->sign_words + static_cast<int64_t>(row) * c->W, p->dense + static_cast<int64_t>(row) * c->cfg.d,
                          out, nullptr, 0.f, 0.f, st);
}
