// Top-k sparsification kernels (Section 3.2 "Top-k sparsification", Section 5.1 "Top-k
// compression" of the DoubleSqueeze paper): keep the k entries of largest absolute value,
// zero the rest.  The message lists (index, value) by ascending index; equal magnitudes are
// resolved towards the lower index.
//
// Selection is exact and deterministic: a radix select on the 31-bit magnitude pattern
// key = bits(v) & 0x7FFFFFFF, 12 + 11 + 8 bits.
//   pass 1   (dense)  v = g + delta is written into the delta buffer and histogrammed on
//                     the top 12 key bits (LDS histogram per persistent workgroup).
//   pick 1            the bin b1 that holds the k-th largest key.
//   compact  (dense)  every element with key >= b1 << 19 becomes a candidate
//                     (index, value), written tile by tile into a compact list; elements of
//                     bin b1 are histogrammed on the next 11 bits.
//   pick 2, hist 3, pick 3   work on the candidate list only (about k entries) and end with
//                     the exact threshold key T and the number of ties at T to keep.
//   count / scan / emit      per tile, in tile order: entries above T plus the first ties
//                     by index, written at their scanned offsets, so the output is sorted
//                     by index with no sort; kept positions of the error buffer are zeroed
//                     (delta = v - Q[v] is 0 there and v elsewhere).
// The candidate order inside a tile is index order (ballot + prefix count), tiles are
// placed by an atomic counter but addressed through a per-tile table, so the result does
// not depend on scheduling.
#include "ds_device.h"
#include "ds_internal.h"

#include <new>

using namespace ds;

namespace {

constexpr int kH1 = 4096, kH2 = 2048, kH3 = 256;
constexpr int kHistRow = kH1 + kH2 + kH3;
constexpr int kTilesPerBlock = kWaves;  // wave-per-tile kernels

struct Sel {
    uint32_t b1, k1;   // top-12-bit bin of the k-th key; entries still needed from it
    uint32_t b2, k2;   // next 11 bits; entries still needed from that sub-bin
    uint32_t T, k3;    // threshold key; ties at T to keep (lowest indices first)
    uint32_t n_cand;   // candidates = elements with key >= b1 << 19
    uint32_t alloc;    // running allocation in the candidate list
};

__device__ __forceinline__ uint32_t key_of(float v) { return __float_as_uint(v) & 0x7FFFFFFFu; }

// number of set bits of m below this lane
__device__ __forceinline__ uint32_t lanes_below(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(m >> 32), __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(m), 0u));
}

}  // namespace

struct ds_topk_scratch {
    uint32_t *hist;      // [rows][kHistRow]
    Sel *sel;            // [rows]
    u32x2 *cand;         // [rows][d]  (index, value bits)
    uint32_t *tile_off;  // [rows][n_tiles] start of the tile's candidates
    uint32_t *tile_cnt;  // [rows][n_tiles] number of candidates
    uint32_t *tile_gt;   // [rows][n_tiles] candidates with key > T
    uint32_t *tile_eq;   // [rows][n_tiles] candidates with key == T
    uint32_t *tile_eqb;  // [rows][n_tiles] ties at T in earlier tiles
    uint32_t *tile_out;  // [rows][n_tiles] first output slot of the tile
    int rows;
};

namespace {

__global__ __launch_bounds__(kBlock) void k_topk_zero(uint32_t *hist, Sel *sel, int rows)
{
    const int total = rows * kHistRow;
    for (int i = blockIdx.x * kBlock + threadIdx.x; i < total; i += gridDim.x * kBlock) hist[i] = 0u;
    if (blockIdx.x == 0 && threadIdx.x < rows) sel[threadIdx.x].alloc = 0u;
    if (blockIdx.x == 0)
        for (int r = threadIdx.x + kBlock; r < rows; r += kBlock) sel[r].alloc = 0u;
}

__device__ __forceinline__ void hist4(uint32_t *h, f32x4 v, int64_t e, int64_t d)
{
    if (e + 0 < d) atomicAdd(&h[key_of(v.x) >> 19], 1u);
    if (e + 1 < d) atomicAdd(&h[key_of(v.y) >> 19], 1u);
    if (e + 2 < d) atomicAdd(&h[key_of(v.z) >> 19], 1u);
    if (e + 3 < d) atomicAdd(&h[key_of(v.w) >> 19], 1u);
}

// Pass 1, worker: v = g + delta -> delta buffer, 12-bit histogram.  Persistent workgroups.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void k_topk_pass1_worker(const void *g, int64_t gs, float *delta, int64_t dstr,
                                                              int64_t d, int64_t n_tiles, uint32_t *hist)
{
    __shared__ uint32_t h[kH1];
    const int row = blockIdx.y;
    for (int i = threadIdx.x; i < kH1; i += kBlock) h[i] = 0u;
    __syncthreads();
    const void *grow = BF16 ? static_cast<const void *>(static_cast<const uint16_t *>(g) + row * gs)
                            : static_cast<const void *>(static_cast<const float *>(g) + row * gs);
    float *drow = delta + row * dstr;
    const bool gvec = BF16 ? aligned8(grow) : aligned16(grow);
    const bool dvec = aligned16(drow);
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t e = tile * kTile + threadIdx.x * 4;
        if (e >= d) continue;
        const f32x4 v = ld4_grad<BF16>(grow, e, d, gvec) + ld4(drow, e, d, dvec);
        st4(drow, e, d, dvec, v);
        hist4(h, v, e, d);
    }
    __syncthreads();
    uint32_t *hrow = hist + static_cast<int64_t>(row) * kHistRow;
    for (int i = threadIdx.x; i < kH1; i += kBlock)
        if (h[i]) atomicAdd(&hrow[i], h[i]);
}

// First position in idx-sorted pairs[0..k) whose index is >= target.
__device__ __forceinline__ int64_t lower_bound_idx(const u32x2 *__restrict__ pairs, int64_t k, int64_t target)
{
    int64_t lo = 0, hi = k;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (static_cast<int64_t>(static_cast<int32_t>(pairs[mid].x)) < target) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// Adds, in worker order, the entries of every worker's message that fall into the tile
// [base, base + 2048) onto the tile held in LDS: tilev[j] = fma(val, 1/n, tilev[j]).
// A message lists each index once, so one worker's entries never collide; workers are
// separated by barriers, which keeps the chain order of the server's average.
__device__ __forceinline__ void scatter_messages(float *tilev, int64_t *lo_sh, int64_t *hi_sh,
                                                 const u32x2 *__restrict__ pairs_in, int n, int64_t k,
                                                 float inv_n, int64_t base)
{
    for (int i0 = 0; i0 < n; i0 += kBlock) {
        const int cnt = (n - i0 < kBlock) ? n - i0 : kBlock;
        __syncthreads();
        if (static_cast<int>(threadIdx.x) < cnt) {
            const u32x2 *p = pairs_in + static_cast<int64_t>(i0 + threadIdx.x) * k;
            lo_sh[threadIdx.x] = lower_bound_idx(p, k, base);
            hi_sh[threadIdx.x] = lower_bound_idx(p, k, base + kTile);
        }
        __syncthreads();
        for (int i = 0; i < cnt; ++i) {
            const u32x2 *p = pairs_in + static_cast<int64_t>(i0 + i) * k;
            for (int64_t j = lo_sh[i] + threadIdx.x; j < hi_sh[i]; j += kBlock) {
                const u32x2 pr = p[j];
                const uint32_t rel = pr.x - static_cast<uint32_t>(base);
                if (rel < static_cast<uint32_t>(kTile)) tilev[rel] = __fmaf_rn(__uint_as_float(pr.y), inv_n, tilev[rel]);
            }
            __syncthreads();
        }
    }
}

// Pass 1, server: v = delta_s + (1/n) sum_i Q[v_i] for sparse messages, written into the
// delta_s buffer, 12-bit histogram.
__global__ __launch_bounds__(kBlock) void k_topk_pass1_server(const u32x2 *pairs_in, int n, int64_t k, float inv_n,
                                                              float *delta_s, int64_t d, int64_t n_tiles,
                                                              uint32_t *hist)
{
    __shared__ uint32_t h[kH1];
    __shared__ float tilev[kTile];
    __shared__ int64_t lo_sh[kBlock], hi_sh[kBlock];
    for (int i = threadIdx.x; i < kH1; i += kBlock) h[i] = 0u;
    const bool dvec = aligned16(delta_s);
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t base = tile * kTile;
        const int64_t e = base + threadIdx.x * 4;
        const f32x4 a = ld4(delta_s, e, d, dvec);
        tilev[threadIdx.x * 4 + 0] = a.x; tilev[threadIdx.x * 4 + 1] = a.y;
        tilev[threadIdx.x * 4 + 2] = a.z; tilev[threadIdx.x * 4 + 3] = a.w;
        scatter_messages(tilev, lo_sh, hi_sh, pairs_in, n, k, inv_n, base);
        const f32x4 v = {tilev[threadIdx.x * 4 + 0], tilev[threadIdx.x * 4 + 1], tilev[threadIdx.x * 4 + 2],
                         tilev[threadIdx.x * 4 + 3]};
        if (e < d) {
            st4(delta_s, e, d, dvec, v);
            hist4(h, v, e, d);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kH1; i += kBlock)
        if (h[i]) atomicAdd(&hist[i], h[i]);
}

// Largest bin b of hist[0..NB) with  sum_{bins >= b} >= need ;  rem = need - sum_{bins > b},
// ge = sum_{bins >= b}.  One workgroup; the thread that owns b writes the three outputs.
template <int NB>
__device__ __forceinline__ void pick_bin(const uint32_t *__restrict__ hist, uint32_t need, uint32_t *part,
                                         uint32_t *b_out, uint32_t *rem_out, uint32_t *ge_out)
{
    constexpr int PER = (NB >= kBlock) ? NB / kBlock : 1;
    const int t = threadIdx.x;
    const bool active = t * PER < NB;
    uint32_t local[PER];
    uint32_t sum = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        local[j] = active ? hist[t * PER + j] : 0u;
        sum += local[j];
    }
    part[t] = sum;
    __syncthreads();
    for (int off = 1; off < kBlock; off <<= 1) {   // inclusive suffix sums of part[]
        const uint32_t add = (t + off < kBlock) ? part[t + off] : 0u;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    uint32_t running = (t + 1 < kBlock) ? part[t + 1] : 0u;   // keys in bins above my chunk
    if (active) {
#pragma unroll
        for (int j = PER - 1; j >= 0; --j) {
            const uint32_t above = running;
            running += local[j];
            if (running >= need && above < need) {
                *b_out = static_cast<uint32_t>(t * PER + j);
                *rem_out = need - above;
                *ge_out = running;
            }
        }
    }
}

template <int LEVEL>
__global__ __launch_bounds__(kBlock) void k_topk_pick(const uint32_t *hist, Sel *sel, uint32_t k)
{
    __shared__ uint32_t part[kBlock];
    __shared__ uint32_t out[3];
    const int row = blockIdx.x;
    const uint32_t *hrow = hist + static_cast<int64_t>(row) * kHistRow;
    Sel *s = sel + row;
    if (LEVEL == 1) pick_bin<kH1>(hrow, k, part, &out[0], &out[1], &out[2]);
    if (LEVEL == 2) pick_bin<kH2>(hrow + kH1, s->k1, part, &out[0], &out[1], &out[2]);
    if (LEVEL == 3) pick_bin<kH3>(hrow + kH1 + kH2, s->k2, part, &out[0], &out[1], &out[2]);
    __syncthreads();
    if (threadIdx.x == 0) {
        if (LEVEL == 1) { s->b1 = out[0]; s->k1 = out[1]; s->n_cand = out[2]; }
        if (LEVEL == 2) { s->b2 = out[0]; s->k2 = out[1]; }
        if (LEVEL == 3) { s->T = (s->b1 << 19) | (s->b2 << 8) | out[0]; s->k3 = out[1]; }
    }
}

// Dense look 2: candidates (key >= b1 << 19) of one tile, in index order, appended to the
// row's candidate list; 11-bit histogram of the elements of bin b1.
__global__ __launch_bounds__(kBlock) void k_topk_compact(const float *buf, int64_t stride, int64_t d, int64_t n_tiles,
                                                         Sel *sel, uint32_t *hist, u32x2 *cand, uint32_t *tile_off,
                                                         uint32_t *tile_cnt)
{
    __shared__ uint32_t h2[kH2];
    __shared__ uint32_t wtot[kWaves];
    __shared__ uint32_t base_sh;
    const int row = blockIdx.y;
    const int64_t tile = blockIdx.x;
    const float *brow = buf + row * stride;
    const int64_t e = tile * kTile + threadIdx.x * 4;
    for (int i = threadIdx.x; i < kH2; i += kBlock) h2[i] = 0u;
    const uint32_t b1 = sel[row].b1;
    const uint32_t lo_key = b1 << 19;
    const f32x4 v = ld4(brow, e, d, aligned16(brow));
    const uint32_t key[4] = {key_of(v.x), key_of(v.y), key_of(v.z), key_of(v.w)};
    const uint32_t bits[4] = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
    bool f[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) f[c] = (e + c < d) && key[c] >= lo_key;
    const uint64_t m0 = __ballot(f[0]), m1 = __ballot(f[1]), m2 = __ballot(f[2]), m3 = __ballot(f[3]);
    const uint32_t before = lanes_below(m0) + lanes_below(m1) + lanes_below(m2) + lanes_below(m3);
    const uint32_t wave_total = __popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3);
    if (lane_id() == 0) wtot[wave_id()] = wave_total;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 4; ++c)
        if (f[c] && (key[c] >> 19) == b1) atomicAdd(&h2[(key[c] >> 8) & (kH2 - 1)], 1u);
    uint32_t wave_off = 0, tile_total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave_id()) wave_off += wtot[w];
        tile_total += wtot[w];
    }
    if (threadIdx.x == 0) {
        const uint32_t b = tile_total ? atomicAdd(&sel[row].alloc, tile_total) : 0u;
        base_sh = b;
        tile_off[row * n_tiles + tile] = b;
        tile_cnt[row * n_tiles + tile] = tile_total;
    }
    __syncthreads();
    u32x2 *out = cand + static_cast<int64_t>(row) * d + base_sh + wave_off + before;
    uint32_t r = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c)
        if (f[c]) out[r++] = u32x2{static_cast<uint32_t>(e + c), bits[c]};
    uint32_t *h2g = hist + static_cast<int64_t>(row) * kHistRow + kH1;
    for (int i = threadIdx.x; i < kH2; i += kBlock)
        if (h2[i]) atomicAdd(&h2g[i], h2[i]);
}

// Histogram of the low 8 key bits of the candidates that share the 23-bit prefix (b1, b2).
__global__ __launch_bounds__(kBlock) void k_topk_hist3(const u32x2 *cand, int64_t d, const Sel *sel, uint32_t *hist)
{
    __shared__ uint32_t h3[kH3];
    const int row = blockIdx.y;
    if (threadIdx.x < kH3) h3[threadIdx.x] = 0u;
    __syncthreads();
    const Sel s = sel[row];
    const uint32_t prefix = (s.b1 << 11) | s.b2;
    const u32x2 *crow = cand + static_cast<int64_t>(row) * d;
    for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < s.n_cand; i += gridDim.x * kBlock) {
        const uint32_t key = crow[i].y & 0x7FFFFFFFu;
        if ((key >> 8) == prefix) atomicAdd(&h3[key & 255u], 1u);
    }
    __syncthreads();
    uint32_t *h3g = hist + static_cast<int64_t>(row) * kHistRow + kH1 + kH2;
    if (threadIdx.x < kH3 && h3[threadIdx.x]) atomicAdd(&h3g[threadIdx.x], h3[threadIdx.x]);
}

// One wavefront per tile: how many of its candidates lie above T, how many tie with T.
__global__ __launch_bounds__(kBlock) void k_topk_tile_count(const u32x2 *cand, int64_t d, const Sel *sel,
                                                            const uint32_t *tile_off, const uint32_t *tile_cnt,
                                                            int64_t n_tiles, uint32_t *tile_gt, uint32_t *tile_eq)
{
    const int row = blockIdx.y;
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * kTilesPerBlock + wave_id();
    if (tile >= n_tiles) return;
    const uint32_t T = sel[row].T;
    const u32x2 *c = cand + static_cast<int64_t>(row) * d + tile_off[row * n_tiles + tile];
    const uint32_t cnt = tile_cnt[row * n_tiles + tile];
    uint32_t gt = 0, eq = 0;
    for (uint32_t i = lane_id(); i < cnt; i += 64) {
        const uint32_t key = c[i].y & 0x7FFFFFFFu;
        gt += key > T;
        eq += key == T;
    }
    gt = wave_sum_u32(gt);
    eq = wave_sum_u32(eq);
    if (lane_id() == 0) {
        tile_gt[row * n_tiles + tile] = gt;
        tile_eq[row * n_tiles + tile] = eq;
    }
}

// Exclusive scan over the workgroup of one value per thread (Hillis-Steele in LDS).
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t *tmp)
{
    const int t = threadIdx.x;
    __syncthreads();
    tmp[t] = x;
    __syncthreads();
    for (int off = 1; off < kBlock; off <<= 1) {
        const uint32_t add = (t >= off) ? tmp[t - off] : 0u;
        __syncthreads();
        tmp[t] += add;
        __syncthreads();
    }
    return tmp[t] - x;
}

// Per row, in tile order: ties seen before each tile, and each tile's first output slot.
__global__ __launch_bounds__(kBlock) void k_topk_scan(const Sel *sel, int64_t n_tiles, const uint32_t *tile_gt,
                                                      const uint32_t *tile_eq, uint32_t *tile_eqb, uint32_t *tile_out)
{
    __shared__ uint32_t tmp[kBlock];
    const int row = blockIdx.x;
    const uint32_t k3 = sel[row].k3;
    const int64_t per = (n_tiles + kBlock - 1) / kBlock;
    const int64_t t0 = threadIdx.x * per, t1 = (t0 + per < n_tiles) ? t0 + per : n_tiles;
    const uint32_t *gt = tile_gt + row * n_tiles, *eq = tile_eq + row * n_tiles;
    uint32_t *eqb = tile_eqb + row * n_tiles, *out = tile_out + row * n_tiles;
    uint32_t s = 0;
    for (int64_t t = t0; t < t1; ++t) s += eq[t];
    uint32_t run = block_exclusive_scan(s, tmp);
    uint32_t sel_sum = 0;
    for (int64_t t = t0; t < t1; ++t) {
        eqb[t] = run;
        const uint32_t left = (k3 > run) ? k3 - run : 0u;
        sel_sum += gt[t] + ((eq[t] < left) ? eq[t] : left);
        run += eq[t];
    }
    uint32_t o = block_exclusive_scan(sel_sum, tmp);
    for (int64_t t = t0; t < t1; ++t) {
        out[t] = o;
        const uint32_t left = (k3 > eqb[t]) ? k3 - eqb[t] : 0u;
        o += gt[t] + ((eq[t] < left) ? eq[t] : left);
    }
}

// One wavefront per tile: write the kept entries in index order and zero them in the
// error buffer (delta = v - Q[v]).
__global__ __launch_bounds__(kBlock) void k_topk_emit(const u32x2 *cand, int64_t d, const Sel *sel,
                                                      const uint32_t *tile_off, const uint32_t *tile_cnt,
                                                      const uint32_t *tile_eqb, const uint32_t *tile_out,
                                                      int64_t n_tiles, int64_t k, u32x2 *pairs, float *buf,
                                                      int64_t stride)
{
    const int row = blockIdx.y;
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * kTilesPerBlock + wave_id();
    if (tile >= n_tiles) return;
    const Sel s = sel[row];
    const u32x2 *c = cand + static_cast<int64_t>(row) * d + tile_off[row * n_tiles + tile];
    const uint32_t cnt = tile_cnt[row * n_tiles + tile];
    uint32_t eq_seen = tile_eqb[row * n_tiles + tile];
    uint32_t out = tile_out[row * n_tiles + tile];
    u32x2 *prow = pairs + static_cast<int64_t>(row) * k;
    float *brow = buf + row * stride;
    for (uint32_t i0 = 0; i0 < cnt; i0 += 64) {
        const uint32_t i = i0 + lane_id();
        const bool valid = i < cnt;
        u32x2 pr = {0u, 0u};
        if (valid) pr = c[i];
        const uint32_t key = pr.y & 0x7FFFFFFFu;
        const bool is_eq = valid && key == s.T;
        const uint64_t eq_mask = __ballot(is_eq);
        const bool keep = valid && (key > s.T || (is_eq && eq_seen + lanes_below(eq_mask) < s.k3));
        const uint64_t keep_mask = __ballot(keep);
        if (keep) {
            const uint32_t slot = out + lanes_below(keep_mask);
            if (slot < k) prow[slot] = pr;
            brow[pr.x] = 0.f;
        }
        out += __popcll(keep_mask);
        eq_seen += __popcll(eq_mask);
    }
}

// x <- fma(-gamma, val, x) at the kept indices (Algorithm 1, model update, sparse message).
__global__ __launch_bounds__(kBlock) void k_topk_update_sparse(const u32x2 *pairs, int64_t k, float *x, int64_t d,
                                                               float gamma)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= k) return;
    const u32x2 pr = pairs[i];
    if (pr.x < static_cast<uint32_t>(d)) x[pr.x] = __fmaf_rn(-gamma, __uint_as_float(pr.y), x[pr.x]);
}

// Dense use of one sparse message: decode it tile by tile in LDS, then either write it out
// (decoder) or run the momentum update, which touches every element.
template <bool MOM, bool DECODE_ONLY>
__global__ __launch_bounds__(kBlock) void k_topk_dense_apply(const u32x2 *pairs, int64_t k, float *x, float *m,
                                                             int64_t d, float gamma, float beta)
{
    __shared__ float tilev[kTile];
    __shared__ int64_t lo_sh[kBlock], hi_sh[kBlock];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kTile;
    const int64_t e = base + threadIdx.x * 4;
#pragma unroll
    for (int c = 0; c < 4; ++c) tilev[threadIdx.x * 4 + c] = 0.f;
    scatter_messages(tilev, lo_sh, hi_sh, pairs, 1, k, 1.0f, base);
    if (e >= d) return;
    const f32x4 q = {tilev[threadIdx.x * 4 + 0], tilev[threadIdx.x * 4 + 1], tilev[threadIdx.x * 4 + 2],
                     tilev[threadIdx.x * 4 + 3]};
    apply_q4<MOM, DECODE_ONLY>(q, e, d, x, m, gamma, beta);
}

// selection pipeline shared by worker (rows = n) and server (rows = 1), after pass 1
ds_status_t select_and_emit(ds_ctx *c, int rows, float *buf, int64_t stride, u32x2 *pairs, hipStream_t st)
{
    ds_topk_scratch *t = c->topk;
    const int64_t d = c->cfg.d, n_tiles = c->n_tiles, k = c->cfg.k;
    const unsigned tile_blocks = static_cast<unsigned>((n_tiles + kTilesPerBlock - 1) / kTilesPerBlock);
    k_topk_pick<1><<<rows, kBlock, 0, st>>>(t->hist, t->sel, static_cast<uint32_t>(k));
    k_topk_compact<<<dim3(static_cast<unsigned>(n_tiles), rows), kBlock, 0, st>>>(buf, stride, d, n_tiles, t->sel, t->hist,
                                                                                 t->cand, t->tile_off, t->tile_cnt);
    k_topk_pick<2><<<rows, kBlock, 0, st>>>(t->hist, t->sel, 0u);
    k_topk_hist3<<<dim3(64, rows), kBlock, 0, st>>>(t->cand, d, t->sel, t->hist);
    k_topk_pick<3><<<rows, kBlock, 0, st>>>(t->hist, t->sel, 0u);
    k_topk_tile_count<<<dim3(tile_blocks, rows), kBlock, 0, st>>>(t->cand, d, t->sel, t->tile_off, t->tile_cnt, n_tiles,
                                                                 t->tile_gt, t->tile_eq);
    k_topk_scan<<<rows, kBlock, 0, st>>>(t->sel, n_tiles, t->tile_gt, t->tile_eq, t->tile_eqb, t->tile_out);
    k_topk_emit<<<dim3(tile_blocks, rows), kBlock, 0, st>>>(t->cand, d, t->sel, t->tile_off, t->tile_cnt, t->tile_eqb,
                                                           t->tile_out, n_tiles, k, pairs, buf, stride);
    return ds_launch_status();
}

unsigned persistent_blocks(int64_t n_tiles, int rows)
{
    int64_t per_row = (1024 + rows - 1) / rows;   // about 4 workgroups per compute unit in total
    if (per_row < 1) per_row = 1;
    if (per_row > n_tiles) per_row = n_tiles;
    return static_cast<unsigned>(per_row);
}

}  // namespace

ds_status_t ds_topk_init(ds_ctx *c)
{
    ds_topk_scratch *t = new (std::nothrow) ds_topk_scratch();
    if (!t) return DS_ERR_DEVICE;
    *t = ds_topk_scratch{};
    c->topk = t;
    const size_t rows = static_cast<size_t>(c->cfg.n), nt = static_cast<size_t>(c->n_tiles);
    t->rows = c->cfg.n;
    DS_HIP_TRY(hipMalloc(&t->hist, rows * kHistRow * sizeof(uint32_t)));
    DS_HIP_TRY(hipMalloc(&t->sel, rows * sizeof(Sel)));
    DS_HIP_TRY(hipMalloc(&t->cand, rows * static_cast<size_t>(c->cfg.d) * sizeof(u32x2)));
    uint32_t **tabs[6] = {&t->tile_off, &t->tile_cnt, &t->tile_gt, &t->tile_eq, &t->tile_eqb, &t->tile_out};
    for (auto tab : tabs) DS_HIP_TRY(hipMalloc(tab, rows * nt * sizeof(uint32_t)));
    DS_HIP_TRY(hipMemset(t->sel, 0, rows * sizeof(Sel)));
    return DS_OK;
}

void ds_topk_fini(ds_ctx *c)
{
    ds_topk_scratch *t = c->topk;
    if (!t) return;
    void *ptrs[9] = {t->hist, t->sel, t->cand, t->tile_off, t->tile_cnt, t->tile_gt, t->tile_eq, t->tile_eqb, t->tile_out};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    delete t;
    c->topk = nullptr;
}

ds_status_t ds_topk_worker(ds_ctx *c, const void *g, int64_t gs, float *delta, int64_t dstr, const ds_payload_t *out,
                           hipStream_t st)
{
    ds_topk_scratch *t = c->topk;
    const int rows = c->cfg.n;
    k_topk_zero<<<8, kBlock, 0, st>>>(t->hist, t->sel, rows);
    dim3 grid(persistent_blocks(c->n_tiles, rows), rows);
    if (c->cfg.grad_dtype == DS_BF16)
        k_topk_pass1_worker<true><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, c->cfg.d, c->n_tiles, t->hist);
    else
        k_topk_pass1_worker<false><<<grid, kBlock, 0, st>>>(g, gs, delta, dstr, c->cfg.d, c->n_tiles, t->hist);
    return select_and_emit(c, rows, delta, dstr, reinterpret_cast<u32x2 *>(out->pairs), st);
}

ds_status_t ds_topk_server(ds_ctx *c, const ds_payload_t *in, float *delta_s, const ds_payload_t *out, hipStream_t st)
{
    ds_topk_scratch *t = c->topk;
    k_topk_zero<<<8, kBlock, 0, st>>>(t->hist, t->sel, 1);
    k_topk_pass1_server<<<persistent_blocks(c->n_tiles, 1), kBlock, 0, st>>>(
        reinterpret_cast<const u32x2 *>(in->pairs), c->cfg.n, c->cfg.k, c->inv_n, delta_s, c->cfg.d, c->n_tiles, t->hist);
    return select_and_emit(c, 1, delta_s, c->cfg.d, reinterpret_cast<u32x2 *>(out->pairs), st);
}

ds_status_t ds_topk_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma, float beta, hipStream_t st)
{
    const u32x2 *pairs = reinterpret_cast<const u32x2 *>(srv->pairs);
    if (m) {
        k_topk_dense_apply<true, false><<<static_cast<unsigned>(c->n_tiles), kBlock, 0, st>>>(pairs, c->cfg.k, x, m, c->cfg.d,
                                                                                           gamma, beta);
    } else {
        const unsigned blocks = static_cast<unsigned>((c->cfg.k + kBlock - 1) / kBlock);
        k_topk_update_sparse<<<blocks, kBlock, 0, st>>>(pairs, c->cfg.k, x, c->cfg.d, gamma);
    }
    return ds_launch_status();
}

ds_status_t ds_topk_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st)
{
    const u32x2 *pairs = reinterpret_cast<const u32x2 *>(p->pairs) + static_cast<int64_t>(row) * c->cfg.k;
    k_topk_dense_apply<false, true><<<static_cast<unsigned>(c->n_tiles), kBlock, 0, st>>>(pairs, c->cfg.k, out, nullptr,
                                                                                       c->cfg.d, 0.f, 0.f);
    return ds_launch_status();
}
