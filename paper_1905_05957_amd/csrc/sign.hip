// 1-bit compressor kernels (Section 3.2 "1-Bit Quantization", Section 5.1 "1-bit
// compression" of the DoubleSqueeze paper) for the three calls of Algorithm 1.
//
// A message is a sign plane (bit = v < 0) plus one scale per group, scale = mean |v| of
// the group, so that the decoded group has the l1 magnitude of v.
//
// Two routes:
//  * fused (groups are chunks of 512..2048 elements, a multiple of 128): one workgroup holds
//    a whole chunk in registers, so v = g + delta, sum |v|, the sign bits and
//    delta' = v - Q[v] happen in ONE pass over HBM.
//  * general (whole vector, arbitrary segments, other chunk sizes): the scale needs a sum
//    over more than one workgroup, so pass 1 writes v into the delta buffer together with
//    the sign bits and fp64 partial sums, a small kernel reduces them in a fixed order,
//    and pass 2 turns v into delta' = v - Q[v].
//
// Sums of |v| are accumulated in fp64 and rounded once, in an order that depends only on
// the shape, so results are bit-reproducible run to run.
#include "ds_device.h"
#include "ds_internal.h"

#include <mutex>
#include <type_traits>
#include <vector>

using namespace ds;

namespace {

// ---------------------------------------------------------------------------------------
// sources of the vector v that is being compressed
// ---------------------------------------------------------------------------------------

// Worker: v = g + delta  (Algorithm 1, worker block, first step; Section 3.1).
template <bool BF16>
struct WorkerSrc {
    const void *g;
    int64_t g_stride;
    const float *delta;
    int64_t delta_stride;

    __device__ __forceinline__ const void *grow(int row) const
    {
        if constexpr (BF16) return static_cast<const uint16_t *>(g) + row * g_stride;
        else return static_cast<const float *>(g) + row * g_stride;
    }
};

// Server with one scale per chunk: v = delta_s + (1/n) sum_i Q[v_i], taken as the chain
// acc = fma(q_i, 1/n, acc) over workers in ascending order (Algorithm 1, parameter-server
// block, first step).
struct ServerArgs {
    const uint64_t *words_in;  // [n, W]
    const float *scales_in;    // [n, S]
    int32_t n;
    int64_t W, S;
    float inv_n;
};

// What a group sums to find its scale: |v| (scale = mean |v|, the l1 reading of "the same
// magnitude", Section 5.1) or v^2 (scale = root mean square, the l2 reading of Section 3.2's
// norm).  The product of two fp32 values is exact in fp64.
// (A compile-time switch: as a run-time one it cost the 124 M-element step 4 %.)
template <bool RMS>
__device__ __forceinline__ double measure(float x)
{
    if constexpr (RMS) return static_cast<double>(x) * static_cast<double>(x);
    else return static_cast<double>(fabsf(x));
}

// (s0, s1, s2, s3) with the sign flipped where the element's bit of `nib` is set.
__device__ __forceinline__ f32x4 signed4(float s0, float s1, float s2, float s3, uint32_t nib)
{
    return f32x4{__uint_as_float(__float_as_uint(s0) ^ ((nib << 31) & 0x80000000u)),
                 __uint_as_float(__float_as_uint(s1) ^ ((nib << 30) & 0x80000000u)),
                 __uint_as_float(__float_as_uint(s2) ^ ((nib << 29) & 0x80000000u)),
                 __uint_as_float(__float_as_uint(s3) ^ ((nib << 28) & 0x80000000u))};
}

// The same chain step with the lane's four sign bits in bits 28..31 of `top` (element 0 in bit
// 28): the sign bit of the scale is flipped where the element's bit is set, which is what
// "bit ? -scale : scale" does for every float.  Shift, mask, exclusive-or instead of test,
// compare and select: no condition-code hazards in a loop that runs n times per element.
__device__ __forceinline__ f32x4 chain4_top(f32x4 a, uint32_t top, float s, float inv_n)
{
    const uint32_t sb = __float_as_uint(s);
    a.x = __fmaf_rn(__uint_as_float(sb ^ ((top << 3) & 0x80000000u)), inv_n, a.x);
    a.y = __fmaf_rn(__uint_as_float(sb ^ ((top << 2) & 0x80000000u)), inv_n, a.y);
    a.z = __fmaf_rn(__uint_as_float(sb ^ ((top << 1) & 0x80000000u)), inv_n, a.z);
    a.w = __fmaf_rn(__uint_as_float(sb ^ (top & 0x80000000u)), inv_n, a.w);
    return a;
}

template <bool RMS>
__device__ __forceinline__ double abs_sum4(f32x4 v)
{
    return ((measure<RMS>(v.x) + measure<RMS>(v.y)) + measure<RMS>(v.z)) + measure<RMS>(v.w);
}

__device__ __forceinline__ float group_scale(double total, double len, bool rms)
{
    return rms ? static_cast<float>(sqrt(total / len)) : static_cast<float>(total / len);
}

// delta' = v - Q[v] with Q[v]_j = (v_j < 0) ? -scale : +scale
__device__ __forceinline__ f32x4 sign_error4(f32x4 v, float s)
{
    f32x4 o;
    o.x = v.x - ((v.x < 0.f) ? -s : s);
    o.y = v.y - ((v.y < 0.f) ? -s : s);
    o.z = v.z - ((v.z < 0.f) ? -s : s);
    o.w = v.w - ((v.w < 0.f) ? -s : s);
    return o;
}

// ---------------------------------------------------------------------------------------
// fused route: one workgroup per chunk
// ---------------------------------------------------------------------------------------
// Common tail: scale from the held values, sign plane, error, stores.
template <bool RMS>
__device__ __forceinline__ float fused_finish(f32x4 v, int64_t base, int64_t lim,
                                             float *__restrict__ err_row, bool err_vec,
                                             uint64_t *__restrict__ words_row, int64_t bit_lim,
                                             float *__restrict__ scale_out, double *lds, uint32_t *sw_lds)
{
    // sign words: gathered in LDS, one store per workgroup after the barrier of the reduction
    stash_sign_words(sw_lds, wave_sign_word(v.x < 0.f, v.y < 0.f, v.z < 0.f, v.w < 0.f));
    const double total = block_sum(abs_sum4<RMS>(v), lds, false);
    const float scale = group_scale(total, static_cast<double>(lim - base), RMS);
    if (threadIdx.x == 0) *scale_out = scale;
    flush_sign_words(sw_lds, words_row, base, bit_lim);
    const int64_t e = base + threadIdx.x * 4;
    if (err_row && e < lim) st4_stream(err_row, e, lim, err_vec, sign_error4(v, scale));   // no buffer: no compensation
    return scale;
}

// NOFB: Algorithm 1 without compensation, v = g; no error buffer is touched.
// CPW chunks per workgroup, all loads issued before the first is used.  With compensation one
// chunk per workgroup is fastest; without it a chunk is only 4 to 8 KiB of traffic and a
// workgroup per chunk is bound by the rate at which workgroups can be dispatched (486 k
// workgroups took 0.88 ms for 2.1 GB on the 124 M-element workload), so that variant takes four.
template <bool BF16, bool RMS, bool NOFB, int CPW>
__global__ __launch_bounds__(kBlock) void k_sign_chunk_worker(WorkerSrc<BF16> src, float *delta,
                                                              int64_t d, int64_t chunk,
                                                              uint64_t *words, int64_t W,
                                                              float *scales, int64_t S)
{
    __shared__ double lds[CPW][kWaves];
    __shared__ __attribute__((aligned(16))) uint32_t sw_lds[CPW][kWaves * 8];
    const int row = blockIdx.y;
    const void *grow = src.grow(row);
    float *drow = NOFB ? nullptr : delta + row * src.delta_stride;
    const bool gvec = BF16 ? aligned8(grow) : aligned16(grow);
    const bool dvec = aligned16(drow);
    f32x4 v[CPW];
    int64_t base[CPW], lim[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int64_t ci = static_cast<int64_t>(blockIdx.x) * CPW + c;
        base[c] = ci * chunk;
        lim[c] = (base[c] + chunk < d) ? base[c] + chunk : d;     // base >= d: empty chunk, lim < base
        const int64_t e = base[c] + threadIdx.x * 4;
        v[c] = ld4_grad<BF16>(grow, e, lim[c], gvec);
        if constexpr (!NOFB) v[c] = v[c] + ld4_stream(drow, e, lim[c], dvec);
    }
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int64_t ci = static_cast<int64_t>(blockIdx.x) * CPW + c;
        if (base[c] < d)    // uniform over the workgroup
            fused_finish<RMS>(v[c], base[c], lim[c], drow, dvec, words + row * W, (lim[c] == d) ? W * 64 : lim[c],
                              scales + row * S + ci, lds[c], sw_lds[c]);
    }
}

// UPD: 0 = the parameter-server block alone; 1, 2 = followed by the model update of Algorithm 1
// for the same elements (2: through the momentum buffer), from the registers that hold the
// server's sign bits and scale: x and m stream through once and the server's message is not
// read back.
template <int CPW, bool RMS, int UPD>   // CPW chunks per workgroup: independent chunks, more bytes in flight per thread
__global__ __launch_bounds__(kBlock) void k_sign_chunk_server(ServerArgs a, float *delta_s, int64_t d,
                                                              int64_t chunk, uint64_t *words_out,
                                                              float *scales_out, float *x, float *m, float gamma,
                                                              float beta)
{
    __shared__ double lds[CPW][kWaves];
    __shared__ __attribute__((aligned(16))) uint32_t sw_lds[CPW][kWaves * 8];
    const bool dvec = aligned16(delta_s);
    const int lane = lane_id();
    f32x4 v[CPW];
    int64_t base[CPW], lim[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int64_t ci = static_cast<int64_t>(blockIdx.x) * CPW + c;
        base[c] = ci * chunk;
        lim[c] = (base[c] + chunk < d) ? base[c] + chunk : d;     // base >= d: empty chunk, lim < base
        v[c] = delta_s ? ld4_stream(delta_s, base[c] + threadIdx.x * 4, lim[c], dvec) : f32x4{0.f, 0.f, 0.f, 0.f};   // no buffer: no server error
    }
    // the update's operands are fetched up front, beside the error: more bytes in flight
    f32x4 xv[CPW], mv[CPW];
    if constexpr (UPD != 0) {
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            xv[c] = ld4_stream(x, base[c] + threadIdx.x * 4, lim[c], aligned16(x));
            if constexpr (UPD == 2) mv[c] = ld4_stream(m, base[c] + threadIdx.x * 4, lim[c], aligned16(m));
        }
    }
    // The wavefront's 256 elements are 32 bytes of each worker's sign plane.  Eight workers at
    // a time: lane L loads 32-bit word (L & 7) of worker (L >> 3), one load instruction for
    // all of them; the nibble a lane needs for worker i then sits in lane 8 i + (L >> 3).
    for (int i0 = 0; i0 < a.n; i0 += 8) {
        const int nb = (a.n - i0 < 8) ? a.n - i0 : 8;
        const int wi = lane >> 3;
        uint32_t word[CPW];
        float sc[CPW];
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int64_t ci = static_cast<int64_t>(blockIdx.x) * CPW + c;
            const int64_t wave_first = base[c] + wave_id() * 256;
            word[c] = 0u;
            if (wi < nb && wave_first + 32 * (lane & 7) < a.W * 64)
                word[c] = reinterpret_cast<const uint32_t *>(a.words_in + (i0 + wi) * a.W)[(wave_first >> 5) + (lane & 7)];
            sc[c] = (lane < nb && base[c] < d) ? a.scales_in[(i0 + lane) * a.S + ci] : 0.f;
        }
        // Lanes past the end of their chunk run the chain too (their values are cleared below):
        // no branch inside the loop.  A full batch of eight workers is unrolled, so that the
        // eight cross-lane fetches are in flight together instead of one wait per worker.
        const int top_shift = 28 - 4 * (lane & 7);
        if (nb == 8) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
#pragma unroll
                for (int c = 0; c < CPW; ++c) {
                    const uint32_t w = __shfl(word[c], i * 8 + (lane >> 3), 64);
                    const float s = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sc[c]), i));
                    v[c] = chain4_top(v[c], w << top_shift, s, a.inv_n);
                }
            }
        } else {
            for (int i = 0; i < nb; ++i) {
#pragma unroll
                for (int c = 0; c < CPW; ++c) {
                    const uint32_t w = __shfl(word[c], i * 8 + (lane >> 3), 64);
                    const float s = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sc[c]), i));
                    v[c] = chain4_top(v[c], w << top_shift, s, a.inv_n);
                }
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int64_t ci = static_cast<int64_t>(blockIdx.x) * CPW + c;
        // components past lim must stay zero: they count in the sum of |v|
        v[c] = zero_past(v[c], base[c] + threadIdx.x * 4, lim[c]);
        if (base[c] < d) {   // uniform over the workgroup
            const float s = fused_finish<RMS>(v[c], base[c], lim[c], delta_s, dvec, words_out,
                                              (lim[c] == d) ? a.W * 64 : lim[c], scales_out + ci, lds[c], sw_lds[c]);
            if constexpr (UPD != 0) {
                // q = decode of the message just written: bit ? -scale : +scale, bit = (v < 0)
                const int64_t e = base[c] + threadIdx.x * 4;
                if (e < lim[c]) {
                    f32x4 q = {(v[c].x < 0.f) ? -s : s, (v[c].y < 0.f) ? -s : s, (v[c].z < 0.f) ? -s : s, (v[c].w < 0.f) ? -s : s};
                    if constexpr (UPD == 2) {
                        q = fma4(beta, mv[c], q);
                        st4_stream(m, e, lim[c], aligned16(m), q);
                    }
                    st4_stream(x, e, lim[c], aligned16(x), fma4(-gamma, q, xv[c]));
                }
            }
        }
    }
}

// One thread per 4 elements.
template <bool MOM, bool DECODE_ONLY>
__global__ __launch_bounds__(kBlock) void k_sign_chunk_update(const uint64_t *__restrict__ words,
                                                              const float *__restrict__ scales,
                                                              int64_t chunk, float *x, float *m,
                                                              int64_t d, float gamma, float beta)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * 4;
    if (e >= d) return;
    // chunk is a multiple of 4 on this route, so the four elements share a chunk;
    // e < 2^31, so the chunk index is a 32-bit division
    const float s = scales[static_cast<uint32_t>(e) / static_cast<uint32_t>(chunk)];
    const uint32_t nib = load_sign_nibble(words, e);
    apply_q4<MOM, DECODE_ONLY>(signed4(s, s, s, s, nib), e, d, x, m, gamma, beta);
}

// ---------------------------------------------------------------------------------------
// general route: tiles x pieces
// ---------------------------------------------------------------------------------------
// Pieces [p0, p1) of a tile; seg0 = its group when it has one piece, else -1.
struct TilePieces {
    int32_t p0, p1, seg0;
};

__device__ __forceinline__ TilePieces tile_pieces(const ds_sign_tables &tb, int64_t tile)
{
    if (tb.whole_d > 0) return TilePieces{static_cast<int32_t>(tile), static_cast<int32_t>(tile) + 1, 0};
    const int2 ti = tb.tile_info[tile];
    return (ti.y >= 0) ? TilePieces{ti.x, ti.x + 1, ti.y} : TilePieces{ti.x, ti.x - ti.y, -1};
}

// Group of element e, given the pieces [p0, p1) of its tile.
__device__ __forceinline__ int32_t seg_of(const ds_sign_tables &tb, int32_t p0, int32_t p1, int64_t e)
{
    int32_t p = p0;
    while (p + 1 < p1 && tb.piece_start[p + 1] <= e) ++p;
    return tb.piece_seg[p];
}

template <bool RMS>
__device__ __forceinline__ double masked_abs(float x, int64_t e, int64_t lo, int64_t hi)
{
    return (e >= lo && e < hi) ? measure<RMS>(x) : 0.0;
}

// v - Q[v] for the four elements of a thread, with the group scales of its tile's pieces.
__device__ __forceinline__ f32x4 sign_error_tile(f32x4 v, int64_t e, int64_t d, const float *__restrict__ srow,
                                                 const ds_sign_tables &tb, int32_t p0, int32_t p1, int32_t seg0)
{
    if (seg0 >= 0) return sign_error4(v, srow[seg0]);
    float s[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) s[c] = (e + c < d) ? srow[seg_of(tb, p0, p1, e + c)] : 0.f;
    v.x = v.x - ((v.x < 0.f) ? -s[0] : s[0]);
    v.y = v.y - ((v.y < 0.f) ? -s[1] : s[1]);
    v.z = v.z - ((v.z < 0.f) ? -s[2] : s[2]);
    v.w = v.w - ((v.w < 0.f) ? -s[3] : s[3]);
    return v;
}

// Pass-1 tail: store v, sign bits, per-piece partial sums of |v| (or v^2).  STREAM: v is not
// read again in this call (deferred error form), so it leaves non-temporally.
template <bool RMS, bool STREAM, bool KEEP = true>   // KEEP = false: v is not stored (no compensation: it is not needed again)
__device__ __forceinline__ void pass1_finish(f32x4 v, int64_t base, int64_t d,
                                             float *__restrict__ vrow, bool vvec,
                                             uint64_t *__restrict__ words_row, int64_t bit_lim,
                                             const ds_sign_tables &tb, int32_t p0, int32_t p1,
                                             double *__restrict__ partial_row, double *lds, uint32_t *sw_lds)
{
    const int64_t e = base + threadIdx.x * 4;
    if (KEEP && vrow && e < d) {             // no buffer: no compensation either
        if constexpr (STREAM) st4_stream(vrow, e, d, vvec, v);
        else st4(vrow, e, d, vvec, v);
    }
    stash_sign_words(sw_lds, wave_sign_word(v.x < 0.f, v.y < 0.f, v.z < 0.f, v.w < 0.f));
    if (p1 - p0 == 1) {
        const double total = block_sum(abs_sum4<RMS>(v), lds, false);   // elements past d are zero
        if (threadIdx.x == 0) partial_row[p0] = total;
        flush_sign_words(sw_lds, words_row, base, bit_lim);
    } else {
        __syncthreads();
        flush_sign_words(sw_lds, words_row, base, bit_lim);
        for (int32_t p = p0; p < p1; ++p) {
            const int64_t lo = tb.piece_start[p], hi = tb.piece_start[p + 1];
            const double part = ((masked_abs<RMS>(v.x, e, lo, hi) + masked_abs<RMS>(v.y, e + 1, lo, hi)) +
                                 masked_abs<RMS>(v.z, e + 2, lo, hi)) + masked_abs<RMS>(v.w, e + 3, lo, hi);
            const double total = block_sum(part, lds, true);
            if (threadIdx.x == 0) partial_row[p] = total;
        }
    }
}

// DEFERRED: the error buffer holds the previous call's v and `prev_scales` that call's group
// scales; the error delta = v_prev - Q[v_prev] is formed on the fly (the same subtraction
// pass 2 would have stored), so the buffer is looked at once per call.
// MODE 0: plain.  1 (deferred): as described above.  2: Algorithm 1 without compensation, v = g,
// no error buffer is touched.
template <bool BF16, int MODE, bool RMS>
__global__ __launch_bounds__(kBlock) void k_sign_pass1_worker(WorkerSrc<BF16> src, float *delta,
                                                              int64_t d, uint64_t *words, int64_t W,
                                                              ds_sign_tables tb, double *partials,
                                                              const float *__restrict__ prev_scales, int64_t S)
{
    __shared__ double lds[kWaves];
    __shared__ __attribute__((aligned(16))) uint32_t sw_lds[kWaves * 8];
    const int row = blockIdx.y;
    const int64_t tile = blockIdx.x;
    const int64_t base = tile * kTile;
    const void *grow = src.grow(row);
    constexpr bool DEFERRED = MODE == 1, NOFB = MODE == 2;
    float *drow = NOFB ? nullptr : delta + row * src.delta_stride;
    const bool gvec = BF16 ? aligned8(grow) : aligned16(grow);
    const bool dvec = aligned16(drow);
    const int64_t e = base + threadIdx.x * 4;
    const TilePieces tp = tile_pieces(tb, tile);
    const int32_t p0 = tp.p0, p1 = tp.p1;
    f32x4 v = ld4_grad<BF16>(grow, e, d, gvec);
    if constexpr (!NOFB) {
        f32x4 dl = DEFERRED ? ld4_stream(drow, e, d, dvec) : ld4(drow, e, d, dvec);
        if (DEFERRED && e < d) dl = zero_past(sign_error_tile(dl, e, d, prev_scales + row * S, tb, p0, p1, tp.seg0), e, d);
        v = v + dl;
    }
    pass1_finish<RMS, DEFERRED, !NOFB>(v, base, d, drow, dvec, words + row * W, W * 64, tb, p0, p1,
                      partials + static_cast<int64_t>(row) * tb.n_pieces, lds, sw_lds);
}

// STREAM: the error buffer is read and written non-temporally (see ds_sign_server).
template <bool DEFERRED, bool RMS, bool STREAM>
__global__ __launch_bounds__(kBlock) void k_sign_pass1_server(ServerArgs a, float *delta_s, int64_t d,
                                                              uint64_t *words_out, ds_sign_tables tb,
                                                              double *partials, const float *__restrict__ prev_scales)
{
    __shared__ double lds[kWaves];
    __shared__ __attribute__((aligned(16))) uint32_t sw_lds[kWaves * 8];
    const int64_t tile = blockIdx.x;
    const int64_t base = tile * kTile;
    const bool dvec = aligned16(delta_s);
    const TilePieces tp = tile_pieces(tb, tile);
    const int32_t p0 = tp.p0, p1 = tp.p1;
    const int64_t e = base + threadIdx.x * 4;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};                                      // no buffer: no server error
    if (delta_s) v = STREAM ? ld4_stream(delta_s, e, d, dvec) : ld4(delta_s, e, d, dvec);
    const int lane = lane_id();
    const int64_t wave_first = base + wave_id() * 256;
    // sign words of the first eight workers (lane L: word L & 7 of worker L >> 3): their
    // addresses do not depend on the tile's pieces, so they leave together with the table
    // entry and the error instead of after the scales that the entry leads to
    const bool word_in = wave_first + 32 * (lane & 7) < a.W * 64;
    uint32_t word0 = 0u;
    if ((lane >> 3) < a.n && word_in)
        word0 = reinterpret_cast<const uint32_t *>(a.words_in + (lane >> 3) * a.W)[(wave_first >> 5) + (lane & 7)];
    // scales of the first eight workers (lane i: worker i), asked for before the previous
    // call's scale below is waited for: both hang on the table entry alone
    float sc0 = 0.f;
    if (tp.seg0 >= 0 && lane < a.n && lane < 8) sc0 = a.scales_in[lane * a.S + tp.seg0];
    if (DEFERRED && e < d) v = sign_error_tile(v, e, d, prev_scales, tb, p0, p1, tp.seg0);   // past d: cleared below
    if (p1 - p0 == 1) {
        // the whole tile lies in one scale group: same batched loads as the chunk route
        const int32_t sg = tp.seg0;
        for (int i0 = 0; i0 < a.n; i0 += 8) {
            const int nb = (a.n - i0 < 8) ? a.n - i0 : 8;
            uint32_t word = word0;
            float sc = sc0;
            if (i0 > 0) {
                word = 0u;
                if ((lane >> 3) < nb && word_in)
                    word = reinterpret_cast<const uint32_t *>(a.words_in + (i0 + (lane >> 3)) * a.W)[(wave_first >> 5) + (lane & 7)];
                sc = (lane < nb) ? a.scales_in[(i0 + lane) * a.S + sg] : 0.f;
            }
            // lanes past d run the chain too (cleared below); a full batch is unrolled so that
            // its eight cross-lane fetches are in flight together
            const int top_shift = 28 - 4 * (lane & 7);
            if (nb == 8) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t w = __shfl(word, i * 8 + (lane >> 3), 64);
                    const float sv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sc), i));
                    v = chain4_top(v, w << top_shift, sv, a.inv_n);
                }
            } else {
                for (int i = 0; i < nb; ++i) {
                    const uint32_t w = __shfl(word, i * 8 + (lane >> 3), 64);
                    const float sv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sc), i));
                    v = chain4_top(v, w << top_shift, sv, a.inv_n);
                }
            }
        }
    } else if (e < d) {
        int32_t seg[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) seg[c] = (e + c < d) ? seg_of(tb, p0, p1, e + c) : 0;
        for (int i = 0; i < a.n; ++i) {
            const float *srow = a.scales_in + i * a.S;
            const uint32_t nib = load_sign_nibble(a.words_in + i * a.W, e);
            const float s0 = srow[seg[0]], s1 = srow[seg[1]], s2 = srow[seg[2]], s3 = srow[seg[3]];
            v = fma4(a.inv_n, signed4(s0, s1, s2, s3, nib), v);
        }
    }
    v = zero_past(v, e, d);
    pass1_finish<RMS, STREAM>(v, base, d, delta_s, dvec, words_out, a.W * 64, tb, p0, p1, partials, lds, sw_lds);
}

// scale[row][s] = (float)( sum of the group's partials / |group| ), fixed order.
// `keep` (may be null): the context's own copy of the scales, for the deferred error form.
__global__ __launch_bounds__(kBlock) void k_sign_reduce(const double *__restrict__ partials,
                                                        ds_sign_tables tb, float *scales, int64_t S, float *keep)
{
    __shared__ double lds[kWaves];
    const int32_t s = blockIdx.x;
    const int row = blockIdx.y;
    const double *prow = partials + static_cast<int64_t>(row) * tb.n_pieces;
    const bool whole = tb.whole_d > 0;
    const int32_t p0 = whole ? 0 : tb.seg_piece_first[s], p1 = whole ? tb.n_pieces : tb.seg_piece_first[s + 1];
    double acc = 0.0;
    for (int32_t p = p0 + threadIdx.x; p < p1; p += kBlock) acc += prow[p];
    const double total = block_sum(acc, lds, false);
    if (threadIdx.x == 0) {
        const double len = static_cast<double>(whole ? tb.whole_d : tb.seg_off[s + 1] - tb.seg_off[s]);
        const float sc = group_scale(total, len, tb.rms);
        scales[row * S + s] = sc;
        if (keep) keep[row * S + s] = sc;
    }
}

// Pass 2: the buffer holds v; overwrite with delta' = v - Q[v].
__global__ __launch_bounds__(kBlock) void k_sign_pass2(float *buf, int64_t stride, int64_t d,
                                                       const float *__restrict__ scales, int64_t S,
                                                       ds_sign_tables tb)
{
    // Pass 2 walks the rows and tiles in the opposite order to pass 1: what pass 1 wrote last
    // is still in the 256 MB memory-side cache, so those reads (and the v lines they
    // overwrite) never reach HBM.
    const int row = gridDim.y - 1 - blockIdx.y;
    const int64_t tile = gridDim.x - 1 - blockIdx.x;
    float *brow = buf + row * stride;
    const float *srow = scales + row * S;
    const bool vec = aligned16(brow);
    const TilePieces tp = tile_pieces(tb, tile);
    const int64_t e = tile * kTile + threadIdx.x * 4;
    if (e >= d) return;
    const f32x4 v = ld4_stream(brow, e, d, vec);
    st4_stream(brow, e, d, vec, sign_error_tile(v, e, d, srow, tb, tp.p0, tp.p1, tp.seg0));
}

template <bool MOM, bool DECODE_ONLY, bool STREAM>
__global__ __launch_bounds__(kBlock) void k_sign_update(const uint64_t *__restrict__ words,
                                                        const float *__restrict__ scales,
                                                        ds_sign_tables tb, float *x, float *m,
                                                        int64_t d, float gamma, float beta)
{
    const int64_t tile = blockIdx.x;
    const TilePieces tp = tile_pieces(tb, tile);
    const int64_t e = tile * kTile + threadIdx.x * 4;
    if (e >= d) return;
    // the model (and momentum) words leave before the scale that the table entry leads to is
    // waited for
    const bool xvec = aligned16(x), mvec = aligned16(m);
    f32x4 xv = {0.f, 0.f, 0.f, 0.f}, mv = xv;
    if constexpr (!DECODE_ONLY) {
        xv = STREAM ? ld4_stream(x, e, d, xvec) : ld4(x, e, d, xvec);
        if constexpr (MOM) mv = STREAM ? ld4_stream(m, e, d, mvec) : ld4(m, e, d, mvec);
    }
    const uint32_t nib = load_sign_nibble(words, e);
    float q[4];
    if (tp.seg0 >= 0) {
        const float s = scales[tp.seg0];
#pragma unroll
        for (int c = 0; c < 4; ++c) q[c] = (e + c < d) ? s : 0.f;
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) q[c] = (e + c < d) ? scales[seg_of(tb, tp.p0, tp.p1, e + c)] : 0.f;
    }
    f32x4 qv = signed4(q[0], q[1], q[2], q[3], nib);
    if constexpr (DECODE_ONLY) {
        st4_stream(x, e, d, xvec, qv);             // a decoded message: written once, read by the caller
    } else {
        if constexpr (MOM) {                       // m <- beta m + q ; x <- x - gamma m
            qv = fma4(beta, mv, qv);
            if constexpr (STREAM) st4_stream(m, e, d, mvec, qv);
            else st4(m, e, d, mvec, qv);
        }
        if constexpr (STREAM) st4_stream(x, e, d, xvec, fma4(-gamma, qv, xv));
        else st4(x, e, d, xvec, fma4(-gamma, qv, xv));
    }
}

// Server that does not compress (Section 5.1 "MEM-SGD"): a = (1/n) sum_i Q[v_i] by the chain
// from +0, per element: the element's bit and the scale of its group from every worker's
// message.  CHUNKS: the groups are chunks of `chunk` elements (a multiple of 4), else they come
// from the tile tables.
template <bool CHUNKS>
__global__ __launch_bounds__(kBlock) void k_sign_server_identity(ServerArgs a, int64_t d, int64_t chunk, ds_sign_tables tb,
                                                                 float *dense_out, ds_update_args u)
{
    const int64_t tile = blockIdx.x;
    const int64_t e = tile * kTile + threadIdx.x * 4;
    if (e >= d) return;
    int32_t seg[4];
    if constexpr (CHUNKS) {
        seg[0] = seg[1] = seg[2] = seg[3] = static_cast<int32_t>(static_cast<uint32_t>(e) / static_cast<uint32_t>(chunk));
    } else {
        const TilePieces tp = tile_pieces(tb, tile);
#pragma unroll
        for (int c = 0; c < 4; ++c) seg[c] = (tp.seg0 >= 0) ? tp.seg0 : ((e + c < d) ? seg_of(tb, tp.p0, tp.p1, e + c) : 0);
    }
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < a.n; ++i) {
        const float *srow = a.scales_in + i * a.S;
        const uint32_t nib = load_sign_nibble(a.words_in + i * a.W, e);
        v = fma4(a.inv_n, signed4(srow[seg[0]], srow[seg[1]], srow[seg[2]], srow[seg[3]], nib), v);
    }
    put_average4(zero_past(v, e, d), e, d, dense_out, u.x, u.m, u.gamma, u.beta);
}

}  // namespace

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
ds_status_t ds_sign_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st)
{
    const ds_config_t &cfg = c->cfg;
    ServerArgs a{in->sign_words, in->scales, cfg.n, c->W, c->S, c->inv_n};
    const unsigned blocks = static_cast<unsigned>(c->n_tiles);
    if (c->sign_fused) k_sign_server_identity<true><<<blocks, kBlock, 0, st>>>(a, cfg.d, cfg.chunk, c->sign_tb, dense_out, u);
    else k_sign_server_identity<false><<<blocks, kBlock, 0, st>>>(a, cfg.d, 0, c->sign_tb, dense_out, u);
    return ds_launch_status();
}

ds_status_t ds_sign_init(ds_ctx *c)
{
    const ds_config_t &cfg = c->cfg;
    const int64_t d = cfg.d;
    c->sign_fused = false;
    c->sign_defer = c->sign_w_deferred = c->sign_s_deferred = false;
    c->sign_prev_w = c->sign_prev_s = nullptr;
    c->sign_tb_mem = nullptr;
    c->sign_partials = nullptr;
    std::vector<int64_t> seg_off;
    if (cfg.scale_mode == DS_SCALE_WHOLE) {
        seg_off = {0, d};
    } else if (cfg.scale_mode == DS_SCALE_SEGMENTS) {
        seg_off.assign(cfg.seg_offsets, cfg.seg_offsets + cfg.n_seg + 1);
    } else {
        if (cfg.chunk % 128 == 0 && cfg.chunk >= 512 && cfg.chunk <= kTile) {
            c->sign_fused = true;
            c->S = (d + cfg.chunk - 1) / cfg.chunk;
            return DS_OK;
        }
        for (int64_t o = 0; o < d; o += cfg.chunk) seg_off.push_back(o);
        seg_off.push_back(d);
    }
    const int64_t S = static_cast<int64_t>(seg_off.size()) - 1;
    c->S = S;
    const int64_t n_tiles = c->n_tiles;
    std::vector<int32_t> tile_piece_first(n_tiles + 1), piece_seg, seg_piece_first(S + 1);
    std::vector<int2> tile_info(n_tiles);
    std::vector<int64_t> piece_start;
    int64_t s = 0;
    for (int64_t t = 0; t < n_tiles; ++t) {
        const int64_t lo = t * kTile, hi = (lo + kTile < d) ? lo + kTile : d;
        tile_piece_first[t] = static_cast<int32_t>(piece_start.size());
        int64_t pos = lo;
        while (pos < hi) {
            while (seg_off[s + 1] <= pos) ++s;
            if (pos == seg_off[s]) seg_piece_first[s] = static_cast<int32_t>(piece_start.size());
            piece_start.push_back(pos);
            piece_seg.push_back(static_cast<int32_t>(s));
            pos = (seg_off[s + 1] < hi) ? seg_off[s + 1] : hi;
        }
    }
    const int64_t n_pieces = static_cast<int64_t>(piece_seg.size());
    if (n_pieces > 0x7FFFFFFF) return DS_ERR_SHAPE;
    tile_piece_first[n_tiles] = static_cast<int32_t>(n_pieces);
    seg_piece_first[S] = static_cast<int32_t>(n_pieces);
    piece_start.push_back(d);
    for (int64_t t = 0; t < n_tiles; ++t) {
        const int32_t p0 = tile_piece_first[t], cnt = tile_piece_first[t + 1] - p0;
        tile_info[t] = int2{p0, cnt == 1 ? piece_seg[p0] : -cnt};
    }

    // one allocation: int64 arrays first (8-byte aligned), then the int32 arrays
    const size_t b_ps = sizeof(int64_t) * (n_pieces + 1), b_so = sizeof(int64_t) * (S + 1);
    const size_t b_tpf = sizeof(int32_t) * (n_tiles + 1), b_pseg = sizeof(int32_t) * n_pieces;
    const size_t b_spf = sizeof(int32_t) * (S + 1), b_ti = sizeof(int2) * n_tiles;
    char *mem = nullptr;
    DS_HIP_TRY(hipMalloc(&mem, b_ps + b_so + b_ti + b_tpf + b_pseg + b_spf));
    c->sign_tb_mem = mem;
    char *p = mem;
    auto put = [&](const void *src, size_t bytes) -> const void * {
        const void *at = p;
        if (bytes) (void)hipMemcpy(p, src, bytes, hipMemcpyHostToDevice);
        p += bytes;
        return at;
    };
    c->sign_tb.piece_start = static_cast<const int64_t *>(put(piece_start.data(), b_ps));
    c->sign_tb.seg_off = static_cast<const int64_t *>(put(seg_off.data(), b_so));
    c->sign_tb.tile_info = static_cast<const int2 *>(put(tile_info.data(), b_ti));
    c->sign_tb.tile_piece_first = static_cast<const int32_t *>(put(tile_piece_first.data(), b_tpf));
    c->sign_tb.piece_seg = static_cast<const int32_t *>(put(piece_seg.data(), b_pseg));
    c->sign_tb.seg_piece_first = static_cast<const int32_t *>(put(seg_piece_first.data(), b_spf));
    c->sign_tb.n_pieces = static_cast<int32_t>(n_pieces);
    c->sign_tb.n_seg = static_cast<int32_t>(S);
    c->sign_tb.rms = (cfg.flags & DS_FLAG_SIGN_RMS) != 0;
    c->sign_tb.whole_d = 0;
    if (hipGetLastError() != hipSuccess) return DS_ERR_DEVICE;
    DS_HIP_TRY(hipMalloc(&c->sign_partials, sizeof(double) * n_pieces * static_cast<size_t>(cfg.n)));
    if ((cfg.flags & DS_FLAG_DEFERRED_ERROR) && !c->nofb) {
        c->sign_defer = true;
        DS_HIP_TRY(hipMalloc(&c->sign_prev_w, sizeof(float) * static_cast<size_t>(S) * cfg.n));
        DS_HIP_TRY(hipMalloc(&c->sign_prev_s, sizeof(float) * static_cast<size_t>(S)));
    }
    return DS_OK;
}

void ds_sign_fini(ds_ctx *c)
{
    if (c->sign_tb_mem) (void)hipFree(c->sign_tb_mem);
    if (c->sign_partials) (void)hipFree(c->sign_partials);
    if (c->sign_prev_w) (void)hipFree(c->sign_prev_w);
    if (c->sign_prev_s) (void)hipFree(c->sign_prev_s);
    c->sign_prev_w = c->sign_prev_s = nullptr;
    c->sign_tb_mem = nullptr;
    c->sign_partials = nullptr;
}

// Calls f with the run-time flags turned into compile-time constants (std::bool_constant).
template <class F>
static void with_flags(bool a, bool b, bool c, F f)
{
    auto l2 = [&](auto ta, auto tb) { if (c) f(ta, tb, std::true_type{}); else f(ta, tb, std::false_type{}); };
    auto l1 = [&](auto ta) { if (b) l2(ta, std::true_type{}); else l2(ta, std::false_type{}); };
    if (a) l1(std::true_type{}); else l1(std::false_type{});
}

ds_status_t ds_sign_worker(ds_ctx *c, const void *g, int64_t gs, float *delta, int64_t dstr,
                           const ds_payload_t *out, hipStream_t st)
{
    const ds_config_t &cfg = c->cfg;
    const bool bf16 = cfg.grad_dtype == DS_BF16;
    const bool rms = (cfg.flags & DS_FLAG_SIGN_RMS) != 0;
    if (c->sign_fused) {
        with_flags(bf16, rms, c->nofb, [&](auto bf, auto rm, auto nf) {
            constexpr bool BF = decltype(bf)::value, RM = decltype(rm)::value, NF = decltype(nf)::value;
            constexpr int CPW = NF ? 4 : 2;
            const dim3 grid(static_cast<unsigned>((c->S + CPW - 1) / CPW), static_cast<unsigned>(cfg.n));
            WorkerSrc<BF> src{g, gs, delta, dstr};
            k_sign_chunk_worker<BF, RM, NF, CPW><<<grid, kBlock, 0, st>>>(src, delta, cfg.d, cfg.chunk, out->sign_words, c->W,
                                                                          out->scales, c->S);
        });
        return ds_launch_status();
    }
    dim3 grid(static_cast<unsigned>(c->n_tiles), static_cast<unsigned>(cfg.n));
    const bool deferred = c->sign_defer && c->sign_w_deferred;     // never set without compensation
    with_flags(bf16, deferred || c->nofb, rms, [&](auto bf, auto md, auto rm) {
        constexpr bool BF = decltype(bf)::value, MD = decltype(md)::value, RM = decltype(rm)::value;
        WorkerSrc<BF> src{g, gs, delta, dstr};
        if (!MD)
            k_sign_pass1_worker<BF, 0, RM><<<grid, kBlock, 0, st>>>(src, delta, cfg.d, out->sign_words, c->W, c->sign_tb,
                                                                    c->sign_partials, c->sign_prev_w, c->S);
        else if (deferred)
            k_sign_pass1_worker<BF, 1, RM><<<grid, kBlock, 0, st>>>(src, delta, cfg.d, out->sign_words, c->W, c->sign_tb,
                                                                    c->sign_partials, c->sign_prev_w, c->S);
        else
            k_sign_pass1_worker<BF, 2, RM><<<grid, kBlock, 0, st>>>(src, delta, cfg.d, out->sign_words, c->W, c->sign_tb,
                                                                    c->sign_partials, c->sign_prev_w, c->S);
    });
    k_sign_reduce<<<dim3(static_cast<unsigned>(c->S), static_cast<unsigned>(cfg.n)), kBlock, 0, st>>>(
        c->sign_partials, c->sign_tb, out->scales, c->S, c->sign_defer ? c->sign_prev_w : nullptr);
    if (!c->sign_defer && delta) k_sign_pass2<<<grid, kBlock, 0, st>>>(delta, dstr, cfg.d, out->scales, c->S, c->sign_tb);
    const ds_status_t rc = ds_launch_status();
    if (rc == DS_OK && c->sign_defer) c->sign_w_deferred = true;   // the buffer now holds v; delta = v - Q[v] is applied by the next load
    return rc;
}

// x != nullptr (chunk route only): the model update for the same elements in the same kernel.
ds_status_t ds_sign_server(ds_ctx *c, const ds_payload_t *in, float *delta_s, const ds_payload_t *out,
                           hipStream_t st, float *x, float *m, float gamma, float beta)
{
    const ds_config_t &cfg = c->cfg;
    ServerArgs a{in->sign_words, in->scales, cfg.n, c->W, c->S, c->inv_n};
    const bool rms = (cfg.flags & DS_FLAG_SIGN_RMS) != 0;
    if (c->sign_fused) {
        // two chunks per workgroup: more bytes in flight per thread (measured 271 us against
        // 292 us with one and 285 us with four on the 124 M-element workload)
        const dim3 grid(static_cast<unsigned>((c->S + 1) / 2));
        auto launch = [&](auto rm, auto upd) {
            constexpr bool RM = decltype(rm)::value;
            constexpr int UPD = decltype(upd)::value;
            k_sign_chunk_server<2, RM, UPD><<<grid, kBlock, 0, st>>>(a, delta_s, cfg.d, cfg.chunk, out->sign_words, out->scales,
                                                                      x, m, gamma, beta);
        };
        auto with_upd = [&](auto rm) {
            if (!x) launch(rm, std::integral_constant<int, 0>{});
            else if (!m) launch(rm, std::integral_constant<int, 1>{});
            else launch(rm, std::integral_constant<int, 2>{});
        };
        if (rms) with_upd(std::true_type{}); else with_upd(std::false_type{});
        return ds_launch_status();
    }
    if (x) return DS_ERR_UNSUPPORTED;   // the caller asks for the fused form on the chunk route only
    dim3 grid(static_cast<unsigned>(c->n_tiles));
    const bool deferred = c->sign_defer && c->sign_s_deferred && delta_s;
    // Deferred form: the buffer is looked at once per call, so it may stream past the caches.
    // Measured on the 11 M-element workload (45 MB per buffer) that costs more than it saves:
    // server call 35.0 us streamed, 33.7 us with ordinary accesses, the next worker pass 1 us
    // slower; the 124 M-element measurements that led to streaming stand for large buffers.
    const bool stream = deferred && ds_stream_worthwhile(cfg.d);
    with_flags(deferred, rms, stream, [&](auto df, auto rm, auto sm) {
        constexpr bool DF = decltype(df)::value, RM = decltype(rm)::value, SM = decltype(sm)::value;
        k_sign_pass1_server<DF, RM, SM><<<grid, kBlock, 0, st>>>(a, delta_s, cfg.d, out->sign_words, c->sign_tb, c->sign_partials,
                                                             deferred ? c->sign_prev_s : nullptr);
    });
    k_sign_reduce<<<dim3(static_cast<unsigned>(c->S), 1), kBlock, 0, st>>>(c->sign_partials, c->sign_tb, out->scales, c->S,
                                                                          c->sign_defer ? c->sign_prev_s : nullptr);
    if (!c->sign_defer && delta_s) k_sign_pass2<<<grid, kBlock, 0, st>>>(delta_s, cfg.d, cfg.d, out->scales, c->S, c->sign_tb);
    const ds_status_t rc = ds_launch_status();
    if (rc == DS_OK && c->sign_defer) c->sign_s_deferred = true;
    return rc;
}

// Deferred error form -> plain form, in place; a no-op for buffers that are in plain form.
ds_status_t ds_sign_materialize(ds_ctx *c, float *delta, int64_t dstr, float *delta_s, hipStream_t st)
{
    const ds_config_t &cfg = c->cfg;
    if (!c->sign_defer) return DS_OK;
    if (delta && c->sign_w_deferred) {
        k_sign_pass2<<<dim3(static_cast<unsigned>(c->n_tiles), static_cast<unsigned>(cfg.n)), kBlock, 0, st>>>(
            delta, dstr, cfg.d, c->sign_prev_w, c->S, c->sign_tb);
        c->sign_w_deferred = false;
    }
    if (delta_s && c->sign_s_deferred) {
        k_sign_pass2<<<dim3(static_cast<unsigned>(c->n_tiles)), kBlock, 0, st>>>(delta_s, cfg.d, cfg.d, c->sign_prev_s, c->S,
                                                                                c->sign_tb);
        c->sign_s_deferred = false;
    }
    return ds_launch_status();
}

template <bool DECODE_ONLY>
static ds_status_t sign_update_impl(ds_ctx *c, const uint64_t *words, const float *scales, float *x, float *m,
                                    float gamma, float beta, hipStream_t st)
{
    const ds_config_t &cfg = c->cfg;
    if (c->sign_fused) {
        const unsigned blocks = static_cast<unsigned>((cfg.d + kBlock * 4 - 1) / (kBlock * 4));
        if (m && !DECODE_ONLY)
            k_sign_chunk_update<true, false><<<blocks, kBlock, 0, st>>>(words, scales, cfg.chunk, x, m, cfg.d, gamma, beta);
        else
            k_sign_chunk_update<false, DECODE_ONLY><<<blocks, kBlock, 0, st>>>(words, scales, cfg.chunk, x, m, cfg.d, gamma, beta);
    } else {
        const unsigned blocks = static_cast<unsigned>(c->n_tiles);
        // ordinary accesses to a small model: 20.4 us -> 18.8 us on the 11 M-element workload
        const bool stream = DECODE_ONLY || ds_stream_worthwhile(cfg.d);
        if (m && !DECODE_ONLY) {
            if (stream) k_sign_update<true, false, true><<<blocks, kBlock, 0, st>>>(words, scales, c->sign_tb, x, m, cfg.d, gamma, beta);
            else k_sign_update<true, false, false><<<blocks, kBlock, 0, st>>>(words, scales, c->sign_tb, x, m, cfg.d, gamma, beta);
        } else {
            if (stream) k_sign_update<false, DECODE_ONLY, true><<<blocks, kBlock, 0, st>>>(words, scales, c->sign_tb, x, m, cfg.d, gamma, beta);
            else k_sign_update<false, DECODE_ONLY, false><<<blocks, kBlock, 0, st>>>(words, scales, c->sign_tb, x, m, cfg.d, gamma, beta);
        }
    }
    return ds_launch_status();
}

ds_status_t ds_sign_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma, float beta,
                           hipStream_t st)
{
    return sign_update_impl<false>(c, srv->sign_words, srv->scales, x, m, gamma, beta, st);
}

ds_status_t ds_sign_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st)
{
    return sign_update_impl<true>(c, p->sign_words + row * c->W, p->scales + row * c->S, out, nullptr, 0.f, 0.f, st);
}

// ---------------------------------------------------------------------------------------
// the worker block without a context and without any allocation
// ---------------------------------------------------------------------------------------
// The general route needs the fp64 partial sums of every tile between its first pass and the
// reduce.  ds_create allocates them; callers that cannot allocate get them from this fixed
// array instead (one copy per device, held until the process ends).
#define DS_NOALLOC_MAX_PARTIALS 65536
static __device__ __align__(256) double scratch[DS_NOALLOC_MAX_PARTIALS];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, looked up once
}  // namespace

extern "C" ds_status_t ds_worker_compress_sign_noalloc(int32_t n, int64_t d, int32_t grad_dtype, int32_t flags,
                                                       const void *g, int64_t g_row_stride, float *delta,
                                                       int64_t delta_row_stride, uint64_t *sign_words, float *scales,
                                                       void *hip_stream)
{
    if (!g || !delta || !sign_words || !scales) return DS_ERR_NULL;
    if (n < 1 || n > 65535 || d < 1 || d > 0x7FFFFFFFLL) return DS_ERR_SHAPE;
    if (g_row_stride < d || delta_row_stride < d) return DS_ERR_SHAPE;
    if (grad_dtype != DS_F32 && grad_dtype != DS_BF16) return DS_ERR_CONFIG;
    if (flags & ~static_cast<int32_t>(DS_FLAG_SIGN_RMS)) return DS_ERR_CONFIG;
    const int64_t n_tiles = (d + kTile - 1) / kTile;
    if (n_tiles * n > DS_NOALLOC_MAX_PARTIALS) return DS_ERR_SHAPE;
    auto misaligned = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
    if (misaligned(g) || misaligned(delta) || misaligned(sign_words) || misaligned(scales)) return DS_ERR_ALIGN;
    int dev = -1;
    DS_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return DS_ERR_DEVICE;
    double *partials = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            // every device holds its own copy of the array at its own address
            void *p = nullptr;
            DS_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            g_scratch_ptr[dev] = static_cast<double *>(p);
        }
        partials = g_scratch_ptr[dev];
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    ds_sign_tables tb{};
    tb.n_pieces = static_cast<int32_t>(n_tiles);
    tb.n_seg = 1;
    tb.rms = (flags & DS_FLAG_SIGN_RMS) != 0;
    tb.whole_d = d;
    const int64_t W = (d + 63) / 64;
    const dim3 grid(static_cast<unsigned>(n_tiles), static_cast<unsigned>(n));
    with_flags(grad_dtype == DS_BF16, tb.rms, false, [&](auto bf, auto rm, auto) {
        constexpr bool BF = decltype(bf)::value, RM = decltype(rm)::value;
        WorkerSrc<BF> src{g, g_row_stride, delta, delta_row_stride};
        k_sign_pass1_worker<BF, 0, RM><<<grid, kBlock, 0, st>>>(src, delta, d, sign_words, W, tb, partials, nullptr, 1);
    });
    k_sign_reduce<<<dim3(1, static_cast<unsigned>(n)), kBlock, 0, st>>>(partials, tb, scales, 1, nullptr);
    k_sign_pass2<<<grid, kBlock, 0, st>>>(delta, delta_row_stride, d, scales, 1, tb);
    return ds_launch_status();
}
