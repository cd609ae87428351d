// Device-side helpers shared by the gfx950 kernels of the DoubleSqueeze step.
//
// Tile geometry used by every dense kernel: a workgroup of 512 threads (8 wavefronts of
// 64 lanes) owns a tile of 2048 consecutive elements that starts at a multiple of 2048.
// Thread t touches the four consecutive elements
//     tile_base + 4*t + {0,1,2,3}
// so that one wavefront instruction moves 64 x 16 B = 1 KiB of contiguous fp32 data
// (128-bit loads), and a wavefront's 256 elements are exactly four 64-bit words of the sign
// plane.  One 128-bit load per thread and many resident wavefronts measured faster on
// MI355X than fewer threads with several loads each (copy kernel: 6.26 TB/s with one
// load per thread against 5.65 TB/s with four).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ds {

constexpr int kBlock = 512;
constexpr int kWaves = kBlock / 64;
constexpr int kTile = 2048;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
__device__ __forceinline__ bool aligned8(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 7u) == 0; }

typedef float f32x2 __attribute__((ext_vector_type(2)));

// Four consecutive fp32 elements e..e+3 of a row, zero where e+c >= lim.  `vec` = the row
// starts on a 16-byte boundary.  Rows that start on an 8-byte boundary only (contiguous
// [n, d] with d = 2 mod 4) take two 64-bit accesses instead of four 32-bit ones; e is a
// multiple of 4, so the row's alignment is that of every access.
__device__ __forceinline__ f32x4 ld4(const float *__restrict__ row, int64_t e, int64_t lim, bool vec)
{
    if (vec && e + 4 <= lim) return *reinterpret_cast<const f32x4 *>(row + e);
    if (!vec && e + 4 <= lim && aligned8(row)) {
        const f32x2 a = *reinterpret_cast<const f32x2 *>(row + e), b = *reinterpret_cast<const f32x2 *>(row + e + 2);
        return f32x4{a.x, a.y, b.x, b.y};
    }
    f32x4 r = {0.f, 0.f, 0.f, 0.f};
    if (e < lim) r.x = row[e];
    if (e + 1 < lim) r.y = row[e + 1];
    if (e + 2 < lim) r.z = row[e + 2];
    if (e + 3 < lim) r.w = row[e + 3];
    return r;
}

// Same, streaming (read once): bypasses cache retention.
__device__ __forceinline__ f32x4 ld4_stream(const float *__restrict__ row, int64_t e, int64_t lim, bool vec)
{
    if (vec && e + 4 <= lim) return __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(row + e));
    if (!vec && e + 4 <= lim && aligned8(row)) {
        const f32x2 a = __builtin_nontemporal_load(reinterpret_cast<const f32x2 *>(row + e));
        const f32x2 b = __builtin_nontemporal_load(reinterpret_cast<const f32x2 *>(row + e + 2));
        return f32x4{a.x, a.y, b.x, b.y};
    }
    return ld4(row, e, lim, false);
}

__device__ __forceinline__ float bf16_widen(uint32_t h) { return __uint_as_float(h << 16); }

// Four consecutive bf16 elements widened exactly to fp32.
__device__ __forceinline__ f32x4 ld4_bf16(const uint16_t *__restrict__ row, int64_t e, int64_t lim, bool vec)
{
    f32x4 r = {0.f, 0.f, 0.f, 0.f};
    if (vec && e + 4 <= lim) {
        u32x2 u = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(row + e));
        r.x = __uint_as_float(u.x << 16);
        r.y = __uint_as_float(u.x & 0xFFFF0000u);
        r.z = __uint_as_float(u.y << 16);
        r.w = __uint_as_float(u.y & 0xFFFF0000u);
        return r;
    }
    if (!vec && e + 4 <= lim && (reinterpret_cast<uintptr_t>(row) & 3u) == 0) {   // 4-byte aligned row: two 32-bit loads
        const uint32_t a = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(row + e));
        const uint32_t b = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(row + e + 2));
        return f32x4{__uint_as_float(a << 16), __uint_as_float(a & 0xFFFF0000u), __uint_as_float(b << 16),
                     __uint_as_float(b & 0xFFFF0000u)};
    }
    if (e < lim) r.x = bf16_widen(row[e]);
    if (e + 1 < lim) r.y = bf16_widen(row[e + 1]);
    if (e + 2 < lim) r.z = bf16_widen(row[e + 2]);
    if (e + 3 < lim) r.w = bf16_widen(row[e + 3]);
    return r;
}

__device__ __forceinline__ void st4(float *__restrict__ row, int64_t e, int64_t lim, bool vec, f32x4 v)
{
    if (vec && e + 4 <= lim) { *reinterpret_cast<f32x4 *>(row + e) = v; return; }
    if (!vec && e + 4 <= lim && aligned8(row)) {
        *reinterpret_cast<f32x2 *>(row + e) = f32x2{v.x, v.y};
        *reinterpret_cast<f32x2 *>(row + e + 2) = f32x2{v.z, v.w};
        return;
    }
    if (e < lim) row[e] = v.x;
    if (e + 1 < lim) row[e + 1] = v.y;
    if (e + 2 < lim) row[e + 2] = v.z;
    if (e + 3 < lim) row[e + 3] = v.w;
}

// Store of state that is rewritten in place and not read again before the next call.  A
// buffer that is read and written in the same pass is fastest with BOTH sides non-temporal:
// in-place g + delta -> delta over 8 x 25.6 M elements took 441 us with plain accesses to
// delta, 480 us with only the load non-temporal, 438 us with only the store, 399 us with both
// (424 us out of place).
__device__ __forceinline__ void st4_stream(float *__restrict__ row, int64_t e, int64_t lim, bool vec, f32x4 v)
{
    if (vec && e + 4 <= lim) { __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(row + e)); return; }
    st4(row, e, lim, vec, v);
}

// Gradient row of either dtype.
template <bool BF16>
__device__ __forceinline__ f32x4 ld4_grad(const void *__restrict__ row, int64_t e, int64_t lim, bool vec)
{
    if constexpr (BF16) return ld4_bf16(static_cast<const uint16_t *>(row), e, lim, vec);
    else return ld4_stream(static_cast<const float *>(row), e, lim, vec);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// Lane exchange inside a row of 16 lanes by data-parallel-primitive controls: no index
// arithmetic and no trip through the LDS crossbar.  Every lane of the wavefront must be active.
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]: lane i reads lane i ^ 1
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]: lane i reads lane i ^ 2
constexpr int kDppHalfMirror = 0x141;  // lane i of an 8-lane group reads lane 7 - i: the other quad
constexpr int kDppRowMirror = 0x140;   // lane i of a 16-lane row reads lane 15 - i: the other 8-lane group

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x)
{
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, 0xF, 0xF, true));
}

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x)
{
    const uint64_t b = __double_as_longlong(x);
    const uint64_t lo = dpp_u32<CTRL>(static_cast<uint32_t>(b)), hi = dpp_u32<CTRL>(static_cast<uint32_t>(b >> 32));
    return __longlong_as_double(static_cast<long long>(lo | (hi << 32)));
}

// Sum over each aligned group of 16 lanes; every lane of a group returns the same value (each
// step adds the same two partial sums on both sides), the order is fixed.
__device__ __forceinline__ double row_sum(double x)
{
    x += dpp_f64<kDppXor1>(x);
    x += dpp_f64<kDppXor2>(x);
    x += dpp_f64<kDppHalfMirror>(x);
    x += dpp_f64<kDppRowMirror>(x);
    return x;
}

// x of this lane plus x of the lane 16 (ROWS = 16) or 32 (ROWS = 32) away, lane i ^ ROWS: the
// gfx950 row-swap instruction exchanges the odd rows of one copy with the even rows of another,
// after which one copy holds the even row's value in both rows of a pair and the other the odd
// row's.  Both lanes of a pair add the same two numbers in the same order.
template <int ROWS>
__device__ __forceinline__ double pair_row_sum(double x)
{
    const uint64_t b = __double_as_longlong(x);
    const uint32_t lo = static_cast<uint32_t>(b), hi = static_cast<uint32_t>(b >> 32);
    uint32_t lo0, lo1, hi0, hi1;
    if constexpr (ROWS == 16) {
        const auto l = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto h = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        lo0 = l[0]; lo1 = l[1]; hi0 = h[0]; hi1 = h[1];
    } else {
        const auto l = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        const auto h = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        lo0 = l[0]; lo1 = l[1]; hi0 = h[0]; hi1 = h[1];
    }
    return __longlong_as_double(static_cast<long long>(lo0 | (static_cast<uint64_t>(hi0) << 32))) +
           __longlong_as_double(static_cast<long long>(lo1 | (static_cast<uint64_t>(hi1) << 32)));
}

// Sum over the 64 lanes; every lane returns the same value, the order is fixed.
__device__ __forceinline__ double wave_sum(double x)
{
    x = row_sum(x);
    x = pair_row_sum<16>(x);
    x = pair_row_sum<32>(x);
    return x;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x)
{
    x += dpp_u32<kDppXor1>(x);
    x += dpp_u32<kDppXor2>(x);
    x += dpp_u32<kDppHalfMirror>(x);
    x += dpp_u32<kDppRowMirror>(x);
    const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    x = a[0] + a[1];
    const auto b = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return b[0] + b[1];
}

// Inclusive prefix sum over the 64 lanes: four shifted adds inside each row of 16 lanes (lanes
// shifted in from outside the row read 0), then the total of row 0 (its lane 15) goes to row 1
// and that of row 2 to row 3, then the total of rows 0-1 (lane 31) to rows 2 and 3.  Every lane
// of the wavefront must be active.
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t x)
{
    x += dpp_u32<0x111>(x);   // row_shr:1
    x += dpp_u32<0x112>(x);   // row_shr:2
    x += dpp_u32<0x114>(x);   // row_shr:4
    x += dpp_u32<0x118>(x);   // row_shr:8
    x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x142, 0xA, 0xF, false));   // row_bcast:15 into rows 1, 3
    x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x143, 0xC, 0xF, false));   // row_bcast:31 into rows 2, 3
    return x;
}

// Sum over the threads of the workgroup in a fixed order; lds holds kWaves doubles.
// Every thread returns the total.  `guard` = the buffer may still be read from an earlier
// call (adds a barrier in front).
__device__ __forceinline__ double block_sum(double x, double *lds, bool guard = true)
{
    const double w = wave_sum(x);
    if (guard) __syncthreads();
    if (lane_id() == 0) lds[wave_id()] = w;
    __syncthreads();
    double t = lds[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) t += lds[i];
    return t;
}

__device__ __forceinline__ uint32_t spread4(uint32_t x)   // bit i of the low byte -> bit 4 i
{
    x = (x | (x << 12)) & 0x000F000Fu;
    x = (x | (x << 6)) & 0x03030303u;
    x = (x | (x << 3)) & 0x11111111u;
    return x;
}

// Sign-plane packing.  Each lane passes the "negative" flags of its four consecutive elements;
// the wavefront's 256 elements form eight 32-bit words of the plane (element j of the wavefront
// = bit j & 31 of word j >> 5), word q from lanes 8q .. 8q+7.  Every lane returns the word of
// its own 8-lane group: the lane's four bits are shifted to their place and the eight lanes
// are OR-ed together in three cross-lane steps.  Every lane of the wavefront must be active.
__device__ __forceinline__ uint32_t wave_sign_word(bool n0, bool n1, bool n2, bool n3)
{
    const uint32_t nib = static_cast<uint32_t>(n0) | (static_cast<uint32_t>(n1) << 1) |
                         (static_cast<uint32_t>(n2) << 2) | (static_cast<uint32_t>(n3) << 3);
    uint32_t w = nib << (4 * (lane_id() & 7));
    w |= dpp_u32<kDppXor1>(w);
    w |= dpp_u32<kDppXor2>(w);
    w |= dpp_u32<kDppHalfMirror>(w);
    return w;
}

// Every wavefront deposits its eight words in `sw_lds` (64 words, 16-byte aligned) with stash_sign_words BEFORE a workgroup barrier; AFTER it, flush_sign_words writes
// the tile's 256 bytes (tile_first = first element of the 2048-element tile) as one
// non-temporal store of 16 x 16 bytes.  Only 128-bit groups whose first element is below
// `bit_lim` are written; bit_lim is a multiple of 64: the end of the caller's chunk, or
// 64*ceil(d/64) at the end of the row so that the pad bits of the last word are written as zero.
// Measured on the fused sign worker pass while the error buffer was still accessed with
// plain loads and stores: the 1.2 % side stream of sign words cost 9 % with ordinary stores
// per wavefront (1.77 ms against 1.61 ms without them), 1.69 ms with one non-temporal 32-byte
// store per wavefront and 1.66 ms with a single non-temporal store per workgroup.  With the
// error buffer streamed non-temporally the words are best left in the cache for the server
// that reads them next: 1.668 ms with a plain store here against 1.682 ms non-temporal.
__device__ __forceinline__ void stash_sign_words(uint32_t *sw_lds, uint32_t word)
{
    if ((lane_id() & 7) == 0) sw_lds[wave_id() * 8 + (lane_id() >> 3)] = word;
}

__device__ __forceinline__ void flush_sign_words(const uint32_t *sw_lds, uint64_t *__restrict__ words_row,
                                                 int64_t tile_first, int64_t bit_lim)
{
    const int t = threadIdx.x;
    if (t < 16 && tile_first + 128 * t < bit_lim) {
        uint32_t *dst = reinterpret_cast<uint32_t *>(words_row) + (tile_first >> 5) + 4 * t;
        const u32x4 w4 = reinterpret_cast<const u32x4 *>(sw_lds)[t];
        if (tile_first + 128 * (t + 1) <= bit_lim) {
            *reinterpret_cast<u32x4 *>(dst) = w4;
        } else {                                  // bit_lim is a multiple of 64: two of the four words
            dst[0] = w4.x;
            dst[1] = w4.y;
        }
    }
}

// The four sign bits of elements e..e+3 (e a multiple of 4) read from a sign plane.
__device__ __forceinline__ uint32_t load_sign_nibble(const uint64_t *__restrict__ words_row, int64_t e)
{
    const uint32_t byte = reinterpret_cast<const uint8_t *>(words_row)[e >> 3];
    return (byte >> (e & 4)) & 15u;
}

// a ^ b ^ c as one three-input bit operation (truth table 0x96) of gfx950; the compiler emits
// two exclusive-ors for the plain expression.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies.
__device__ __forceinline__ u32x4 philox4x32_10(u32x4 c, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c.x;
        const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c.z;
        u32x4 nx;
        nx.x = xor3(static_cast<uint32_t>(p1 >> 32), c.y, k0);
        nx.y = static_cast<uint32_t>(p1);
        nx.z = xor3(static_cast<uint32_t>(p0 >> 32), c.w, k1);
        nx.w = static_cast<uint32_t>(p0);
        c = nx;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c;
}

// Zeroes the components of e..e+3 that lie at or past lim.
__device__ __forceinline__ f32x4 zero_past(f32x4 v, int64_t e, int64_t lim)
{
    if (e + 0 >= lim) v.x = 0.f;
    if (e + 1 >= lim) v.y = 0.f;
    if (e + 2 >= lim) v.z = 0.f;
    if (e + 3 >= lim) v.w = 0.f;
    return v;
}

__device__ __forceinline__ f32x4 fma4(float a, f32x4 b, f32x4 c)
{
    return f32x4{__fmaf_rn(a, b.x, c.x), __fmaf_rn(a, b.y, c.y), __fmaf_rn(a, b.z, c.z), __fmaf_rn(a, b.w, c.w)};
}

// Tail shared by every update kernel (Algorithm 1, last worker block), q = decoded
// server message for elements e..e+3:
//   DECODE_ONLY: x <- q ;  plain: x <- fma(-gamma, q, x) ;
//   MOM: m <- fma(beta, m, q), x <- fma(-gamma, m, x).
template <bool MOM, bool DECODE_ONLY>
__device__ __forceinline__ void apply_q4(f32x4 q, int64_t e, int64_t d, float *x, float *m, float gamma, float beta)
{
    const bool xvec = aligned16(x);
    if constexpr (DECODE_ONLY) {
        st4_stream(x, e, d, xvec, q);
    } else {
        const f32x4 xv = ld4_stream(x, e, d, xvec);
        if constexpr (MOM) {
            const bool mvec = aligned16(m);
            q = fma4(beta, ld4_stream(m, e, d, mvec), q);
            st4_stream(m, e, d, mvec, q);
        }
        st4_stream(x, e, d, xvec, fma4(-gamma, q, xv));
    }
}

// Server that sends its average back uncompressed: a = (1/n) sum_i Q[v_i] for elements e..e+3 is
// the message.  dense_out != nullptr: written there; x != nullptr: the model update from it
// (through the momentum buffer if m != nullptr).
__device__ __forceinline__ void put_average4(f32x4 a, int64_t e, int64_t d, float *dense_out, float *x, float *m,
                                             float gamma, float beta)
{
    if (dense_out) st4(dense_out, e, d, aligned16(dense_out), a);
    if (x) {
        if (m) apply_q4<true, false>(a, e, d, x, m, gamma, beta);
        else apply_q4<false, false>(a, e, d, x, m, gamma, beta);
    }
}

}  // namespace ds
