// Top-k sparsification kernels (Section 3.2 "Top-k sparsification", Section 5.1 "Top-k
// compression" of the DoubleSqueeze paper): keep the k entries of largest absolute value,
// zero the rest.  The message lists (index, value) by ascending index; equal magnitudes are
// resolved towards the lower index.
//
// Selection is exact and deterministic: a radix select on the 31-bit magnitude pattern
// key = bits(v) & 0x7FFFFFFF, arranged so that the dense vector is looked at ONCE:
//   sample     512 evenly spread 256-element subtiles of v are histogrammed: 12 key bits,
//              and 20 key bits inside a one-octave window around the threshold key of the
//              previous call (kept per row in the context; the result never depends on it).
//              The sample's r-th largest key, r about 1.15 k |sample| / d, is a lower bound
//              lo_key for the k-th key with overwhelming probability.  The fine window
//              matters: error feedback piles values up just below the threshold, and a
//              12-bit bin edge would let in up to twice as many candidates.
//   pass 1     (dense, the one HBM pass) v is formed and written into the error buffer, with
//              0 at the positions of candidates = elements with key >= lo_key.  A workgroup
//              compacts the candidates of its 2048-element tile, in index order, into the
//              tile's fixed slot region (ballots, wavefront totals through LDS): no shared
//              counters.
//   refine     over the candidates only (about 1.2 k of them): histograms relative to lo_key,
//              each followed by a pick of the bin that holds the k-th key -> exact threshold
//              key T and the number of ties at T to keep; then, per 32768-element group in
//              order, entries above T plus the first ties by index are written at offsets
//              from running sums over the groups, so the output is sorted by index without a
//              sort, and candidates that are not kept get v back in the error buffer
//              (delta = v - Q[v] is 0 at kept positions and v elsewhere).
//   verify     if the candidates number fewer than k, or the k-th key lies outside the
//              histogram window (the sample misjudged), the row takes the exact two-look
//              route: v restored, dense 12-bit histogram, pick, dense compaction.
// The refinement exists twice: as ONE launch whose workgroups are all resident and wait for
// each other per row (k_topk_finish, the default), and as a chain of small launches in which
// the last workgroup of a row finishes each step (12 + 11 + 8 key bits), for contexts whose
// calls may overlap on the device.  Nothing depends on scheduling order, so results are
// bit-reproducible and the two routes agree bit for bit.
#include "ds_device.h"
#include "ds_internal.h"

#include <new>
#include <type_traits>

using namespace ds;

namespace {

constexpr int kSub = 256;                  // elements per subtile = one wavefront of the dense pass
constexpr int kReg = kTile;                // elements per candidate region = one workgroup of the dense pass
constexpr int kGroupRegs = 16;             // regions per group (32768 elements) = one wavefront of the candidate passes
constexpr int kH1 = 4096, kH2 = 2048, kH3 = 256;
// The candidates' level-1 histogram covers only the 256 top-12-bit bins from lo_bin upwards
// (16 octaves of magnitude); anything above is clamped into its last bin.  If the k-th key
// falls into that last bin the row takes the fallback route.
constexpr int kH1W = 256;
constexpr int kOffSample = 0, kOffH1 = kH1, kOffH2 = 2 * kH1, kOffH3 = 2 * kH1 + kH2, kOffH1F = 2 * kH1 + kH2 + kH3;
constexpr int kOffFine = 3 * kH1 + kH2 + kH3;   // sample, 16 bins x 256 sub-bins around the previous threshold
constexpr int kFineBins = 16;                   // 12-bit bins covered by the fine window (one octave)
constexpr int kHistRow = 4 * kH1 + kH2 + kH3;
constexpr int kSampleSubs = 512;           // subtiles sampled per row
constexpr uint32_t kNone = 0xFFFFFFFFu;
constexpr int kSyncStride = 256;           // bytes of synchronisation memory per row of k_topk_finish: the counter in the first 128-byte line, the published words in the second
constexpr int kStages = 4;                 // arrival counters per row: sample, candidate histogram, fallback histogram, count
enum { kStageSample = 0, kStageHist = 1, kStageFallback = 2, kStageCount = 3 };

struct Sel {
    uint32_t lo_key;    // candidates are the elements with key >= lo_key
    uint32_t lo_bin;    // lo_key >> 19
    uint32_t fallback;  // 1: too few candidates, the row takes the two-look route
    uint32_t b1, k1;    // top-12-bit bin of the k-th key; entries still needed from it
    uint32_t b2, k2;    // next 11 bits; entries still needed from that sub-bin
    uint32_t T, k3;     // threshold key; ties at T to keep (lowest indices first)
};

__device__ __forceinline__ uint32_t key_of(float v) { return __float_as_uint(v) & 0x7FFFFFFFu; }

// number of set bits of m below this lane
__device__ __forceinline__ uint32_t lanes_below(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(m >> 32), __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(m), 0u));
}

}  // namespace

struct ds_topk_scratch {
    uint32_t *hist;       // [rows][kHistRow], zero between calls: every call clears what it used
    uint32_t *prev_T;     // [rows + 1] threshold key of the previous call per worker row, and of the server
    uint32_t *done;       // [rows][kStages] arrival counters of the "last workgroup finishes the row" steps
    Sel *sel;             // [rows]
    u32x2 *slots;         // [rows][n_reg * 2048] candidate (index, value bits), one region per 2048-element tile
    uint32_t *reg_cnt;    // [rows][reg_pad]  candidates per region
    uint32_t *grp_gt;     // [rows][n_groups] candidates with key > T
    uint32_t *grp_eq;     // [rows][n_groups] candidates with key == T
    uint32_t *grp_eqb;    // [rows][n_groups] ties at T in earlier groups
    uint32_t *grp_out;    // [rows][n_groups] first output slot of the group
    uint32_t *sub_start;  // [n_sub + 1][n]   server: first entry of each worker's message per subtile
    int64_t n_sub;        // 256-element subtiles per row (sampling, server ranges)
    int64_t n_reg, reg_pad, n_groups;
    int rows;
    // fused refinement route (k_topk_finish)
    uint32_t *fhist;      // [rows][kFRow], zero between calls
    char *sync;           // [rows][kSyncStride] arrival counters and published picks
    uint32_t *abort_host; // pinned host word, raised by a kernel that gave up waiting
    int64_t capacity;     // workgroups of k_topk_finish the device holds at once; 0: route off
    uint32_t spin_limit;  // polls a workgroup of k_topk_finish spends on one wait before it gives up
};

namespace {

// ---------------------------------------------------------------------------------------
// sources of v, one f32x4 per lane, one 256-element subtile per wavefront
// ---------------------------------------------------------------------------------------
template <bool BF16>
struct WorkerV {   // v = g + delta
    static constexpr int kLdsWords = 1;
    __device__ __forceinline__ void prepare(float *) const {}
    const void *g;
    int64_t gs;
    const float *delta;
    int64_t dstr;
    __device__ __forceinline__ f32x4 load(int row, int64_t e, int64_t d, float *) const
    {
        const void *grow = BF16 ? static_cast<const void *>(static_cast<const uint16_t *>(g) + row * gs)
                                : static_cast<const void *>(static_cast<const float *>(g) + row * gs);
        const float *drow = delta + row * dstr;
        return ld4_grad<BF16>(grow, e, d, BF16 ? aligned8(grow) : aligned16(grow)) + ld4_stream(drow, e, d, aligned16(drow));
    }
};

struct GradV {     // v = g: Algorithm 1 without compensation (fp32 gradients)
    static constexpr int kLdsWords = 1;
    __device__ __forceinline__ void prepare(float *) const {}
    const float *g;
    int64_t gs;
    __device__ __forceinline__ f32x4 load(int row, int64_t e, int64_t d, float *) const
    {
        const float *grow = g + row * gs;
        return ld4_stream(grow, e, d, aligned16(grow));
    }
};

struct BufferV {   // v already stored
    static constexpr int kLdsWords = 1;
    __device__ __forceinline__ void prepare(float *) const {}
    const float *buf;
    int64_t stride;
    __device__ __forceinline__ f32x4 load(int row, int64_t e, int64_t d, float *) const
    {
        const float *brow = buf + row * stride;
        return ld4(brow, e, d, aligned16(brow));
    }
};

// Server: v = delta_s + (1/n) sum_i Q[v_i] for sparse messages, as the chain
// acc = fma(val, 1/n, acc) over workers in ascending order.  The wavefront keeps its subtile
// in a private LDS strip.  Lane i fetches worker i's entry range for the subtile (one load
// instruction for all workers), the entries of all workers are then fetched flattened in
// worker order (one more load instruction per 64 entries) and applied to the strip in
// rounds: in each round, of the pending entries that hit one element the one in the lowest
// lane (= the lowest worker: a message lists an index once) claims it through an LDS minimum
// and is applied.  Most elements are hit once, so a batch takes one or two rounds whatever
// the number of workers.
struct ServerV {
    static constexpr int kLdsWords = 2 * kSub;   // per wavefront: the strip, then one claim tag per element
    const u32x2 *pairs_in;      // [n][k]
    const uint32_t *sub_start;  // [n_sub + 1][n]
    const float *delta_s;
    int64_t k, n_sub;
    int32_t n;
    float inv_n;
    // once per wavefront, before the first load
    __device__ __forceinline__ void prepare(float *strip) const
    {
        uint32_t *tag = reinterpret_cast<uint32_t *>(strip + kSub);
        for (int i = lane_id(); i < kSub; i += 64) tag[i] = kNone;
    }
    __device__ __forceinline__ f32x4 load(int, int64_t e, int64_t d, float *strip) const
    {
        const int lane = lane_id();
        uint32_t *tag = reinterpret_cast<uint32_t *>(strip + kSub);
        const f32x4 a = ld4(delta_s, e, d, aligned16(delta_s));
        strip[lane * 4 + 0] = a.x; strip[lane * 4 + 1] = a.y; strip[lane * 4 + 2] = a.z; strip[lane * 4 + 3] = a.w;
        const int64_t sub = e >> 8;
        const uint32_t base = static_cast<uint32_t>(sub << 8);
        for (int w0 = 0; w0 < n; w0 += 64) {
            const int nw = (n - w0 < 64) ? n - w0 : 64;
            const int nsteps = (nw <= 1) ? 0 : 32 - __builtin_clz(static_cast<uint32_t>(nw - 1));   // ceil(log2 nw)
            uint32_t s0 = 0u, c = 0u;
            if (lane < nw) {
                s0 = sub_start[sub * n + w0 + lane];
                uint32_t s1 = sub_start[(sub + 1) * n + w0 + lane];
                if (s1 > static_cast<uint32_t>(k)) s1 = static_cast<uint32_t>(k);
                c = (s1 > s0) ? s1 - s0 : 0u;
            }
            const uint32_t P = wave_inclusive_scan_u32(c);    // inclusive prefix over workers (c = 0 past them)
            const uint32_t total = __shfl(P, nw - 1, 64);
            for (uint32_t i0 = 0; i0 < total; i0 += 64) {
                const uint32_t i = i0 + lane;
                const bool valid = i < total;
                int lo = 0, hi = nw - 1;                      // first worker w with P_w > i
                for (int step = 0; step < nsteps; ++step) {
                    const int mid = (lo + hi) >> 1;
                    if (__shfl(P, mid, 64) > (valid ? i : 0u)) hi = mid; else lo = mid + 1;
                }
                const uint32_t pw = __shfl(P, lo, 64), cw = __shfl(c, lo, 64), sw = __shfl(s0, lo, 64);
                u32x2 pr = {0u, 0u};
                if (valid) pr = pairs_in[static_cast<int64_t>(w0 + lo) * k + sw + (i - (pw - cw))];
                const uint32_t rel = pr.x - base;
                bool pending = valid && rel < static_cast<uint32_t>(kSub);
                while (__ballot(pending)) {
                    if (pending) atomicMin(&tag[rel], static_cast<uint32_t>(lane));
                    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                    const bool win = pending && tag[rel] == static_cast<uint32_t>(lane);
                    if (win) {
                        strip[rel] = __fmaf_rn(__uint_as_float(pr.y), inv_n, strip[rel]);
                        tag[rel] = kNone;
                    }
                    pending = pending && !win;
                    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        return f32x4{strip[lane * 4 + 0], strip[lane * 4 + 1], strip[lane * 4 + 2], strip[lane * 4 + 3]};
    }
};

// ---------------------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------------------
// "The last workgroup finishes the row": data that workgroups of one kernel hand to the last
// of them travels only through device-scope atomics (adds into histograms, stores and loads
// of counts and picks), which are performed at the device's coherence point, so no cache
// write-back or invalidation is needed -- an agent-scope fence per workgroup costs a full L2
// write-back on this GPU and tripled the step time when tried.
//
// DevShared<T> is the type of every word that workgroups of ONE launch hand to each other
// (histograms, group counts, arrival counters, published picks): it offers device-scope
// operations only, so a plain load or store on that path does not compile.  The memory is
// allocated and cleared as plain words by the host and by other launches (a launch boundary
// makes those visible); `as_shared` is the one place where such a pointer becomes typed.
template <class T>
class DevShared {
    T w_;

public:
    DevShared() = delete;
    __device__ __forceinline__ T load() const { return __hip_atomic_load(&w_, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    __device__ __forceinline__ void store(T v) { __hip_atomic_store(&w_, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    __device__ __forceinline__ T fetch_add(T v) { return __hip_atomic_fetch_add(&w_, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    __device__ __forceinline__ void add(T v) { (void)__hip_atomic_fetch_add(&w_, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    // Plain store of zero, for the one case where the word is dead for the rest of this launch
    // (nothing of it reads or adds to it any more) and the next launch expects it cleared.
    __device__ __forceinline__ void clear_for_next_launch() { w_ = T(0); }
};
using DevWord = DevShared<uint32_t>;
using DevWord64 = DevShared<uint64_t>;
static_assert(sizeof(DevWord) == 4 && sizeof(DevWord64) == 8, "a shared word is just the word");

template <class T>
__host__ __device__ __forceinline__ DevShared<T> *as_shared(T *p) { return reinterpret_cast<DevShared<T> *>(p); }

// True in exactly one workgroup of those that call it with the same counter: the last of
// `expected` to arrive.  Every wavefront first waits until the memory system has acknowledged
// its own outstanding atomics and stores (an explicit wait on the vector memory counter: a
// workgroup-scope release fence emits no such wait on this target, and without it the
// announcement can overtake another wavefront's histogram atomics, which go to other
// channels), the barrier collects the wavefronts, then one device-scope increment announces
// the workgroup.  The counter is left at zero for its next use.  All threads of the
// workgroup must call.
__device__ __forceinline__ bool last_workgroup(DevWord *counter, uint32_t expected, uint32_t *flag_sh)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t prev = counter->fetch_add(1u);
        const bool last = prev + 1u == expected;
        if (last) counter->store(0u);
        *flag_sh = last ? 1u : 0u;
    }
    __syncthreads();
    return *flag_sh != 0u;
}

// First position in idx-sorted pairs[0..k) whose index is >= target.
__device__ __forceinline__ int64_t lower_bound_idx(const u32x2 *__restrict__ pairs, int64_t k, int64_t target)
{
    int64_t lo = 0, hi = k;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (static_cast<int64_t>(pairs[mid].x) < target) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// Server: sub_start[i][s] = first entry of worker i's message with index >= 256 s
// (a binary search per subtile boundary: the cost does not depend on how k relates to d).
__global__ __launch_bounds__(kBlock) void k_topk_sub_starts(const u32x2 *pairs_in, int64_t k, int64_t n_sub,
                                                            uint32_t *sub_start)
{
    const int i = blockIdx.y;
    const int64_t s = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (s > n_sub) return;
    sub_start[s * gridDim.y + i] = static_cast<uint32_t>(lower_bound_idx(pairs_in + i * k, k, s * kSub));
}

// The same table from the entries' side: entry j of a sorted message is the first one of
// every subtile s with sub(j-1) < s <= sub(j) (sub = index >> 8; j = k stands for the end).
// One coalesced pass over the message instead of a search per subtile; the host picks it
// when the message has an entry in most subtiles, so that the loop below stays short.
// Indices are clamped, so a malformed message cannot make it write outside the table.
__global__ __launch_bounds__(kBlock) void k_topk_sub_starts_scan(const u32x2 *pairs_in, int64_t k, int64_t n_sub,
                                                                 uint32_t *sub_start)
{
    const int i = blockIdx.y, n = gridDim.y;
    const int64_t j = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (j > k) return;
    const u32x2 *p = pairs_in + i * k;
    int64_t prev = -1, cur = n_sub;
    if (j > 0) { prev = p[j - 1].x >> 8; if (prev > n_sub) prev = n_sub; }
    if (j < k) { cur = p[j].x >> 8; if (cur > n_sub) cur = n_sub; }
    for (int64_t s = prev + 1; s <= cur; ++s) sub_start[s * n + i] = static_cast<uint32_t>(j);
}

// Largest bin b of hist[0..NB) with  sum_{bins >= b} >= need ;  rem = need - sum_{bins > b}.
// One workgroup; the thread that owns b writes the outputs (untouched if the histogram
// holds fewer than `need` keys).
template <int NB>
__device__ __forceinline__ void pick_bin(const DevWord *__restrict__ hist, uint32_t need, uint32_t *part,
                                         uint32_t *b_out, uint32_t *rem_out, uint32_t *cnt_out = nullptr)
{
    constexpr int PER = (NB >= kBlock) ? NB / kBlock : 1;
    const int t = threadIdx.x;
    const bool active = t * PER < NB;
    uint32_t local[PER];
    uint32_t sum = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        local[j] = active ? hist[t * PER + j].load() : 0u;
        sum += local[j];
    }
    // suffix sums over the threads: shuffles inside a wavefront, wavefront totals through LDS
    const int lane = lane_id();
    // sum over lanes >= mine of my wavefront: the wavefront's total less what lies before me
    const uint32_t pre = wave_inclusive_scan_u32(sum);
    const uint32_t incl = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(pre), 63)) - pre + sum;
    __syncthreads();                                            // part[] may still be read by an earlier pick
    if (lane == 0) part[wave_id()] = incl;
    __syncthreads();
    uint32_t running = incl - sum;                              // keys in bins above my chunk
    for (int w = wave_id() + 1; w < kWaves; ++w) running += part[w];
    if (active) {
#pragma unroll
        for (int j = PER - 1; j >= 0; --j) {
            const uint32_t above = running;
            running += local[j];
            if (running >= need && above < need) {
                *b_out = static_cast<uint32_t>(t * PER + j);
                *rem_out = need - above;
                if (cnt_out) *cnt_out = local[j];
            }
        }
    }
}

// Run by one whole workgroup per row.
// LEVEL 0: sample -> lo_bin.  1: candidates' 12-bit histogram -> b1, k1 or fallback.
// 2: -> b2, k2.  3: -> T, k3.  4: dense 12-bit histogram of a fallback row -> b1, k1.
template <int LEVEL>
__device__ __forceinline__ void pick_level(const DevWord *hrow, Sel *s, uint32_t need0, uint32_t *part, uint32_t *out,
                                           uint32_t *prev_T = nullptr)
{
    if (threadIdx.x == 0) { out[0] = kNone; out[1] = 0u; }
    __syncthreads();
    if (LEVEL == 0) pick_bin<kH1>(hrow + kOffSample, need0, part, &out[0], &out[1]);
    if (LEVEL == 1) pick_bin<kH1W>(hrow + kOffH1, need0, part, &out[0], &out[1]);
    if (LEVEL == 2) pick_bin<kH2>(hrow + kOffH2, s->k1, part, &out[0], &out[1]);
    if (LEVEL == 3) pick_bin<kH3>(hrow + kOffH3, s->k2, part, &out[0], &out[1]);
    if (LEVEL == 4) pick_bin<kH1>(hrow + kOffH1F, need0, part, &out[0], &out[1]);
    __syncthreads();
    if (threadIdx.x == 0) {
        if (LEVEL == 0) {       // out[0] = bin of the sample's rank-`need0` key (kNone: sample too small)
            const uint32_t lo = (out[0] == kNone) ? 0u : (out[0] << 19);
            s->lo_key = lo;
            s->lo_bin = lo >> 19;
        }
        if (LEVEL == 1) {
            // no bin found: fewer than k candidates; last window bin: bins are lumped there
            const bool bad = out[0] == kNone || (out[0] == kH1W - 1 && s->lo_bin + kH1W - 1 < kH1 - 1);
            s->fallback = bad ? 1u : 0u;
            out[2] = bad ? 1u : 0u;     // for the caller: a plain re-read of *s could hit a stale scalar cache line
            if (!bad) { s->b1 = s->lo_bin + out[0]; s->k1 = out[1]; }
        }
        if (LEVEL == 2) { s->b2 = out[0]; s->k2 = out[1]; }
        if (LEVEL == 3) {
            s->T = (s->b1 << 19) | (s->b2 << 8) | out[0];
            s->k3 = out[1];
            *prev_T = s->T;        // centre of the next call's fine sampling window
        }
        if (LEVEL == 4) { s->b1 = out[0]; s->k1 = out[1]; }
    }
}

__device__ __forceinline__ int64_t sample_subtile(int64_t j, int64_t ns, int64_t n_sub)
{
    // evenly spread, with a small hashed jitter inside each stride
    const int64_t lo = (j * n_sub) / ns, hi = ((j + 1) * n_sub) / ns;
    const int64_t span = hi - lo;
    const uint32_t h = static_cast<uint32_t>(j) * 2654435761u;
    return lo + ((span > 1) ? static_cast<int64_t>((h >> 8) % static_cast<uint32_t>(span)) : 0);
}

// 12-bit histogram of v over the sampled subtiles.
template <class Src>
__global__ __launch_bounds__(kBlock) void k_topk_sample(Src src, int64_t d, int64_t n_sub, int64_t ns, DevWord *hist,
                                                        Sel *sel, DevWord *done, uint32_t rank, const uint32_t *prev_T,
                                                        DevWord *sync_words)
{
    // the single-launch refinement of this call finds its row's synchronisation words at zero
    // (its own previous launch is complete by stream order and did not clear them itself)
    if (blockIdx.x == 0 && threadIdx.x < kSyncStride / 4)
        sync_words[blockIdx.y * (kSyncStride / 4) + threadIdx.x].store(0u);
    __shared__ uint32_t h[kH1];        // 12-bit bins
    __shared__ uint32_t hf[kH1];       // fine window: kFineBins 12-bit bins x 256 sub-bins (key bits 18..11)
    __shared__ uint32_t part[kBlock], out[2], flag;
    __shared__ float strips[kWaves][Src::kLdsWords];
    const int row = blockIdx.y;
    src.prepare(strips[wave_id()]);
    for (int i = threadIdx.x; i < kH1; i += kBlock) { h[i] = 0u; hf[i] = 0u; }
    __syncthreads();
    const uint32_t tb = prev_T[row] >> 19;
    const uint32_t bw = (tb > kFineBins / 2) ? tb - kFineBins / 2 : 0u;   // first 12-bit bin of the window
    const int64_t j = static_cast<int64_t>(blockIdx.x) * kWaves + wave_id();
    if (j < ns) {
        const int64_t e = sample_subtile(j, ns, n_sub) * kSub + lane_id() * 4;
        const f32x4 v = src.load(row, e, d, strips[wave_id()]);
        const uint32_t key[4] = {key_of(v.x), key_of(v.y), key_of(v.z), key_of(v.w)};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (e + c >= d) continue;
            const uint32_t bin = key[c] >> 19;
            atomicAdd(&h[bin], 1u);
            if (bin - bw < static_cast<uint32_t>(kFineBins)) atomicAdd(&hf[((bin - bw) << 8) | ((key[c] >> 11) & 255u)], 1u);
        }
    }
    __syncthreads();
    DevWord *hrow = hist + static_cast<int64_t>(row) * kHistRow;
    for (int i = threadIdx.x; i < kH1; i += kBlock) {
        if (h[i]) hrow[kOffSample + i].add(h[i]);
        if (hf[i]) hrow[kOffFine + i].add(hf[i]);
    }
    if (last_workgroup(done + row * kStages + kStageSample, gridDim.x, &flag)) {
        Sel *s = sel + row;
        pick_level<0>(hrow, s, rank, part, out);          // 12-bit bin of the rank-th sample key
        __syncthreads();
        const uint32_t b = out[0], rem = out[1];
        __syncthreads();
        if (b != kNone && b - bw < static_cast<uint32_t>(kFineBins)) {
            // refine inside the bin: the sub-bin that holds the key `rem` places from the bin's top
            if (threadIdx.x == 0) { out[0] = kNone; out[1] = 0u; }
            __syncthreads();
            pick_bin<256>(hrow + kOffFine + ((b - bw) << 8), rem, part, &out[0], &out[1]);
            __syncthreads();
            if (threadIdx.x == 0 && out[0] != kNone) s->lo_key = (b << 19) | (out[0] << 11);
        }
    }
}

// ---------------------------------------------------------------------------------------
// the dense pass
// ---------------------------------------------------------------------------------------
// FALLBACK = false: v from src, stored into buf, candidates with key >= lo_key.
// FALLBACK = true : rows flagged for the two-look route only; v is read back from buf,
//                   candidates with bin >= b1.
// WR = false: nothing is stored into buf (the mode without compensation: there is no error
//             buffer, and the second look of the fallback reads the gradient itself).
template <bool WR>
__device__ __forceinline__ void pass1_tile_v(f32x4 v, float *buf, int64_t stride, int64_t d, uint32_t lo_key, u32x2 *slots,
                                             uint32_t *reg_cnt, int64_t n_reg, int64_t reg_pad, int row, int64_t tile,
                                             uint32_t *wtot)
{
    const int64_t e = tile * kTile + threadIdx.x * 4;
    const uint32_t bits[4] = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
    bool f[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) f[c] = (e + c < d) && (bits[c] & 0x7FFFFFFFu) >= lo_key;
    // The error buffer gets v where the element is no candidate and 0 where it is: most
    // candidates end up kept (delta = 0 there), so the emit pass only has to put v back at
    // the few candidates that are not kept instead of zeroing every kept position.
    if (WR && e < d) {
        float *brow = buf + row * stride;
        st4_stream(brow, e, d, aligned16(brow), f32x4{f[0] ? 0.f : v.x, f[1] ? 0.f : v.y, f[2] ? 0.f : v.z, f[3] ? 0.f : v.w});
    }
    // index-ordered compaction over the workgroup: ballots inside a wavefront, wavefront
    // totals through LDS
    const uint64_t m0 = __ballot(f[0]), m1 = __ballot(f[1]), m2 = __ballot(f[2]), m3 = __ballot(f[3]);
    const uint32_t before = lanes_below(m0) + lanes_below(m1) + lanes_below(m2) + lanes_below(m3);
    __syncthreads();                                  // wtot may still be read (persistent launch)
    if (lane_id() == 0) wtot[wave_id()] = __popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3);
    __syncthreads();
    uint32_t wave_off = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        if (w < wave_id()) wave_off += wtot[w];
        total += wtot[w];
    }
    u32x2 *out = slots + (static_cast<int64_t>(row) * n_reg + tile) * kReg + wave_off + before;
    uint32_t r = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c)
        if (f[c]) out[r++] = u32x2{static_cast<uint32_t>(e + c), bits[c]};
    if (threadIdx.x == 0) reg_cnt[row * reg_pad + tile] = total;
}

template <class Src, bool FALLBACK, bool WR = true>
__device__ __forceinline__ void pass1_tile(const Src &src, float *buf, int64_t stride, int64_t d, int64_t n_sub,
                                           uint32_t lo_key, u32x2 *slots, uint32_t *reg_cnt, int64_t n_reg,
                                           int64_t reg_pad, int row, int64_t tile, float *strip, uint32_t *wtot)
{
    const int64_t e = tile * kTile + threadIdx.x * 4;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if ((e >> 8) < n_sub) v = src.load(row, e, d, strip);        // whole wavefronts
    pass1_tile_v<WR>(v, buf, stride, d, lo_key, slots, reg_cnt, n_reg, reg_pad, row, tile, wtot);
}

template <class Src, bool FALLBACK, bool WR = true>
__global__ __launch_bounds__(kBlock) void k_topk_pass1(Src src, float *buf, int64_t stride, int64_t d, int64_t n_sub,
                                                       const Sel *sel, u32x2 *slots, uint32_t *reg_cnt, int64_t n_reg,
                                                       int64_t reg_pad)
{
    __shared__ float strips[kWaves][Src::kLdsWords];
    __shared__ uint32_t wtot[kWaves];
    const int row = blockIdx.y;
    if (FALLBACK && !sel[row].fallback) return;
    src.prepare(strips[wave_id()]);
    const uint32_t lo_key = FALLBACK ? (sel[row].b1 << 19) : sel[row].lo_key;
    if constexpr (FALLBACK) {
        // a small grid that exits at once for rows that do not need it and strides over the tiles otherwise
        for (int64_t tile = blockIdx.x; tile < n_reg; tile += gridDim.x)
            pass1_tile<Src, FALLBACK, WR>(src, buf, stride, d, n_sub, lo_key, slots, reg_cnt, n_reg, reg_pad, row, tile,
                                          strips[wave_id()], wtot);
    } else {
        // the regular launch: one workgroup per tile (two tiles per workgroup with both loads
        // issued first measured 3.5 % slower on the 8 x 25.6 M workload)
        pass1_tile<Src, FALLBACK, WR>(src, buf, stride, d, n_sub, lo_key, slots, reg_cnt, n_reg, reg_pad, row, blockIdx.x,
                                      strips[wave_id()], wtot);
    }
}

// The server's dense pass (row 0 only): the same work as k_topk_pass1<ServerV, false> with
// FOUR subtiles (1024 elements) per wavefront and four candidate regions per workgroup.  A
// subtile holds only about 8 n k / d entries, so with one subtile per wavefront most lanes idle
// through the entry handling; four subtiles fill the 64-entry batches, share one range
// look-up and prefix, and keep four independent 128-bit loads in flight per lane.  The claim
// tags are hashed (element & 255): two pending entries that share a tag but not an element
// merely take turns.
constexpr int kSpan = 4 * kSub;              // elements per wavefront
constexpr int kTags = kSub;                  // claim tags per wavefront (128 would let a fourth workgroup share a compute unit; measured: no gain, the pass is bound by instruction issue)

// SID: the server does not compress (its message is the average itself): the wavefront's span
// of the average, built from +0, is written to `buf` (if not null) and / or applied to the
// model (u), and the kernel ends there.
template <bool SID>
__global__ __launch_bounds__(kBlock) void k_topk_pass1_server(ServerV src, float *buf, int64_t d, const Sel *sel,
                                                              u32x2 *slots, uint32_t *reg_cnt, int64_t n_reg,
                                                              ds_update_args u)
{
    __shared__ float strips[kWaves][kSpan];
    __shared__ uint32_t tags[kWaves][kTags];
    __shared__ uint32_t wtot[kWaves];
    const int lane = lane_id(), wv = wave_id();
    float *strip = strips[wv];
    uint32_t *tag = tags[wv];
    for (int i = lane; i < kTags; i += 64) tag[i] = kNone;
    const int64_t span_base = (static_cast<int64_t>(blockIdx.x) * kWaves + wv) * kSpan;
    const uint32_t lo_key = SID ? 0u : sel[0].lo_key;
    const bool vec = aligned16(buf);
    const bool live = span_base < d;                       // uniform over the wavefront
    const int64_t sub0 = span_base >> 8;
    const int64_t sub1 = (sub0 + 4 < src.n_sub) ? sub0 + 4 : src.n_sub;
    const uint32_t base = static_cast<uint32_t>(span_base);
    const int n = src.n;

    // The loads are issued in the order of the dependent chain, longest first: the workers'
    // entry ranges (which the entries' addresses wait for), then the span of the server's
    // error, then the first batch of entries; only then is anything used.  (With the error
    // copied into the strip first, the range look-up waited for it: 4.5 us of latency in a row
    // per wavefront instead of 2.5.)
    struct Ranges {
        uint32_t s0, c, P, total;
        int nw, nsteps;
    };
    auto load_bounds = [&](int w0, uint32_t &s0, uint32_t &s1) {
        const int nw = (n - w0 < 64) ? n - w0 : 64;
        s0 = s1 = 0u;
        if (live && lane < nw) {
            s0 = src.sub_start[sub0 * n + w0 + lane];
            s1 = src.sub_start[sub1 * n + w0 + lane];
        }
    };
    auto make_ranges = [&](int w0, uint32_t s0, uint32_t s1) -> Ranges {
        Ranges r;
        r.nw = (n - w0 < 64) ? n - w0 : 64;
        r.nsteps = (r.nw <= 1) ? 0 : 32 - __builtin_clz(static_cast<uint32_t>(r.nw - 1));
        if (s1 > static_cast<uint32_t>(src.k)) s1 = static_cast<uint32_t>(src.k);
        r.s0 = s0;
        r.c = (lane < r.nw && s1 > s0) ? s1 - s0 : 0u;
        const uint32_t P = wave_inclusive_scan_u32(r.c);   // inclusive prefix over workers (c = 0 past them)
        r.P = P;
        r.total = __shfl(P, r.nw - 1, 64);
        return r;
    };
    // entry number i0 + lane of the workers w0 .. w0 + nw - 1, flattened in worker order
    auto fetch = [&](const Ranges &r, int w0, uint32_t i0, bool &valid) -> u32x2 {
        const uint32_t i = i0 + lane;
        valid = i < r.total;
        int lo = 0, hi = r.nw - 1;                         // first worker w with P_w > i
        for (int step = 0; step < r.nsteps; ++step) {
            const int mid = (lo + hi) >> 1;
            if (__shfl(r.P, mid, 64) > (valid ? i : 0u)) hi = mid; else lo = mid + 1;
        }
        const uint32_t pw = __shfl(r.P, lo, 64), cw = __shfl(r.c, lo, 64), sw = __shfl(r.s0, lo, 64);
        u32x2 pr = {0u, 0u};
        if (valid) pr = src.pairs_in[static_cast<int64_t>(w0 + lo) * src.k + sw + (i - (pw - cw))];
        return pr;
    };
    auto apply = [&](u32x2 pr, bool valid) {
        const uint32_t rel = pr.x - base;
        bool pending = valid && rel < static_cast<uint32_t>(kSpan);
        while (__ballot(pending)) {
            if (pending) atomicMin(&tag[rel & (kTags - 1)], static_cast<uint32_t>(lane));
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            const bool win = pending && tag[rel & (kTags - 1)] == static_cast<uint32_t>(lane);
            if (win) {
                strip[rel] = __fmaf_rn(__uint_as_float(pr.y), src.inv_n, strip[rel]);
                tag[rel & (kTags - 1)] = kNone;
            }
            pending = pending && !win;
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        }
    };

    uint32_t b0, b1;
    load_bounds(0, b0, b1);
    f32x4 v[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
        v[c] = SID ? f32x4{0.f, 0.f, 0.f, 0.f}
                   : ld4_stream(src.delta_s, span_base + c * kSub + lane * 4, d, aligned16(src.delta_s));
    Ranges r = make_ranges(0, b0, b1);
    bool valid0 = false;
    u32x2 pr0 = {0u, 0u};
    if (live && r.total > 0) pr0 = fetch(r, 0, 0u, valid0);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        float *p = strip + c * kSub + lane * 4;
        p[0] = v[c].x; p[1] = v[c].y; p[2] = v[c].z; p[3] = v[c].w;
    }
    if (live) {
        for (int w0 = 0; w0 < n; w0 += 64) {
            if (w0 > 0) {
                load_bounds(w0, b0, b1);
                r = make_ranges(w0, b0, b1);
            }
            for (uint32_t i0 = 0; i0 < r.total; i0 += 64) {
                bool valid = valid0;
                u32x2 pr = pr0;
                if (w0 > 0 || i0 > 0) pr = fetch(r, w0, i0, valid);
                apply(pr, valid);
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float *p = strip + c * kSub + lane * 4;
            v[c] = f32x4{p[0], p[1], p[2], p[3]};
        }
    }
    if constexpr (SID) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t e = span_base + c * kSub + lane * 4;
            if (e < d) put_average4(v[c], e, d, buf, u.x, u.m, u.gamma, u.beta);
        }
        return;
    }
    // classify, store v with 0 at the candidates, count
    uint32_t bits[4][4];
    bool f[4][4];
    uint32_t before[4], cnt_c[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int64_t e = span_base + c * kSub + lane * 4;
        bits[c][0] = __float_as_uint(v[c].x); bits[c][1] = __float_as_uint(v[c].y);
        bits[c][2] = __float_as_uint(v[c].z); bits[c][3] = __float_as_uint(v[c].w);
#pragma unroll
        for (int j = 0; j < 4; ++j) f[c][j] = (e + j < d) && (bits[c][j] & 0x7FFFFFFFu) >= lo_key;
        if (e < d)
            st4_stream(buf, e, d, vec, f32x4{f[c][0] ? 0.f : v[c].x, f[c][1] ? 0.f : v[c].y, f[c][2] ? 0.f : v[c].z,
                                     f[c][3] ? 0.f : v[c].w});
        const uint64_t m0 = __ballot(f[c][0]), m1 = __ballot(f[c][1]), m2 = __ballot(f[c][2]), m3 = __ballot(f[c][3]);
        before[c] = lanes_below(m0) + lanes_below(m1) + lanes_below(m2) + lanes_below(m3);
        cnt_c[c] = __popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3);
    }
    const uint32_t wave_total = cnt_c[0] + cnt_c[1] + cnt_c[2] + cnt_c[3];
    if (lane == 0) wtot[wv] = wave_total;
    __syncthreads();
    // a region is the two wavefronts 2r, 2r+1: the odd one writes behind the even one
    const int64_t region = static_cast<int64_t>(blockIdx.x) * 4 + (wv >> 1);
    uint32_t off = (wv & 1) ? wtot[wv - 1] : 0u;
    if (region < n_reg) {
        u32x2 *out = slots + region * kReg;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t e = span_base + c * kSub + lane * 4;
            uint32_t r = off + before[c];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (f[c][j]) out[r++] = u32x2{static_cast<uint32_t>(e + j), bits[c][j]};
            off += cnt_c[c];
        }
        if ((wv & 1) && lane == 0) reg_cnt[region] = wtot[wv - 1] + wtot[wv];
    }
}

// Fallback rows: dense 12-bit histogram of the stored v.  Persistent workgroups.
__global__ __launch_bounds__(kBlock) void k_topk_fallback_hist(const float *buf, int64_t stride, int64_t d,
                                                               int64_t n_tiles, Sel *sel, DevWord *hist,
                                                               DevWord *done, uint32_t k)
{
    __shared__ uint32_t h[kH1];
    __shared__ uint32_t part[kBlock], out[3], flag;
    const int row = blockIdx.y;
    if (!sel[row].fallback) return;
    for (int i = threadIdx.x; i < kH1; i += kBlock) h[i] = 0u;
    __syncthreads();
    const float *brow = buf + row * stride;
    const bool vec = aligned16(brow);
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t e = tile * kTile + threadIdx.x * 4;
        if (e >= d) continue;
        const f32x4 v = ld4(brow, e, d, vec);
        if (e + 0 < d) atomicAdd(&h[key_of(v.x) >> 19], 1u);
        if (e + 1 < d) atomicAdd(&h[key_of(v.y) >> 19], 1u);
        if (e + 2 < d) atomicAdd(&h[key_of(v.z) >> 19], 1u);
        if (e + 3 < d) atomicAdd(&h[key_of(v.w) >> 19], 1u);
    }
    __syncthreads();
    DevWord *hrow = hist + static_cast<int64_t>(row) * kHistRow;
    for (int i = threadIdx.x; i < kH1; i += kBlock)
        if (h[i]) hrow[kOffH1F + i].add(h[i]);
    if (last_workgroup(done + row * kStages + kStageFallback, gridDim.x, &flag))
        pick_level<4>(hrow, sel + row, k, part, out);
}

// ---------------------------------------------------------------------------------------
// candidate passes: one wavefront walks the candidates of one group (64 subtiles) in order
// ---------------------------------------------------------------------------------------
struct GroupWalk {
    uint32_t c;      // lane r < kGroupRegs: candidate count of region r of the group
    uint32_t P;      // inclusive prefix over lanes
    uint32_t total;
};

__device__ __forceinline__ GroupWalk group_begin(const uint32_t *__restrict__ cnt_row, int64_t g, int64_t n_reg)
{
    GroupWalk w;
    const int lane = lane_id();
    const int64_t reg = g * kGroupRegs + lane;
    w.c = (lane < kGroupRegs && reg < n_reg) ? cnt_row[reg] : 0u;
    const uint32_t p = wave_inclusive_scan_u32(w.c);            // c = 0 past the group's regions
    w.P = p;
    w.total = __shfl(p, kGroupRegs - 1, 64);
    return w;
}

// Candidate number i (in index order) of the group; all lanes must call.
__device__ __forceinline__ u32x2 group_fetch(const GroupWalk &w, const u32x2 *__restrict__ slots_row, int64_t g,
                                             uint32_t i, bool valid)
{
    int lo = 0, hi = kGroupRegs - 1;              // first region r with P_r > i
#pragma unroll
    for (int step = 0; step < 4; ++step) {
        const int mid = (lo + hi) >> 1;
        const uint32_t pm = __shfl(w.P, mid, 64);
        if (pm > i) hi = mid; else lo = mid + 1;
    }
    const uint32_t ps = __shfl(w.P, lo, 64), cs = __shfl(w.c, lo, 64);
    u32x2 pr = {0u, 0u};
    if (valid) pr = slots_row[(g * kGroupRegs + lo) * kReg + (i - (ps - cs))];
    return pr;
}

// The candidate passes fetch up to kPrefetch batches of 64 candidates before using any of
// them, so that a wavefront has several independent loads in flight instead of a chain of
// dependent ones (a group of 8 regions holds about 250-320 candidates at k = 1 %).
constexpr int kPrefetch = 8;

struct Batch {
    u32x2 pr[kPrefetch];
};

__device__ __forceinline__ Batch group_fetch_batches(const GroupWalk &w, const u32x2 *__restrict__ slots_row,
                                                     int64_t g, uint32_t i0)
{
    Batch b;
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) {
        b.pr[j] = u32x2{0u, 0u};
        if (i0 + j * 64 < w.total) {                       // uniform over the wavefront
            const uint32_t i = i0 + j * 64 + lane_id();
            b.pr[j] = group_fetch(w, slots_row, g, (i < w.total) ? i : 0u, i < w.total);
        }
    }
    return b;
}

// Fallback rows: put v back at every candidate position (the dense pass wrote 0 there), so
// that the two-look route sees the whole of v in the buffer.  Run by one workgroup (the one
// that detects the fallback); slow, but the route is rare.
__device__ __forceinline__ void restore_row(const u32x2 *slots, const uint32_t *reg_cnt, int64_t n_reg, int64_t reg_pad,
                                            int row, float *buf, int64_t stride)
{
    float *brow = buf + row * stride;
    for (int64_t reg = 0; reg < n_reg; ++reg) {
        const uint32_t cnt = reg_cnt[row * reg_pad + reg];
        const u32x2 *src = slots + (static_cast<int64_t>(row) * n_reg + reg) * kReg;
        for (uint32_t i = threadIdx.x; i < cnt; i += kBlock) brow[src[i].x] = __uint_as_float(src[i].y);
    }
}

// LEVEL 1: 12-bit histogram of all candidates.  2: next 11 bits of those in bin b1.
// 3: low 8 bits of those with prefix (b1, b2).  One group per wavefront.
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void k_topk_cand_hist(const u32x2 *slots, const uint32_t *reg_cnt, int64_t n_reg,
                                                           int64_t reg_pad, int64_t n_groups, Sel *sel,
                                                           DevWord *hist, DevWord *done, uint32_t k, uint32_t *prev_T,
                                                           float *buf, int64_t stride, bool wr)
{
    constexpr int NB = (LEVEL == 1) ? kH1W : (LEVEL == 2) ? kH2 : kH3;
    constexpr int OFF = (LEVEL == 1) ? kOffH1 : (LEVEL == 2) ? kOffH2 : kOffH3;
    __shared__ uint32_t h[NB];
    __shared__ uint32_t part[kBlock], out[3], flag;
    const int row = blockIdx.y;
    const Sel s = sel[row];
    for (int i = threadIdx.x; i < NB; i += kBlock) h[i] = 0u;
    __syncthreads();
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kWaves + wave_id();
    if (g < n_groups) {
        const GroupWalk w = group_begin(reg_cnt + row * reg_pad, g, n_reg);
        const u32x2 *srow = slots + static_cast<int64_t>(row) * n_reg * kReg;
        const uint32_t prefix = (s.b1 << 11) | s.b2;
        for (uint32_t i0 = 0; i0 < w.total; i0 += 64 * kPrefetch) {
            const Batch bt = group_fetch_batches(w, srow, g, i0);
#pragma unroll
            for (int j = 0; j < kPrefetch; ++j) {
                if (i0 + j * 64 + lane_id() >= w.total) continue;
                const uint32_t key = bt.pr[j].y & 0x7FFFFFFFu;
                if (LEVEL == 1) {
                    const uint32_t rel = (key >> 19) - s.lo_bin;      // candidates have bin >= lo_bin
                    atomicAdd(&h[rel < kH1W ? rel : kH1W - 1], 1u);
                }
                if (LEVEL == 2 && (key >> 19) == s.b1) atomicAdd(&h[(key >> 8) & (kH2 - 1)], 1u);
                if (LEVEL == 3 && (key >> 8) == prefix) atomicAdd(&h[key & 255u], 1u);
            }
        }
    }
    __syncthreads();
    DevWord *hrow = hist + static_cast<int64_t>(row) * kHistRow;
    for (int i = threadIdx.x; i < NB; i += kBlock)
        if (h[i]) hrow[OFF + i].add(h[i]);
    if (last_workgroup(done + row * kStages + kStageHist, gridDim.x, &flag)) {
        pick_level<LEVEL>(hrow, sel + row, k, part, out, prev_T + row);
        if (LEVEL == 1) {
            __syncthreads();
            if (out[2] && wr) restore_row(slots, reg_cnt, n_reg, reg_pad, row, buf, stride);
        }
    }
}

// Exclusive scan over the workgroup of one value per thread; tmp holds kWaves values.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t *tmp)
{
    const int lane = lane_id();
    const uint32_t p = wave_inclusive_scan_u32(x);
    __syncthreads();
    if (lane == 63) tmp[wave_id()] = p;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave_id(); ++w) before += tmp[w];
    return before + p - x;
}

// Per row, in group order: ties seen before each group, and each group's first output slot.
// Run by one whole workgroup.
__device__ __forceinline__ void scan_row(int row, const Sel *sel, int64_t n_groups, const DevWord *grp_gt,
                                         const DevWord *grp_eq, uint32_t *grp_eqb, uint32_t *grp_out, uint32_t *tmp)
{
    const uint32_t k3 = sel[row].k3;
    const int64_t per = (n_groups + kBlock - 1) / kBlock;
    const int64_t t0 = threadIdx.x * per, t1 = (t0 + per < n_groups) ? t0 + per : n_groups;
    const DevWord *gt = grp_gt + row * n_groups, *eq = grp_eq + row * n_groups;
    uint32_t *eqb = grp_eqb + row * n_groups, *out = grp_out + row * n_groups;
    uint32_t s = 0;
    for (int64_t t = t0; t < t1; ++t) s += eq[t].load();
    uint32_t run = block_exclusive_scan(s, tmp);
    uint32_t sel_sum = 0;
    for (int64_t t = t0; t < t1; ++t) {
        const uint32_t e_t = eq[t].load(), g_t = gt[t].load();
        eqb[t] = run;
        const uint32_t left = (k3 > run) ? k3 - run : 0u;
        sel_sum += g_t + ((e_t < left) ? e_t : left);
        run += e_t;
    }
    uint32_t o = block_exclusive_scan(sel_sum, tmp);
    for (int64_t t = t0; t < t1; ++t) {
        const uint32_t e_t = eq[t].load(), g_t = gt[t].load();
        out[t] = o;
        const uint32_t left = (k3 > eqb[t]) ? k3 - eqb[t] : 0u;
        o += g_t + ((e_t < left) ? e_t : left);
    }
}

// Per group: candidates above T, candidates tying with T; the last workgroup of the row
// then scans the groups.  Every pick of this call is done by now, so the kernel also clears
// the call's histograms (`zero`, `zero_words`) for the next call, which replaces a separate
// clearing launch and leaves no host-side state behind (calls can be captured and replayed).
__global__ __launch_bounds__(kBlock) void k_topk_count(const u32x2 *slots, const uint32_t *reg_cnt, int64_t n_reg,
                                                       int64_t reg_pad, int64_t n_groups, const Sel *sel,
                                                       DevWord *grp_gt, DevWord *grp_eq, uint32_t *grp_eqb,
                                                       uint32_t *grp_out, DevWord *done, uint32_t *zero,
                                                       int64_t zero_words)
{
    __shared__ uint32_t tmp[kWaves], flag;
    const int row = blockIdx.y;
    const int64_t wg = static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x;
    for (int64_t i = wg * kBlock + threadIdx.x; i < zero_words; i += static_cast<int64_t>(gridDim.x) * gridDim.y * kBlock)
        zero[i] = 0u;
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kWaves + wave_id();
    if (g < n_groups) {
        const uint32_t T = sel[row].T;
        const GroupWalk w = group_begin(reg_cnt + row * reg_pad, g, n_reg);
        const u32x2 *srow = slots + static_cast<int64_t>(row) * n_reg * kReg;
        uint32_t gt = 0, eq = 0;
        for (uint32_t i0 = 0; i0 < w.total; i0 += 64 * kPrefetch) {
            const Batch bt = group_fetch_batches(w, srow, g, i0);
#pragma unroll
            for (int j = 0; j < kPrefetch; ++j) {
                const bool valid = i0 + j * 64 + lane_id() < w.total;
                const uint32_t key = bt.pr[j].y & 0x7FFFFFFFu;
                gt += valid && key > T;
                eq += valid && key == T;
            }
        }
        gt = wave_sum_u32(gt);
        eq = wave_sum_u32(eq);
        if (lane_id() == 0) {
            grp_gt[row * n_groups + g].store(gt);
            grp_eq[row * n_groups + g].store(eq);
        }
    }
    if (last_workgroup(done + row * kStages + kStageCount, gridDim.x, &flag))
        scan_row(row, sel, n_groups, grp_gt, grp_eq, grp_eqb, grp_out, tmp);
}

// One group: write the kept entries in index order; the dense pass left 0 at every
// candidate position of the error buffer, so the candidates that are not kept get v back
// (delta = v - Q[v] is 0 at kept positions and v elsewhere).  eq_seen = ties at T in earlier
// groups, out = first output slot of the group.  x != nullptr: the model update of Algorithm 1
// for this message, x <- fma(-gamma, val, x) at the kept indices, in the same pass.
// Called by whole wavefronts.
// One batch of up to 64 candidates in index order (lane = position), see emit_group: the kept
// ones go to their output slots, the others get v back in the error buffer.  Returns whether
// this lane's candidate is kept.
__device__ __forceinline__ bool emit_batch(u32x2 pr, bool valid, uint32_t T, uint32_t k3, uint32_t &eq_seen, uint32_t &out,
                                           u32x2 *prow, float *brow, int64_t k)
{
    const uint32_t key = pr.y & 0x7FFFFFFFu;
    const bool is_eq = valid && key == T;
    const uint64_t eq_mask = __ballot(is_eq);
    const bool keep = valid && (key > T || (is_eq && eq_seen + lanes_below(eq_mask) < k3));
    const uint64_t keep_mask = __ballot(keep);
    if (keep) {
        const uint32_t slot = out + lanes_below(keep_mask);
        if (slot < k) prow[slot] = pr;
    } else if (valid && brow) {
        __builtin_nontemporal_store(__uint_as_float(pr.y), brow + pr.x);   // not kept: delta = v (no buffer: no compensation)
    }
    out += __popcll(keep_mask);
    eq_seen += __popcll(eq_mask);
    return keep;
}

__device__ __forceinline__ void emit_group(const GroupWalk &w, const u32x2 *__restrict__ srow, int64_t g, uint32_t T,
                                           uint32_t k3, uint32_t eq_seen, uint32_t out, u32x2 *prow, float *brow, int64_t k,
                                           float *x = nullptr, float gamma = 0.f)
{
    for (uint32_t i0 = 0; i0 < w.total; i0 += 64 * kPrefetch) {
        const Batch bt = group_fetch_batches(w, srow, g, i0);
        bool kept[kPrefetch];
#pragma unroll
        for (int j = 0; j < kPrefetch; ++j) {
            kept[j] = false;
            if (i0 + j * 64 >= w.total) continue;              // uniform over the wavefront
            kept[j] = emit_batch(bt.pr[j], i0 + j * 64 + lane_id() < w.total, T, k3, eq_seen, out, prow, brow, k);
        }
        if (x) {
            float xv[kPrefetch];
#pragma unroll
            for (int j = 0; j < kPrefetch; ++j) xv[j] = kept[j] ? x[bt.pr[j].x] : 0.f;
#pragma unroll
            for (int j = 0; j < kPrefetch; ++j)
                if (kept[j]) x[bt.pr[j].x] = __fmaf_rn(-gamma, __uint_as_float(bt.pr[j].y), xv[j]);
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_topk_emit(const u32x2 *slots, const uint32_t *reg_cnt, int64_t n_reg,
                                                      int64_t reg_pad, int64_t n_groups, const Sel *sel,
                                                      const uint32_t *grp_eqb, const uint32_t *grp_out, int64_t k,
                                                      u32x2 *pairs, float *buf, int64_t stride, float *x, float gamma,
                                                      bool wr)
{
    const int row = blockIdx.y;
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kWaves + wave_id();
    if (g >= n_groups) return;
    const Sel s = sel[row];
    const GroupWalk w = group_begin(reg_cnt + row * reg_pad, g, n_reg);
    emit_group(w, slots + static_cast<int64_t>(row) * n_reg * kReg, g, s.T, s.k3, grp_eqb[row * n_groups + g],
               grp_out[row * n_groups + g], pairs + static_cast<int64_t>(row) * k, wr ? buf + row * stride : nullptr, k, x, gamma);
}

// ---------------------------------------------------------------------------------------
// fused refinement: everything after the dense pass in one launch
// ---------------------------------------------------------------------------------------
// The candidate phases each touch a few MB that sit in the L2 / memory-side cache, so as
// separate launches they cost mostly dispatch and ramp time.  k_topk_finish runs them in one
// launch whose workgroups are all resident at once (the host sizes the grid from the
// occupancy query) and which synchronise per row:
//   arrive        every wavefront waits for its outstanding atomics, then one device-scope
//                 increment of the row's counter per workgroup;
//   publish       the workgroup whose increment completes the round reads the row's
//                 histogram, picks the bin and publishes (bin, remaining) as one 64-bit
//                 atomic store (a plain barrier publishes an empty word); the others poll
//                 that word, which lies in another cache line than the counter so that the
//                 polls do not queue up in front of the remaining arrivals.  Rows are 256
//                 bytes apart for the same reason.
// A workgroup waits only for workgroups of its own row.  Workgroups are handed to the compute
// units in the order of their linear index (row-major here), so when other kernels share the
// device the rows become resident one after the other: at most the one row at the front of the
// dispatch is incomplete and waiting, the others run, finish and make room.  That order is
// what the hardware does, not a documented guarantee, so every poll loop is bounded as well:
// if a round does not complete within the spin limit, the workgroup raises the context's abort
// word (host memory) and the kernel drains.  ds_status reports it; the next step call resets
// the context's scratch state, switches it to the chain of launches and reports it once.
//
// Radix levels here are relative to lo_key: level A = 2048 bins of 2048 keys from lo_key
// upwards (the last bin also takes everything beyond), level B = the 11 low bits inside bin
// A.  The sample's lower bound is known to 20 key bits and the k-th key lies a few per cent
// above it (200 to 800 such bins on the 25.6 M-element top-1 % workload; a window of a quarter
// of this width missed one server call in ten), so two levels resolve all 31 bits.  A row whose
// k-th key is not below the last bin (or that has fewer than k candidates) takes the exact
// two-look route inside the same launch: put v back, dense 12-bit histogram, pick b1, compact
// again with lo_key = b1 << 19 (the k-th key is then less than 2^19 above lo_key), level A
// again.  Both histograms take 8 KiB of LDS, which leaves room for the wavefronts' candidate
// caches at four workgroups per compute unit.
constexpr int kHA = 2048, kHB = 2048, kShiftA = 11;
constexpr int kFOffA = 0, kFOffA2 = kHA, kFOffB = 2 * kHA, kFOffD = 2 * kHA + kHB;
constexpr int kFRow = 2 * kHA + kHB + kH1;     // words per row of the fused route's histograms
enum { kResA = 0, kResD = 1, kResA2 = 2, kResB = 3, kResCompact = 4, kResCount = 5, kResSlots = 6 };
constexpr uint32_t kSpinLimit = 1u << 22;     // polls per wait before a workgroup gives up (seconds)
constexpr uint64_t kResValid = 1ull << 63;

struct RowSync {
    DevWord *bar;          // arrival counter of the row, 0 between launches
    DevWord64 *res;        // kResSlots published picks of the row, 0 between launches
    uint32_t *abort_flag;  // host memory
    uint32_t *sh;          // 3 LDS words
    uint32_t G;            // workgroups per row
    uint32_t rounds;       // arrival rounds so far (the same in every workgroup of the row)
    uint32_t spin_limit;   // polls per wait
};

__device__ __forceinline__ void raise_abort(uint32_t *abort_flag)
{
    __hip_atomic_store(abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// True in the workgroup whose arrival completes the round.  All threads must call.
__device__ __forceinline__ bool row_arrive(RowSync &rs)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    rs.rounds++;
    if (threadIdx.x == 0) {
        const uint32_t prev = rs.bar->fetch_add(1u);
        rs.sh[0] = (prev + 1u == rs.rounds * rs.G) ? 1u : 0u;
    }
    __syncthreads();
    const bool last = rs.sh[0] != 0u;
    __syncthreads();
    return last;
}

// rem < 2^31; bin = kNone or < 2^31 - 1
__device__ __forceinline__ void row_publish(RowSync &rs, int slot, uint32_t bin, uint32_t rem)
{
    const uint64_t enc = kResValid | (static_cast<uint64_t>((bin == kNone) ? 0u : bin + 1u) << 32) | rem;
    rs.res[slot].store(enc);
}

__device__ __forceinline__ bool row_wait_result(RowSync &rs, int slot, uint32_t *bin, uint32_t *rem)
{
    if (threadIdx.x == 0) {
        uint64_t v = 0;
        uint32_t ok = 1u;
        for (uint32_t spins = 0;; ++spins) {
            v = rs.res[slot].load();
            if (v & kResValid) break;
            __builtin_amdgcn_s_sleep(1);
            if (spins >= rs.spin_limit) { ok = 0u; raise_abort(rs.abort_flag); break; }
        }
        const uint32_t enc = static_cast<uint32_t>(v >> 32) & 0x7FFFFFFFu;
        rs.sh[0] = ok;
        rs.sh[1] = enc ? enc - 1u : kNone;
        rs.sh[2] = static_cast<uint32_t>(v);
    }
    __syncthreads();
    const bool ok = rs.sh[0] != 0u;
    *bin = rs.sh[1];
    *rem = rs.sh[2];
    __syncthreads();
    return ok;
}

// A plain barrier over the row's workgroups.  False: gave up.
__device__ __forceinline__ bool row_barrier(RowSync &rs, int slot)
{
    if (row_arrive(rs) && threadIdx.x == 0) row_publish(rs, slot, kNone, 0u);
    uint32_t b, r;
    return row_wait_result(rs, slot, &b, &r);
}

// Run by the workgroup that completed the round.
template <int NB>
__device__ __forceinline__ void row_pick_publish(RowSync &rs, int slot, const DevWord *hist, uint32_t need,
                                                 uint32_t *part, uint32_t *out)
{
    if (threadIdx.x == 0) { out[0] = kNone; out[1] = 0u; }
    __syncthreads();
    pick_bin<NB>(hist, need, part, &out[0], &out[1]);
    __syncthreads();
    if (threadIdx.x == 0) row_publish(rs, slot, out[0], out[1]);
}

// The candidates of the first group a wavefront owns, kept in LDS across the phases of
// k_topk_finish: the wavefront walks the same groups in every phase, and with one group per
// wavefront (the usual case: the grid is sized for it) only the first phase then reads the
// candidate lists from memory.  A group spans 32768 elements, so an index is kept as 16 bits
// relative to the group's first element.  Holds up to 64 * kPrefetch candidates; a larger group
// is simply not cached.
constexpr uint32_t kCacheCap = 64 * kPrefetch;
struct WaveCache {
    uint32_t *bits;      // LDS, kCacheCap words: value bits (key = bits & 0x7FFFFFFF)
    uint16_t *rel;       // LDS, kCacheCap halfwords: index - 32768 * group
    uint32_t total;      // candidates of the cached group
    bool valid;
};

// f(key) for every candidate of the groups this wavefront owns (the same groups in every
// phase: group = workgroup * 8 + wavefront, then strided by the row's wavefront count).
// FILL: the walk fills the cache from its first group; otherwise a valid cache replaces the
// fetch of that group.
template <bool FILL, class F>
__device__ __forceinline__ void for_each_candidate(const u32x2 *__restrict__ srow, const uint32_t *__restrict__ cnt_row,
                                                   int64_t n_reg, int64_t n_groups, uint32_t G, WaveCache &wc, F f)
{
    const int64_t g0 = static_cast<int64_t>(blockIdx.x) * kWaves + wave_id();
    if (FILL) wc.valid = false;
    for (int64_t g = g0; g < n_groups; g += static_cast<int64_t>(G) * kWaves) {
        if (!FILL && g == g0 && wc.valid) {
#pragma unroll
            for (int j = 0; j < kPrefetch; ++j) {
                const uint32_t i = j * 64 + lane_id();
                if (i < wc.total) f(wc.bits[i] & 0x7FFFFFFFu);
            }
            continue;
        }
        const GroupWalk w = group_begin(cnt_row, g, n_reg);
        const bool fill = FILL && g == g0 && w.total <= kCacheCap;
        for (uint32_t i0 = 0; i0 < w.total; i0 += 64 * kPrefetch) {
            const Batch bt = group_fetch_batches(w, srow, g, i0);
#pragma unroll
            for (int j = 0; j < kPrefetch; ++j)
                if (i0 + j * 64 + lane_id() < w.total) {
                    if (fill) {
                        wc.bits[j * 64 + lane_id()] = bt.pr[j].y;
                        wc.rel[j * 64 + lane_id()] = static_cast<uint16_t>(bt.pr[j].x & (kGroupRegs * kReg - 1));
                    }
                    f(bt.pr[j].y & 0x7FFFFFFFu);
                }
        }
        if (fill) { wc.total = w.total; wc.valid = true; }
    }
}

__device__ __forceinline__ void flush_hist(const uint32_t *h, DevWord *gh, int nb)
{
    for (int i = threadIdx.x; i < nb; i += kBlock)
        if (h[i]) gh[i].add(h[i]);
}

struct FinishArgs {
    u32x2 *slots;
    uint32_t *reg_cnt;
    int64_t n_reg, reg_pad, n_groups, n_sub;
    const Sel *sel;
    DevWord *fhist;        // [rows][kFRow], zero on entry
    char *sync;            // [rows][kSyncStride] arrival counter and published words, zero on entry
    uint32_t *abort_flag;
    uint32_t spin_limit;
    DevWord *grp_gt, *grp_eq;
    uint32_t *prev_T;
    float *buf;
    bool wr;               // false: buf is read only (no compensation: it is the gradient) and nothing is stored into it
    int64_t stride, d, k;
    u32x2 *pairs;
    float *x;              // not null: the model update is applied with the emission (one-row launches only)
    float gamma;
    uint32_t *zero_a;            // the sample's histograms of this call (dead by now), cleared here
    int64_t zero_a_words;
};

__global__ __launch_bounds__(kBlock, 8) void k_topk_finish(FinishArgs a)
{
    __shared__ uint32_t h[kHB];
    __shared__ uint32_t cache_bits[kWaves][kCacheCap];
    __shared__ uint16_t cache_rel[kWaves][kCacheCap];
    __shared__ uint32_t part[kWaves], out[2], sh[3], wtot[kWaves], red[2 * kWaves];
    const int row = blockIdx.y;
    const uint32_t G = gridDim.x;
    WaveCache wc{cache_bits[wave_id()], cache_rel[wave_id()], 0u, false};
    RowSync rs{reinterpret_cast<DevWord *>(a.sync + row * kSyncStride), reinterpret_cast<DevWord64 *>(a.sync + row * kSyncStride + 128),
               a.abort_flag, sh, G, 0u, a.spin_limit};
    DevWord *fh = a.fhist + static_cast<int64_t>(row) * kFRow;
    u32x2 *srow = a.slots + static_cast<int64_t>(row) * a.n_reg * kReg;
    uint32_t *cnt_row = a.reg_cnt + row * a.reg_pad;
    float *brow = a.buf + row * a.stride;          // read by the two-look route
    float *wrow = a.wr ? brow : nullptr;           // where candidates that are not kept get v back
    const uint32_t k32 = static_cast<uint32_t>(a.k);
    {
        const int64_t first = (static_cast<int64_t>(blockIdx.y) * G + blockIdx.x) * kBlock + threadIdx.x;
        const int64_t step = static_cast<int64_t>(gridDim.y) * G * kBlock;
        for (int64_t i = first; i < a.zero_a_words; i += step) a.zero_a[i] = 0u;
    }
    uint32_t lo_key = a.sel[row].lo_key;
    uint32_t bA = kNone, kA = 0u;

    auto level_a = [&](DevWord *gh, int slot) -> bool {
        for (int i = threadIdx.x; i < kHA; i += kBlock) h[i] = 0u;
        __syncthreads();
        for_each_candidate<true>(srow, cnt_row, a.n_reg, a.n_groups, G, wc, [&](uint32_t key) {
            const uint32_t rel = (key - lo_key) >> kShiftA;
            atomicAdd(&h[rel < kHA ? rel : kHA - 1], 1u);
        });
        __syncthreads();
        flush_hist(h, gh, kHA);
        if (row_arrive(rs)) row_pick_publish<kHA>(rs, slot, gh, k32, part, out);
        return row_wait_result(rs, slot, &bA, &kA);
    };

    if (!level_a(fh + kFOffA, kResA)) return;
    if (bA == kNone || bA == kHA - 1) {
        // exact two-look route.  A workgroup owns the same tiles in all of its steps, so what
        // it reads back is what it wrote itself.
        // (the dense histogram has 4096 bins: it takes the memory of the wavefronts' caches, whose
        // candidates are about to be replaced)
        wc.valid = false;
        uint32_t *h = &cache_bits[0][0];
        static_assert(kWaves * kCacheCap >= kH1, "the caches must hold the dense histogram");
        __syncthreads();
        for (int i = threadIdx.x; i < kH1; i += kBlock) h[i] = 0u;
        __syncthreads();
        const bool vec = aligned16(brow);
        for (int64_t tile = blockIdx.x; tile < a.n_reg; tile += G) {
            const uint32_t cnt = cnt_row[tile];
            const u32x2 *src = srow + tile * kReg;
            if (a.wr)
                for (uint32_t i = threadIdx.x; i < cnt; i += kBlock) brow[src[i].x] = __uint_as_float(src[i].y);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            const int64_t e = tile * kTile + threadIdx.x * 4;
            if (e < a.d) {
                const f32x4 v = ld4(brow, e, a.d, vec);
                if (e + 0 < a.d) atomicAdd(&h[key_of(v.x) >> 19], 1u);
                if (e + 1 < a.d) atomicAdd(&h[key_of(v.y) >> 19], 1u);
                if (e + 2 < a.d) atomicAdd(&h[key_of(v.z) >> 19], 1u);
                if (e + 3 < a.d) atomicAdd(&h[key_of(v.w) >> 19], 1u);
            }
        }
        __syncthreads();
        flush_hist(h, fh + kFOffD, kH1);
        if (row_arrive(rs)) row_pick_publish<kH1>(rs, kResD, fh + kFOffD, k32, part, out);
        uint32_t b1, k1;
        if (!row_wait_result(rs, kResD, &b1, &k1)) return;
        if (b1 == kNone) { raise_abort(a.abort_flag); return; }       // cannot happen: k <= d
        lo_key = b1 << 19;
        const BufferV bsrc{a.buf, a.stride};
        for (int64_t tile = blockIdx.x; tile < a.n_reg; tile += G) {
            if (a.wr)
                pass1_tile<BufferV, true, true>(bsrc, a.buf, a.stride, a.d, a.n_sub, lo_key, a.slots, a.reg_cnt, a.n_reg,
                                                a.reg_pad, row, tile, nullptr, wtot);
            else
                pass1_tile<BufferV, true, false>(bsrc, a.buf, a.stride, a.d, a.n_sub, lo_key, a.slots, a.reg_cnt, a.n_reg,
                                                 a.reg_pad, row, tile, nullptr, wtot);
        }
        // the new candidate lists cross workgroups (and their caches) from here on
        __threadfence();
        if (!row_barrier(rs, kResCompact)) return;
        __threadfence();
        if (!level_a(fh + kFOffA2, kResA2)) return;
        if (bA == kNone || bA == kHA - 1) { raise_abort(a.abort_flag); return; }   // cannot happen
    }

    // level B: the low bits inside bin A
    for (int i = threadIdx.x; i < kHB; i += kBlock) h[i] = 0u;
    __syncthreads();
    for_each_candidate<false>(srow, cnt_row, a.n_reg, a.n_groups, G, wc, [&](uint32_t key) {
        const uint32_t rel = key - lo_key;
        if ((rel >> kShiftA) == bA) atomicAdd(&h[rel & (kHB - 1)], 1u);
    });
    __syncthreads();
    flush_hist(h, fh + kFOffB, kHB);
    if (row_arrive(rs)) row_pick_publish<kHB>(rs, kResB, fh + kFOffB, kA, part, out);
    uint32_t bB, k3;
    if (!row_wait_result(rs, kResB, &bB, &k3)) return;
    if (bB == kNone) { raise_abort(a.abort_flag); return; }           // cannot happen
    const uint32_t T = lo_key + (bA << kShiftA) + bB;

    // per group: candidates above T, candidates tying with T
    DevWord *gtr = a.grp_gt + row * a.n_groups, *eqr = a.grp_eq + row * a.n_groups;
    {
        const int64_t g0 = static_cast<int64_t>(blockIdx.x) * kWaves + wave_id();
        for (int64_t g = g0; g < a.n_groups; g += static_cast<int64_t>(G) * kWaves) {
            uint32_t gt = 0, eq = 0;
            if (g == g0 && wc.valid) {
#pragma unroll
                for (int j = 0; j < kPrefetch; ++j) {
                    const uint32_t i = j * 64 + lane_id();
                    const uint32_t key = (i < wc.total) ? (wc.bits[i] & 0x7FFFFFFFu) : 0u;
                    gt += i < wc.total && key > T;
                    eq += i < wc.total && key == T;
                }
            } else {
                const GroupWalk w = group_begin(cnt_row, g, a.n_reg);
                for (uint32_t i0 = 0; i0 < w.total; i0 += 64 * kPrefetch) {
                    const Batch bt = group_fetch_batches(w, srow, g, i0);
#pragma unroll
                    for (int j = 0; j < kPrefetch; ++j) {
                        const bool valid = i0 + j * 64 + lane_id() < w.total;
                        const uint32_t key = bt.pr[j].y & 0x7FFFFFFFu;
                        gt += valid && key > T;
                        eq += valid && key == T;
                    }
                }
            }
            gt = wave_sum_u32(gt);
            eq = wave_sum_u32(eq);
            if (lane_id() == 0) {
                gtr[g].store(gt);
                eqr[g].store(eq);
            }
        }
    }
    if (!row_barrier(rs, kResCount)) return;

    // emit.  Ties are taken in index order, so the ties kept before a group number
    // min(k3, ties before it): two running sums over the groups give every offset.  All the
    // loads of a round are issued before the first is used.
    uint32_t sum_gt = 0, sum_eq = 0;
    int64_t upto = 0;
    u32x2 *prow = a.pairs + static_cast<int64_t>(row) * a.k;
    const int64_t g0 = static_cast<int64_t>(blockIdx.x) * kWaves + wave_id();
    for (int64_t gb = static_cast<int64_t>(blockIdx.x) * kWaves; gb < a.n_groups; gb += static_cast<int64_t>(G) * kWaves) {
        const int64_t g = gb + wave_id();
        uint32_t wg = 0, we = 0;                               // groups gb .. g-1 of this workgroup's round
        if (g < a.n_groups && lane_id() < wave_id()) { wg = gtr[gb + lane_id()].load(); we = eqr[gb + lane_id()].load(); }
        uint32_t pg = 0, pe = 0;
        for (int64_t t = upto + threadIdx.x; t < gb; t += kBlock) {
            pg += gtr[t].load();
            pe += eqr[t].load();
        }
        pg = wave_sum_u32(pg);
        pe = wave_sum_u32(pe);
        __syncthreads();
        if (lane_id() == 0) { red[wave_id()] = pg; red[kWaves + wave_id()] = pe; }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { sum_gt += red[w]; sum_eq += red[kWaves + w]; }
        upto = gb;
        if (g < a.n_groups) {
            const uint32_t gtb = sum_gt + wave_sum_u32(wg), eqb = sum_eq + wave_sum_u32(we);
            uint32_t out_slot = gtb + (eqb < k3 ? eqb : k3), eq_seen = eqb;
            if (g == g0 && wc.valid) {
                const uint32_t base = static_cast<uint32_t>(g) * (kGroupRegs * kReg);
                uint32_t kept = 0u;                            // bit j: this lane's candidate of batch j is kept
#pragma unroll
                for (int j = 0; j < kPrefetch; ++j) {
                    if (j * 64u >= wc.total) continue;         // uniform over the wavefront
                    const uint32_t i = j * 64 + lane_id();
                    const bool valid = i < wc.total;
                    const u32x2 pr = valid ? u32x2{base + wc.rel[i], wc.bits[i]} : u32x2{0u, 0u};
                    if (emit_batch(pr, valid, T, k3, eq_seen, out_slot, prow, wrow, a.k)) kept |= 1u << j;
                }
                if (a.x) {
                    // the model update at the kept entries: all loads first (the entries of a
                    // group are distinct elements), so that they are in flight together
                    float xv[kPrefetch];
#pragma unroll
                    for (int j = 0; j < kPrefetch; ++j) xv[j] = ((kept >> j) & 1u) ? a.x[base + wc.rel[j * 64 + lane_id()]] : 0.f;
#pragma unroll
                    for (int j = 0; j < kPrefetch; ++j)
                        if ((kept >> j) & 1u)
                            a.x[base + wc.rel[j * 64 + lane_id()]] =
                                __fmaf_rn(-a.gamma, __uint_as_float(wc.bits[j * 64 + lane_id()]), xv[j]);
                }
            } else {
                const GroupWalk w = group_begin(cnt_row, g, a.n_reg);
                emit_group(w, srow, g, T, k3, eqb, out_slot, prow, wrow, a.k, a.x, a.gamma);
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) a.prev_T[row] = T;   // centre of the next call's fine sampling window
    // every pick of the row is done (the emission needed the last one) and every workgroup
    // flushed before the pick it waited for: clear the row's histograms for the next call.  The
    // row's synchronisation words are cleared by the next call's sample kernel, which no
    // workgroup of this launch can overlap with.
    for (int i = blockIdx.x * kBlock + threadIdx.x; i < kFRow; i += G * kBlock) fh[i].clear_for_next_launch();
}

// ---------------------------------------------------------------------------------------
// consumers of a sparse message
// ---------------------------------------------------------------------------------------
// x <- fma(-gamma, val, x) at the kept indices (Algorithm 1, model update).
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
    __shared__ int64_t range[2];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kTile;
    const int64_t e = base + threadIdx.x * 4;
#pragma unroll
    for (int c = 0; c < 4; ++c) tilev[threadIdx.x * 4 + c] = 0.f;
    if (threadIdx.x < 2) range[threadIdx.x] = lower_bound_idx(pairs, k, base + threadIdx.x * kTile);
    __syncthreads();
    for (int64_t j = range[0] + threadIdx.x; j < range[1]; j += kBlock) {
        const u32x2 pr = pairs[j];
        const uint32_t rel = pr.x - static_cast<uint32_t>(base);
        if (rel < static_cast<uint32_t>(kTile)) tilev[rel] = __uint_as_float(pr.y);
    }
    __syncthreads();
    if (e >= d) return;
    const f32x4 q = {tilev[threadIdx.x * 4 + 0], tilev[threadIdx.x * 4 + 1], tilev[threadIdx.x * 4 + 2],
                     tilev[threadIdx.x * 4 + 3]};
    apply_q4<MOM, DECODE_ONLY>(q, e, d, x, m, gamma, beta);
}

// Zeroes up to five arrays of 32-bit words (the context's scratch state after a failed launch).
__global__ __launch_bounds__(kBlock) void k_topk_clear(uint32_t *a, int64_t na, uint32_t *b, int64_t nb, uint32_t *c,
                                                       int64_t nc, uint32_t *d, int64_t nd, uint32_t *e, int64_t ne)
{
    const int64_t first = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x, step = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t i = first; i < na; i += step) a[i] = 0u;
    for (int64_t i = first; i < nb; i += step) b[i] = 0u;
    for (int64_t i = first; i < nc; i += step) c[i] = 0u;
    for (int64_t i = first; i < nd; i += step) d[i] = 0u;
    for (int64_t i = first; i < ne; i += step) e[i] = 0u;
}

unsigned persistent_blocks(int64_t n_tiles, int rows)
{
    int64_t per_row = (1024 + rows - 1) / rows;   // about 4 workgroups per compute unit in total
    if (per_row < 1) per_row = 1;
    if (per_row > n_tiles) per_row = n_tiles;
    return static_cast<unsigned>(per_row);
}

// sample -> dense pass -> refinement -> ordered emission, for `rows` vectors
// wr = false: buf is the vector v itself, read only (no compensation: v = g), for the second look
// of the exact route; nothing is stored into it.
template <class Src>
ds_status_t run_select(ds_ctx *c, int rows, const Src &src, float *buf, int64_t stride, u32x2 *pairs, hipStream_t st,
                       uint32_t *prev_T, float *x = nullptr, float gamma = 0.f, bool wr = true)
{
    ds_topk_scratch *t = c->topk;
    if (__atomic_load_n(t->abort_host, __ATOMIC_RELAXED)) {
        // An earlier single launch gave up a wait and left its synchronisation words and
        // histograms dirty.  This call clears them on its stream (kernels: the call may be
        // under capture), moves the context to the chain of launches, which waits for nothing,
        // and reports the failure once.
        const int64_t n_rows = t->rows;
        k_topk_clear<<<64, kBlock, 0, st>>>(t->hist, n_rows * kHistRow, t->fhist, n_rows * kFRow,
                                            reinterpret_cast<uint32_t *>(t->sync), n_rows * (kSyncStride / 4), t->done,
                                            n_rows * kStages, t->prev_T, n_rows + 1);
        t->capacity = 0;
        __atomic_store_n(t->abort_host, 0u, __ATOMIC_RELAXED);
        (void)ds_launch_status();
        return DS_ERR_DEVICE;
    }
    const int64_t d = c->cfg.d, k = c->cfg.k, n_sub = t->n_sub, n_reg = t->n_reg, reg_pad = t->reg_pad, n_groups = t->n_groups;
    const int64_t ns = (n_sub < kSampleSubs) ? n_sub : kSampleSubs;
    // sample rank: 1.15 x the expected number of top-k members in the sample, plus slack
    // (k = 1 % of 25.6 M: 1311 expected in 131072 samples, rank 1539, i.e. 6 standard
    // deviations of the count)
    const double sample_elems = static_cast<double>((ns * kSub < d) ? ns * kSub : d);
    double r = 1.15 * static_cast<double>(k) * sample_elems / static_cast<double>(d) + 32.0;
    if (r > 4.0e9) r = 4.0e9;
    const uint32_t rank = static_cast<uint32_t>(r);
    const unsigned grp_blocks = static_cast<unsigned>((n_groups + kWaves - 1) / kWaves);
    const dim3 dense(static_cast<unsigned>(c->n_tiles), rows), cand(grp_blocks, rows);
    const BufferV bsrc{buf, stride};

    // The scratch memory is plain words to the host and to the clearing code; the launches whose
    // workgroups hand those words to each other see them typed.
    uint32_t *hist = t->hist;
    DevWord *s_hist = as_shared(t->hist), *s_done = as_shared(t->done);
    DevWord *s_gt = as_shared(t->grp_gt), *s_eq = as_shared(t->grp_eq);
    const uint32_t k32 = static_cast<uint32_t>(k);

    k_topk_sample<Src><<<dim3(static_cast<unsigned>((ns + kWaves - 1) / kWaves), rows), kBlock, 0, st>>>(
        src, d, n_sub, ns, s_hist, t->sel, s_done, rank, prev_T, reinterpret_cast<DevWord *>(t->sync));
    if constexpr (std::is_same<Src, ServerV>::value)
        k_topk_pass1_server<false><<<dim3(static_cast<unsigned>((n_reg + 3) / 4)), kBlock, 0, st>>>(
            src, buf, d, t->sel, t->slots, t->reg_cnt, n_reg, ds_update_args{nullptr, nullptr, 0.f, 0.f});
    else if (wr)
        k_topk_pass1<Src, false, true><<<dense, kBlock, 0, st>>>(src, buf, stride, d, n_sub, t->sel, t->slots, t->reg_cnt, n_reg, reg_pad);
    else
        k_topk_pass1<Src, false, false><<<dense, kBlock, 0, st>>>(src, buf, stride, d, n_sub, t->sel, t->slots, t->reg_cnt, n_reg, reg_pad);
    if (t->capacity >= rows) {
        // everything after the dense pass in one launch whose workgroups are all resident
        int64_t G = t->capacity / rows;
        if (G > grp_blocks) G = grp_blocks;
        FinishArgs a;
        a.slots = t->slots; a.reg_cnt = t->reg_cnt;
        a.n_reg = n_reg; a.reg_pad = reg_pad; a.n_groups = n_groups; a.n_sub = n_sub;
        a.sel = t->sel; a.fhist = as_shared(t->fhist); a.sync = t->sync; a.abort_flag = t->abort_host; a.spin_limit = t->spin_limit;
        a.grp_gt = s_gt; a.grp_eq = s_eq; a.prev_T = prev_T;
        a.buf = buf; a.wr = wr; a.stride = stride; a.d = d; a.k = k; a.pairs = pairs; a.x = x; a.gamma = gamma;
        a.zero_a = hist; a.zero_a_words = static_cast<int64_t>(rows) * kHistRow;
        k_topk_finish<<<dim3(static_cast<unsigned>(G), rows), kBlock, 0, st>>>(a);
        return ds_launch_status();
    }
    k_topk_cand_hist<1><<<cand, kBlock, 0, st>>>(t->slots, t->reg_cnt, n_reg, reg_pad, n_groups, t->sel, s_hist, s_done, k32, prev_T, buf, stride, wr);
    // two-look route for rows whose sample misjudged; both launches exit at once otherwise
    k_topk_fallback_hist<<<dim3(persistent_blocks(c->n_tiles, rows), rows), kBlock, 0, st>>>(buf, stride, d, c->n_tiles,
                                                                                            t->sel, s_hist, s_done, k32);
    if (wr)
        k_topk_pass1<BufferV, true, true><<<dim3(persistent_blocks(c->n_tiles, rows), rows), kBlock, 0, st>>>(
            bsrc, buf, stride, d, n_sub, t->sel, t->slots, t->reg_cnt, n_reg, reg_pad);
    else
        k_topk_pass1<BufferV, true, false><<<dim3(persistent_blocks(c->n_tiles, rows), rows), kBlock, 0, st>>>(
            bsrc, buf, stride, d, n_sub, t->sel, t->slots, t->reg_cnt, n_reg, reg_pad);
    // refinement on the candidates
    k_topk_cand_hist<2><<<cand, kBlock, 0, st>>>(t->slots, t->reg_cnt, n_reg, reg_pad, n_groups, t->sel, s_hist, s_done, k32, prev_T, buf, stride, wr);
    k_topk_cand_hist<3><<<cand, kBlock, 0, st>>>(t->slots, t->reg_cnt, n_reg, reg_pad, n_groups, t->sel, s_hist, s_done, k32, prev_T, buf, stride, wr);
    k_topk_count<<<cand, kBlock, 0, st>>>(t->slots, t->reg_cnt, n_reg, reg_pad, n_groups, t->sel, s_gt, s_eq,
                                          t->grp_eqb, t->grp_out, s_done, hist,
                                          static_cast<int64_t>(rows) * kHistRow);
    k_topk_emit<<<cand, kBlock, 0, st>>>(t->slots, t->reg_cnt, n_reg, reg_pad, n_groups, t->sel, t->grp_eqb, t->grp_out, k,
                                         pairs, buf, stride, x, gamma, wr);
    return ds_launch_status();
}

}  // namespace

ds_status_t ds_topk_init(ds_ctx *c)
{
    ds_topk_scratch *t = new (std::nothrow) ds_topk_scratch();
    if (!t) return DS_ERR_DEVICE;
    *t = ds_topk_scratch{};
    c->topk = t;
    const size_t rows = static_cast<size_t>(c->cfg.n);
    t->rows = c->cfg.n;
    t->n_sub = (c->cfg.d + kSub - 1) / kSub;
    t->n_reg = c->n_tiles;
    t->n_groups = (t->n_reg + kGroupRegs - 1) / kGroupRegs;
    t->reg_pad = t->n_groups * kGroupRegs;
    DS_HIP_TRY(hipMalloc(&t->hist, rows * kHistRow * sizeof(uint32_t)));
    DS_HIP_TRY(hipMemset(t->hist, 0, rows * kHistRow * sizeof(uint32_t)));
    DS_HIP_TRY(hipMalloc(&t->prev_T, (rows + 1) * sizeof(uint32_t)));
    DS_HIP_TRY(hipMemset(t->prev_T, 0, (rows + 1) * sizeof(uint32_t)));
    DS_HIP_TRY(hipMalloc(&t->done, rows * kStages * sizeof(uint32_t)));
    DS_HIP_TRY(hipMemset(t->done, 0, rows * kStages * sizeof(uint32_t)));
    DS_HIP_TRY(hipMalloc(&t->sel, rows * sizeof(Sel)));
    DS_HIP_TRY(hipMalloc(&t->slots, rows * static_cast<size_t>(t->n_reg) * kReg * sizeof(u32x2)));
    DS_HIP_TRY(hipMalloc(&t->reg_cnt, rows * static_cast<size_t>(t->reg_pad) * sizeof(uint32_t)));
    uint32_t **tabs[4] = {&t->grp_gt, &t->grp_eq, &t->grp_eqb, &t->grp_out};
    for (auto tab : tabs) DS_HIP_TRY(hipMalloc(tab, rows * static_cast<size_t>(t->n_groups) * sizeof(uint32_t)));
    DS_HIP_TRY(hipMalloc(&t->sub_start, rows * static_cast<size_t>(t->n_sub + 1) * sizeof(uint32_t)));
    DS_HIP_TRY(hipMemset(t->sub_start, 0, rows * static_cast<size_t>(t->n_sub + 1) * sizeof(uint32_t)));
    DS_HIP_TRY(hipMemset(t->reg_cnt, 0, rows * static_cast<size_t>(t->reg_pad) * sizeof(uint32_t)));
    DS_HIP_TRY(hipMalloc(&t->fhist, rows * kFRow * sizeof(uint32_t)));
    DS_HIP_TRY(hipMemset(t->fhist, 0, rows * kFRow * sizeof(uint32_t)));
    DS_HIP_TRY(hipMalloc(&t->sync, rows * kSyncStride));
    DS_HIP_TRY(hipMemset(t->sync, 0, rows * kSyncStride));
    DS_HIP_TRY(hipHostMalloc(reinterpret_cast<void **>(&t->abort_host), sizeof(uint32_t), hipHostMallocDefault));
    *t->abort_host = 0u;
    // The fused route needs its whole grid resident: workgroups per compute unit from the
    // occupancy query times the number of compute units.
    t->capacity = 0;
    if (!(c->cfg.flags & DS_FLAG_TOPK_MULTI_LAUNCH)) {
        int per_cu = 0, cus = 0;
        DS_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_topk_finish, kBlock, 0));
        DS_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device));
        t->capacity = static_cast<int64_t>(per_cu) * cus;
        // ds_config_t::topk_max_workgroups caps the workgroups the single launch uses;
        // ds_config_t::topk_spin_limit sets the polls per wait (-1: none, the host-forced
        // failure for tests of the error path: every wait that is not satisfied at once fails
        // and every workgroup still exits)
        t->spin_limit = kSpinLimit;
        if (c->cfg.topk_spin_limit > 0) t->spin_limit = static_cast<uint32_t>(c->cfg.topk_spin_limit);
        if (c->cfg.topk_spin_limit < 0) t->spin_limit = 0u;
        if (c->cfg.topk_max_workgroups > 0 && c->cfg.topk_max_workgroups < t->capacity) t->capacity = c->cfg.topk_max_workgroups;
    }
    return DS_OK;
}

// The table of every worker's first entry per 256-element subtile, for the server's dense pass.
static void build_sub_starts(ds_ctx *c, const u32x2 *pairs_in, hipStream_t st)
{
    ds_topk_scratch *t = c->topk;
    const int64_t k = c->cfg.k;
    if (k * 4 >= t->n_sub)
        k_topk_sub_starts_scan<<<dim3(static_cast<unsigned>((k + 1 + kBlock - 1) / kBlock), c->cfg.n), kBlock, 0, st>>>(
            pairs_in, k, t->n_sub, t->sub_start);
    else
        k_topk_sub_starts<<<dim3(static_cast<unsigned>((t->n_sub + 1 + kBlock - 1) / kBlock), c->cfg.n), kBlock, 0, st>>>(
            pairs_in, k, t->n_sub, t->sub_start);
}

ds_status_t ds_topk_status(const ds_ctx *c)
{
    const ds_topk_scratch *t = c->topk;
    return (t && __atomic_load_n(t->abort_host, __ATOMIC_RELAXED)) ? DS_ERR_DEVICE : DS_OK;
}

void ds_topk_fini(ds_ctx *c)
{
    ds_topk_scratch *t = c->topk;
    if (!t) return;
    void *ptrs[13] = {t->prev_T, t->done, t->hist, t->sel, t->slots, t->reg_cnt, t->grp_gt, t->grp_eq, t->grp_eqb, t->grp_out,
                      t->sub_start, t->fhist, t->sync};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    if (t->abort_host) (void)hipHostFree(t->abort_host);
    delete t;
    c->topk = nullptr;
}

ds_status_t ds_topk_worker(ds_ctx *c, const void *g, int64_t gs, float *delta, int64_t dstr, const ds_payload_t *out,
                           hipStream_t st)
{
    const int rows = c->cfg.n;
    u32x2 *pairs = reinterpret_cast<u32x2 *>(out->pairs);
    if (!delta) {
        // no compensation (fp32 gradients only, checked by ds_create): v = g, which also serves
        // the second look of the exact route; no buffer is written
        float *gv = static_cast<float *>(const_cast<void *>(g));
        return run_select(c, rows, GradV{gv, gs}, gv, gs, pairs, st, c->topk->prev_T, nullptr, 0.f, false);
    }
    if (c->cfg.grad_dtype == DS_BF16) return run_select(c, rows, WorkerV<true>{g, gs, delta, dstr}, delta, dstr, pairs, st, c->topk->prev_T);
    return run_select(c, rows, WorkerV<false>{g, gs, delta, dstr}, delta, dstr, pairs, st, c->topk->prev_T);
}

// Server that does not compress: the table of the workers' entries per subtile, then one dense
// pass that builds the average from +0 and writes / applies it.
ds_status_t ds_topk_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st)
{
    ds_topk_scratch *t = c->topk;
    const u32x2 *pairs_in = reinterpret_cast<const u32x2 *>(in->pairs);
    const int64_t k = c->cfg.k;
    build_sub_starts(c, pairs_in, st);
    const ServerV src{pairs_in, t->sub_start, nullptr, k, t->n_sub, c->cfg.n, c->inv_n};
    k_topk_pass1_server<true><<<dim3(static_cast<unsigned>((t->n_reg + 3) / 4)), kBlock, 0, st>>>(
        src, dense_out, c->cfg.d, t->sel, t->slots, t->reg_cnt, t->n_reg, u);
    return ds_launch_status();
}

// x != nullptr: also x <- fma(-gamma, val, x) at the kept indices of the server's message.
ds_status_t ds_topk_server(ds_ctx *c, const ds_payload_t *in, float *delta_s, const ds_payload_t *out, hipStream_t st,
                           float *x, float gamma)
{
    ds_topk_scratch *t = c->topk;
    const u32x2 *pairs_in = reinterpret_cast<const u32x2 *>(in->pairs);
    const int64_t k = c->cfg.k;
    build_sub_starts(c, pairs_in, st);
    const ServerV src{pairs_in, t->sub_start, delta_s, k, t->n_sub, c->cfg.n, c->inv_n};
    return run_select(c, 1, src, delta_s, c->cfg.d, reinterpret_cast<u32x2 *>(out->pairs), st, t->prev_T + t->rows, x, gamma);
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
