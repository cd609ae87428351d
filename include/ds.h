/*
 * ds.h -- C-ABI of the MI355X (gfx950) DoubleSqueeze step library, libds_hip.so.
 *
 * The three step calls follow Algorithm 1 and Section 3.1 of
 *   Tang, Yu, Lian, Zhang, Liu, "DoubleSqueeze: Parallel Stochastic Gradient Descent with
 *   Double-pass Error-Compensated Compression", ICML 2019,
 * with the n workers laid out as the n rows of one [n, d] tensor on one GPU:
 *
 *   ds_worker_compress            "On worker", first block of Algorithm 1:
 *                                 v_i = g_i + delta_i ; payload_i = Q[v_i] ;
 *                                 delta_i <- v_i - Q[v_i]
 *   ds_server_aggregate_compress  "On parameter server":
 *                                 v = delta + (1/n) sum_i Q[v_i] ; payload = Q[v] ;
 *                                 delta <- v - Q[v]
 *   ds_apply_update               "On worker", second block:  x <- x - gamma Q[v]
 *
 * Q[.] is pluggable (Section 3.2, "Compression options"): 1-bit sign with a scale
 * (Section 5.1 "1-bit compression"), top-k by absolute value (Section 5.1 "Top-k
 * compression"), two-point unbiased randomised quantisation (Section 3.2 "Randomized
 * Quantization", bucketed with an L2 norm), clipping of low bits (Section 3.2 "Clipping"),
 * randomised sparsification (Section 3.2 "Randomized Sparsification"), the identity
 * (Section 5.1 "Vanilla SGD") and the ternary quantiser of Section 5.1's "QSGD" comparison
 * system.  Two flags turn Algorithm 1 into the other comparison algorithms of Section 5.1:
 * DS_FLAG_SERVER_IDENTITY (no second compression: "MEM-SGD") and DS_FLAG_NO_ERROR_FEEDBACK
 * (no compensation: "Top-k SGD", "QSGD").
 *
 * Conventions that hold for every call
 *   - Every data pointer is DEVICE memory owned by the caller (base address 16-byte
 *     aligned).  The library never frees or keeps a caller pointer after the call.
 *     ds_config_t::seg_offsets is the one HOST pointer; it is copied by ds_create.
 *   - State (delta, delta_s, x, m) is updated in place.
 *   - Calls are asynchronous: they enqueue kernels on the given HIP stream
 *     (hipStream_t passed as void*, NULL = the default stream) and return.
 *   - The step calls allocate nothing, never synchronise with the host and change no
 *     host-side state from one call to the next (exception: the first call of a context in
 *     deferred error form, see DS_FLAG_DEFERRED_ERROR), so they can be captured into a HIP
 *     graph and replayed; a replay draws its random numbers for the `step` it was captured with.
 *   - Errors are return codes only.  Argument errors are detected before anything is
 *     launched and leave every buffer untouched.
 *   - `step` is the caller's iteration counter t; together with the seed it is the only
 *     random state (counter-based Philox4x32-10), so a run can be resumed by passing the
 *     same buffers and the next step.
 *   - A context is bound to the device that was current in ds_create, holds scratch
 *     memory sized for its configuration, and is not thread-safe.
 *   - Non-finite inputs are not detected; they propagate.
 *   - Arithmetic: fp32, one rounding per operation, no contraction; group sums of |v| and
 *     v^2 are accumulated in fp64 and rounded once.
 */
#ifndef DS_H_
#define DS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DS_OK = 0,
    DS_ERR_NULL = 1,        /* a required pointer is NULL */
    DS_ERR_SHAPE = 2,       /* n, d, strides, rows out of range */
    DS_ERR_CONFIG = 3,      /* inconsistent configuration */
    DS_ERR_ALIGN = 4,       /* a base pointer is not 16-byte aligned */
    DS_ERR_UNSUPPORTED = 5, /* valid but not implemented */
    DS_ERR_DEVICE = 6       /* a HIP runtime call failed */
} ds_status_t;

typedef enum {
    DS_COMP_IDENTITY = 0,
    DS_COMP_SIGN = 1,
    DS_COMP_TOPK = 2,
    DS_COMP_QSGD = 3,
    DS_COMP_CLIP = 4,
    DS_COMP_RSPARSE = 5,
    DS_COMP_TERNARY = 6
} ds_compressor_t;

typedef enum { DS_F32 = 0, DS_BF16 = 1 } ds_dtype_t;

/* Scale groups of the 1-bit compressor (the paper uses one scale per vector, Section 5.1;
 * per-segment and per-chunk scales are the workloads' refinement of the same rule). */
typedef enum {
    DS_SCALE_WHOLE = 0,     /* one group: the whole vector */
    DS_SCALE_SEGMENTS = 1,  /* caller-given consecutive segments */
    DS_SCALE_CHUNK = 2      /* fixed-size chunks, last one short */
} ds_scale_mode_t;

/* ds_config_t::flags.
 * DS_FLAG_TOPK_MULTI_LAUNCH: TOPK refines its threshold in a chain of small launches, none of
 * which waits for anything, instead of one launch whose workgroups wait for each other row by
 * row.  The results are the same.  In the single launch (the default, about 45 us faster per
 * worker call at 8 x 25.6 M elements) a workgroup waits only for workgroups of its own row,
 * which precede or surround it in dispatch order, and every wait is bounded
 * (ds_config_t::topk_spin_limit polls).  A launch that gives up a wait raises a flag in
 * host-visible memory; see ds_status for what follows.  ds_config_t::topk_max_workgroups caps
 * the size of the single launch (fewer workgroups than rows selects the chain).
 *
 * DS_FLAG_DEFERRED_ERROR: SIGN with scale groups that span workgroups (whole vector,
 * arbitrary segments, chunks that are no multiple of 128 or exceed 2048) needs the group
 * scale before it can store delta = v - Q[v], i.e. a second look at v.  With this flag the
 * second look is folded into the next call's load: after a call the error buffers hold v, the
 * context holds that call's scales, and the next ds_worker_compress /
 * ds_server_aggregate_compress forms delta = v - Q[v] while it reads the buffer (the same
 * single subtraction, so every message, x, m and the errors themselves are bit-identical to
 * the plain form).  The caller must pass the same logical buffers to consecutive calls and
 * call ds_materialize_error before it reads, copies, checkpoints or edits them.  Contexts for
 * which the flag has no effect (other compressors, chunk scales handled in one pass) ignore
 * it.  Which form a buffer is in is host-side state of the context, and it selects the kernel
 * when a call is enqueued, so a captured graph has the form of its capture time baked in:
 * capture a step only when the buffers are already in deferred form (after at least one
 * eager call), replay it only on buffers in that form, and after ds_materialize_error run one
 * eager call (or capture again) before replaying.
 *
 * DS_FLAG_SIGN_RMS: the SIGN scale of a group is sqrt(mean v^2) instead of mean |v|: the l2
 * reading of Section 3.2's "norm times sign vector" (the decoded group then has the l2 norm
 * of v; with mean |v| it has its l1 norm).
 *
 * DS_FLAG_NO_ERROR_FEEDBACK: Algorithm 1 without its compensation (the un-compensated
 * comparison algorithms of Section 5.1): v_i = g_i on the workers and v = (1/n) sum_i Q[v_i] on
 * the server (the same chain, started from +0).  No error buffer is read or written: the
 * `delta` and `delta_s` arguments are ignored and may be NULL, so a worker pass moves the
 * gradient and the message only.  SIGN, QSGD, CLIP; TOPK with fp32 gradients and
 * DS_FLAG_SERVER_IDENTITY (its selection uses the error buffer as its work space otherwise);
 * TERNARY (which is built for this mode only).  Other combinations: DS_ERR_UNSUPPORTED from
 * ds_create.
 *
 * DS_FLAG_SERVER_IDENTITY: the parameter server averages the workers' messages and sends the
 * average back without compressing it ("MEM-SGD" of Section 5.1; with
 * DS_FLAG_NO_ERROR_FEEDBACK the section's "Top-k SGD" and "QSGD"): v = (1/n) sum_i Q[v_i] by the
 * chain from +0, one kernel that decodes the n messages.  There is no server error (`delta_s`
 * is ignored and may be NULL) and the server's message is the dense vector itself: only
 * `dense` [d] fp32 of its ds_payload_t is used, by ds_server_aggregate_compress (which writes
 * it), ds_apply_update and ds_decompress with rows = 1 (which read it).
 * ds_server_aggregate_compress_update applies the update in the same kernel and writes the
 * average only if out->dense is not NULL.  SIGN, TOPK, QSGD, CLIP, TERNARY. */
typedef enum {
    DS_FLAG_TOPK_MULTI_LAUNCH = 1,
    DS_FLAG_DEFERRED_ERROR = 2,
    DS_FLAG_SIGN_RMS = 4,
    DS_FLAG_NO_ERROR_FEEDBACK = 8,
    DS_FLAG_SERVER_IDENTITY = 16
} ds_flags_t;

typedef struct {
    int32_t comp;             /* ds_compressor_t */
    int32_t n;                /* workers, >= 1 */
    int64_t d;                /* elements per vector, 1 .. 2^31-1 */
    int32_t grad_dtype;       /* ds_dtype_t of g; delta, x, m are always fp32 */
    int32_t scale_mode;       /* SIGN: ds_scale_mode_t */
    int64_t chunk;            /* SIGN + CHUNK: elements per chunk, >= 1 */
    const int64_t *seg_offsets; /* SIGN + SEGMENTS: HOST array of n_seg+1 offsets,
                                 [0] = 0, [n_seg] = d, strictly increasing; copied */
    int32_t n_seg;
    int32_t levels;           /* QSGD: s, number of non-zero levels, 1 .. 15;
                                 CLIP: b, number of low bits set to zero, 1 .. 31 */
    int64_t k;                /* TOPK: entries kept per vector, 1 .. d;
                                 RSPARSE: P24 = p * 2^24, 1 .. 2^24: an element is kept iff its
                                 24-bit uniform is below P24, and kept values are divided by
                                 p = P24 * 2^-24 */
    int32_t bucket;           /* QSGD: elements per bucket, a multiple of 64 (built: the powers of
                                 two 64 .. 2048; other multiples give DS_ERR_UNSUPPORTED) */
    int32_t flags;            /* ds_flags_t bits, 0 for the defaults */
    uint64_t seed;            /* QSGD, RSPARSE, TERNARY: Philox key */
    int32_t topk_max_workgroups; /* TOPK single launch: most workgroups it may use; 0 = what the
                                 device holds at once */
    int32_t topk_spin_limit;  /* TOPK single launch: polls a workgroup spends on one wait before it
                                 gives up; 0 = the default (about 4 million, seconds); -1 = none
                                 (every wait that is not satisfied at once fails: a host-forced
                                 failure for tests of the error path, every kernel still exits) */
} ds_config_t;

typedef struct ds_ctx ds_ctx_t;

/* One kept entry of the top-k message. */
typedef struct { int32_t idx; float val; } ds_pair_t;

/* A batch of `rows` compressed messages, row-major, every member a DEVICE pointer owned by
 * the caller; members the compressor does not use are NULL.  S = number of scale groups,
 * W = ceil(d/64), Bq = ceil(d/bucket).  Sizes come from ds_payload_sizes.
 *   SIGN     sign_words [rows, W]: bit (j & 63) of word (j >> 6) is (v_j < 0), so zero and
 *            negative zero carry bit 0; bits past d are 0.   scales [rows, S]: mean |v|
 *            of each group (root mean square with DS_FLAG_SIGN_RMS).  Decoded element:
 *            bit ? -scale : +scale.
 *   QSGD     levels [rows, ceil(d/2)]: 4-bit code of element j in byte j >> 1, low nibble
 *            for even j; sign_words as above; scales [rows, Bq]: L2 norm of each bucket.
 *            Decoded element: +-(code * (norm / s)).
 *   TOPK     pairs [rows, k]: exactly k entries, ascending idx; the k largest |v| (order
 *            of magnitudes = order of the bit patterns with the sign cleared), equal
 *            magnitudes resolved towards the lower index.  Decoded: val at idx, else 0.
 *   CLIP     levels [rows, d * NB]: the upper 32 - b bits of element j in the NB bytes from
 *            j * NB on, little endian, NB = 1 (b >= 24), 2 (b >= 16) or 4.  Decoded element:
 *            those bits with the cleared low bits as zeros.
 *   RSPARSE  sign_words [rows, W]: bit j = element j is kept (layout as above, bits past d
 *            are written as 0 and ignored when read).  dense [rows, d]: the kept values z / p
 *            of a row packed in index order at its start; what follows them is unspecified.
 *            Decoded element: its packed value if kept, else 0.
 *   TERNARY  (Section 5.1: codes in {-1, 0, +1}; with m = max |v| over the row, element e
 *            becomes sign(e) with probability |e| / m, decided by u < |e| / m with the
 *            element's 24-bit uniform; one scale per row = sum |v| / number of non-zero codes,
 *            0 for an all-zero row)  levels [rows, 8 W] bytes = a plane of W 64-bit words per
 *            row, bit j = code_j is not 0; sign_words [rows, W]: bit j = code_j is -1;
 *            scales [rows, 1].  Decoded element: code * scale.
 *   IDENTITY dense [rows, d]. */
typedef struct {
    uint64_t *sign_words;
    float *scales;
    uint8_t *levels;
    ds_pair_t *pairs;
    float *dense;
} ds_payload_t;

/* Creates a context on the current device and allocates its scratch memory there.
 * Errors: NULL, SHAPE (n, d, k out of range), CONFIG (bad enum, offsets, bucket, levels),
 * UNSUPPORTED (bucket not a power of two up to 2048), DEVICE (allocation failed). */
ds_status_t ds_create(const ds_config_t *cfg, ds_ctx_t **out);

/* Frees the context's scratch memory.  The caller must have synchronised the streams that
 * used it.  NULL is accepted. */
ds_status_t ds_destroy(ds_ctx_t *ctx);

/* Bytes each ds_payload_t member needs for `rows` messages of the context's compressor, in
 * struct order (sign_words, scales, levels, pairs, dense); 0 for unused members.  (The
 * server's message under DS_FLAG_SERVER_IDENTITY is not one of these: it is dense, d * 4
 * bytes.) */
ds_status_t ds_payload_sizes(const ds_ctx_t *ctx, int32_t rows, size_t bytes_out[5]);

/* Worker block of Algorithm 1 for all n workers.
 *   g      [n, g_row_stride]     gradients, cfg.grad_dtype (bf16 is widened exactly)
 *   delta  [n, delta_row_stride] worker errors, fp32, read and overwritten
 *   out    n messages
 * Strides are in elements and >= d.  Rows that are 16-byte aligned take 128-bit loads;
 * other rows take an element-wise path with the same results.
 * QSGD draws its rounding, RSPARSE and TERNARY their keep decisions, from the stream (seed,
 * step, worker i, element j). */
ds_status_t ds_worker_compress(ds_ctx_t *ctx, uint64_t step, const void *g,
                               int64_t g_row_stride, float *delta, int64_t delta_row_stride,
                               const ds_payload_t *out, void *hip_stream);

/* Parameter-server block of Algorithm 1.
 *   in       n messages (as written by ds_worker_compress, or by anything that keeps the
 *            layout above)
 *   delta_s  [d] server error, fp32, read and overwritten
 *   out      1 message
 * The average is the chain acc = delta_s; acc = fma(decode(in_i), 1/n, acc) for
 * i = 0 .. n-1.  QSGD and RSPARSE use the stream (seed, step, 0xFFFFFFFF, j). */
ds_status_t ds_server_aggregate_compress(ds_ctx_t *ctx, uint64_t step, const ds_payload_t *in,
                                         float *delta_s, const ds_payload_t *out,
                                         void *hip_stream);

/* Model update of Algorithm 1 from the server's message `srv` (1 row), q = decode(srv):
 *   m == NULL:  x <- fma(-gamma, q, x)
 *   m != NULL:  m <- fma(beta, m, q) ; x <- fma(-gamma, m, x)     (momentum; the paper's
 *               experiments use none, this is the workloads' extension)
 * x, m: [d] fp32, in place. */
ds_status_t ds_apply_update(ds_ctx_t *ctx, const ds_payload_t *srv, float *x, float *m,
                            float gamma, float beta, void *hip_stream);

/* The parameter-server block followed by the model update, as one call: the same results, bit
 * for bit, as ds_server_aggregate_compress(ctx, step, in, delta_s, out, stream) followed by
 * ds_apply_update(ctx, out, x, m, gamma, beta, stream), for the library to fold the update
 * into the server's kernels where that saves work (TOPK without momentum: x is updated
 * where the kept entries are emitted; RSPARSE: the update takes the offsets of the packed
 * values from the server pass instead of deriving them from the message again).  Arguments
 * and errors as for those two calls. */
ds_status_t ds_server_aggregate_compress_update(ds_ctx_t *ctx, uint64_t step, const ds_payload_t *in,
                                                float *delta_s, const ds_payload_t *out, float *x,
                                                float *m, float gamma, float beta, void *hip_stream);

/* Decodes message `row` of a batch of `rows` messages into dense_out [d] (fp32): the
 * decoder of Q[.] that the server and the update use. */
ds_status_t ds_decompress(ds_ctx_t *ctx, const ds_payload_t *p, int32_t rows, int32_t row,
                          float *dense_out, void *hip_stream);

/* DS_FLAG_DEFERRED_ERROR: rewrites error buffers that are in deferred form (holding v) to
 * delta = v - Q[v] in place and marks them as plain for the next call.  delta [n,
 * delta_row_stride] and delta_s [d] are the buffers given to the last ds_worker_compress /
 * ds_server_aggregate_compress; either may be NULL to leave that side alone.  A no-op
 * (DS_OK) for buffers already in plain form and for contexts without the flag. */
ds_status_t ds_materialize_error(ds_ctx_t *ctx, float *delta, int64_t delta_row_stride,
                                 float *delta_s, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): ds_worker_compress for DS_COMP_SIGN with
 * DS_SCALE_WHOLE (one scale per row), without a context.  It calls no allocating routine.  The
 * per-tile fp64 partial sums that a context would hold live in a fixed array inside the
 * library, 512 KiB on every device the library runs on, held until the process ends; its
 * device address is looked up on the first call on a device (make that call outside a
 * capture).  Limit: n * ceil(d / 2048) <= 65536, beyond it DS_ERR_SHAPE.
 *   flags       0 or DS_FLAG_SIGN_RMS (anything else: DS_ERR_CONFIG)
 *   g, delta    as for ds_worker_compress
 *   sign_words  [n, ceil(d/64)]   scales [n]     (the SIGN message, layout above)
 * Results equal those of ds_worker_compress on a context with the same configuration.  Every
 * call on one device uses the same array (nothing in it needs clearing: each call writes
 * what it reads), so calls that overlap on one device, on any streams, race; calls on one
 * stream are ordered. */
ds_status_t ds_worker_compress_sign_noalloc(int32_t n, int64_t d, int32_t grad_dtype, int32_t flags,
                                            const void *g, int64_t g_row_stride, float *delta,
                                            int64_t delta_row_stride, uint64_t *sign_words,
                                            float *scales, void *hip_stream);

/* Asynchronous failures.  The step calls only enqueue work; the one failure a kernel of this
 * library can meet after its call has returned DS_OK is a TOPK single launch that gives up a
 * bounded wait (see DS_FLAG_TOPK_MULTI_LAUNCH).  ds_status returns DS_ERR_DEVICE from then on
 * (it reads a word in host memory and neither launches nor synchronises: synchronise the
 * stream first to learn about the calls enqueued so far), DS_OK otherwise and for every other
 * compressor.  The first ds_worker_compress / ds_server_aggregate_compress(_update) call after
 * the failure does none of its own work: it enqueues the reset of the context's scratch state on
 * its stream, switches the context to the chain of launches for good, lowers the flag and
 * returns DS_ERR_DEVICE.  Every later call works.  What the failed call left in its error
 * buffer and message is undefined (rows that finished are complete): restore them from the
 * caller's last good copy.  A captured graph that contains a failed single launch must be
 * captured again after that call. */
ds_status_t ds_status(const ds_ctx_t *ctx);

/* Measurement aid, not part of the method: copies `bytes` (a multiple of 16, at most 2^40) of
 * device memory with the plain streaming kernel the dense passes are shaped like (one
 * non-temporal 128-bit load and one such store per thread, 512 threads per workgroup).  Its
 * rate is the practical HBM ceiling that the benchmark reports beside the 8 TB/s peak.  src and
 * dst: 16-byte aligned device pointers, not overlapping. */
ds_status_t ds_probe_copy(const void *src, void *dst, size_t bytes, void *hip_stream);

/* Static string for a status code. */
const char *ds_status_string(ds_status_t s);

/* Library version, "major.minor". */
const char *ds_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DS_H_ */
