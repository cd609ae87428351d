// Host-side internals of libds_hip.so: the context and the per-compressor launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ds.h"

// Tables that map the fixed 2048-element tiles onto the scale groups of the 1-bit
// compressor when a group does not fit one workgroup (whole vector, arbitrary segments,
// odd chunk sizes).  A "piece" is a maximal run of elements inside one tile and one group;
// pieces are numbered in element order, so piece p spans [piece_start[p], piece_start[p+1]).
struct ds_sign_tables {
    // [n_tiles] {first piece, group}: group >= 0 for a tile that lies inside one group (one piece),
    // else minus the number of its pieces.  One 8-byte load tells a workgroup its pieces and, in
    // the common case, the group whose scale it needs.
    const int2 *tile_info;
    const int32_t *tile_piece_first;  // [n_tiles + 1]
    const int64_t *piece_start;       // [n_pieces + 1]
    const int32_t *piece_seg;         // [n_pieces]
    const int32_t *seg_piece_first;   // [S + 1]
    const int64_t *seg_off;           // [S + 1]
    int32_t n_pieces;
    int32_t n_seg;
    bool rms;                         // group scale = root mean square instead of mean |v|
    // whole_d > 0: one group = the whole vector of whole_d elements, piece p = tile p; none of
    // the tables above is read (they may be null)
    int64_t whole_d;
};

struct ds_topk_scratch;  // defined in topk.hip
struct ds_rs_scratch;    // defined in rsparse.hip
struct ds_tern_scratch;  // defined in ternary.hip

// What the update of Algorithm 1 needs when it rides along with a server kernel; x == nullptr:
// no update.
struct ds_update_args {
    float *x, *m;
    float gamma, beta;
};

struct ds_ctx {
    ds_config_t cfg;
    int device;
    int64_t W;        // sign words per row
    int64_t S;        // scale groups per row (SIGN) / buckets per row (QSGD)
    int64_t n_tiles;  // ceil(d / 2048)
    float inv_n;
    bool nofb;        // DS_FLAG_NO_ERROR_FEEDBACK: no error buffer is read or written
    bool sid;         // DS_FLAG_SERVER_IDENTITY: the server's message is its dense average
    // SIGN
    bool sign_fused;  // every group is one chunk handled by one workgroup
    ds_sign_tables sign_tb;
    void *sign_tb_mem;     // one device allocation behind sign_tb
    double *sign_partials; // [n, n_pieces] partial sums of |v|
    bool sign_defer;       // DS_FLAG_DEFERRED_ERROR on the two-look route
    bool sign_w_deferred;  // the worker error buffers hold v of the last call, sign_prev_w its scales
    bool sign_s_deferred;  // the same for the server's buffer and sign_prev_s
    float *sign_prev_w;    // [n, S]
    float *sign_prev_s;    // [S]
    // TOPK
    ds_topk_scratch *topk;
    // RSPARSE
    ds_rs_scratch *rs;
    // TERNARY
    ds_tern_scratch *tern;
};

#define DS_HIP_TRY(expr)                                 \
    do {                                                 \
        hipError_t e_ = (expr);                          \
        if (e_ != hipSuccess) return DS_ERR_DEVICE;      \
    } while (0)

static inline ds_status_t ds_launch_status()
{
    return hipGetLastError() == hipSuccess ? DS_OK : DS_ERR_DEVICE;
}

// Whether a d-element fp32 buffer that one call reads and writes once (the server's error, the
// model, the momentum) should pass the caches non-temporally.  Above 64 MB it should (measured
// at 500 MB); at 45 MB ordinary accesses were faster: short kernels end when their stores are
// in the write-back cache, and the buffers of one call fit the 256 MB memory-side cache.
static inline bool ds_stream_worthwhile(int64_t d)
{
    return d * 4 > (static_cast<int64_t>(64) << 20);
}

// identity.hip
ds_status_t ds_identity_worker(ds_ctx *c, const void *g, int64_t gs, float *delta, int64_t dstr,
                               const ds_payload_t *out, hipStream_t st);
ds_status_t ds_identity_server(ds_ctx *c, const ds_payload_t *in, float *delta_s,
                               const ds_payload_t *out, hipStream_t st);
ds_status_t ds_identity_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma,
                               float beta, hipStream_t st);
ds_status_t ds_identity_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st);

// sign.hip
ds_status_t ds_sign_init(ds_ctx *c);
void ds_sign_fini(ds_ctx *c);
ds_status_t ds_sign_worker(ds_ctx *c, const void *g, int64_t gs, float *delta, int64_t dstr,
                           const ds_payload_t *out, hipStream_t st);
ds_status_t ds_sign_server(ds_ctx *c, const ds_payload_t *in, float *delta_s,
                           const ds_payload_t *out, hipStream_t st, float *x = nullptr, float *m = nullptr,
                           float gamma = 0.f, float beta = 0.f);
ds_status_t ds_sign_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma,
                           float beta, hipStream_t st);
ds_status_t ds_sign_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st);
ds_status_t ds_sign_materialize(ds_ctx *c, float *delta, int64_t dstr, float *delta_s, hipStream_t st);

// Server without compression (DS_FLAG_SERVER_IDENTITY), per compressor: decodes the n messages,
// averages them by the chain from +0, writes the average to dense_out (if not null) and applies
// the update (if u.x is not null), all in one kernel.
ds_status_t ds_sign_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st);
ds_status_t ds_qsgd_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st);
ds_status_t ds_clip_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st);
ds_status_t ds_topk_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st);
ds_status_t ds_ternary_server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st);

// ternary.hip
ds_status_t ds_ternary_init(ds_ctx *c);
void ds_ternary_fini(ds_ctx *c);
ds_status_t ds_ternary_worker(ds_ctx *c, uint64_t step, const void *g, int64_t gs, const ds_payload_t *out, hipStream_t st);
ds_status_t ds_ternary_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st);

// qsgd.hip
ds_status_t ds_qsgd_worker(ds_ctx *c, uint64_t step, const void *g, int64_t gs, float *delta,
                           int64_t dstr, const ds_payload_t *out, hipStream_t st);
ds_status_t ds_qsgd_server(ds_ctx *c, uint64_t step, const ds_payload_t *in, float *delta_s,
                           const ds_payload_t *out, hipStream_t st, float *x = nullptr, float *m = nullptr,
                           float gamma = 0.f, float beta = 0.f);
ds_status_t ds_qsgd_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma,
                           float beta, hipStream_t st);
ds_status_t ds_qsgd_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st);

// clip.hip
int ds_clip_bytes(int bits);   // bytes per element of the message for `bits` cleared low bits
ds_status_t ds_clip_worker(ds_ctx *c, const void *g, int64_t gs, float *delta, int64_t dstr,
                           const ds_payload_t *out, hipStream_t st);
ds_status_t ds_clip_server(ds_ctx *c, const ds_payload_t *in, float *delta_s,
                           const ds_payload_t *out, hipStream_t st);
ds_status_t ds_clip_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma,
                           float beta, hipStream_t st);
ds_status_t ds_clip_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st);

// rsparse.hip
ds_status_t ds_rsparse_init(ds_ctx *c);
void ds_rsparse_fini(ds_ctx *c);
ds_status_t ds_rsparse_worker(ds_ctx *c, uint64_t step, const void *g, int64_t gs, float *delta,
                              int64_t dstr, const ds_payload_t *out, hipStream_t st);
ds_status_t ds_rsparse_server(ds_ctx *c, uint64_t step, const ds_payload_t *in, float *delta_s,
                              const ds_payload_t *out, hipStream_t st);
ds_status_t ds_rsparse_server_update(ds_ctx *c, uint64_t step, const ds_payload_t *in, float *delta_s,
                                     const ds_payload_t *out, float *x, float *m, float gamma, float beta,
                                     hipStream_t st);
ds_status_t ds_rsparse_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma,
                              float beta, hipStream_t st);
ds_status_t ds_rsparse_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st);

// topk.hip
ds_status_t ds_topk_init(ds_ctx *c);
void ds_topk_fini(ds_ctx *c);
ds_status_t ds_topk_status(const ds_ctx *c);
ds_status_t ds_topk_worker(ds_ctx *c, const void *g, int64_t gs, float *delta, int64_t dstr,
                           const ds_payload_t *out, hipStream_t st);
ds_status_t ds_topk_server(ds_ctx *c, const ds_payload_t *in, float *delta_s,
                           const ds_payload_t *out, hipStream_t st, float *x = nullptr, float gamma = 0.f);
ds_status_t ds_topk_update(ds_ctx *c, const ds_payload_t *srv, float *x, float *m, float gamma,
                           float beta, hipStream_t st);
ds_status_t ds_topk_decode(ds_ctx *c, const ds_payload_t *p, int32_t row, float *out, hipStream_t st);
