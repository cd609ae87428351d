// C-ABI of libds_hip.so: argument validation and dispatch to the per-compressor kernels.
// The three step calls are the three blocks of Algorithm 1 of the DoubleSqueeze paper.
#include "ds_internal.h"

#include <new>

namespace {

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

ds_status_t check_payload(const ds_ctx *c, const ds_payload_t *p)
{
    if (!p) return DS_ERR_NULL;
    switch (c->cfg.comp) {
    case DS_COMP_IDENTITY:
        if (!p->dense) return DS_ERR_NULL;
        if (misaligned(p->dense)) return DS_ERR_ALIGN;
        break;
    case DS_COMP_SIGN:
        if (!p->sign_words || !p->scales) return DS_ERR_NULL;
        if (misaligned(p->sign_words) || misaligned(p->scales)) return DS_ERR_ALIGN;
        break;
    case DS_COMP_TOPK:
        if (!p->pairs) return DS_ERR_NULL;
        if (misaligned(p->pairs)) return DS_ERR_ALIGN;
        break;
    case DS_COMP_QSGD:
        if (!p->sign_words || !p->scales || !p->levels) return DS_ERR_NULL;
        if (misaligned(p->sign_words) || misaligned(p->scales) || misaligned(p->levels)) return DS_ERR_ALIGN;
        break;
    case DS_COMP_CLIP:
        if (!p->levels) return DS_ERR_NULL;
        if (misaligned(p->levels)) return DS_ERR_ALIGN;
        break;
    case DS_COMP_RSPARSE:
        if (!p->sign_words || !p->dense) return DS_ERR_NULL;
        if (misaligned(p->sign_words) || misaligned(p->dense)) return DS_ERR_ALIGN;
        break;
    case DS_COMP_TERNARY:
        if (!p->sign_words || !p->scales || !p->levels) return DS_ERR_NULL;
        if (misaligned(p->sign_words) || misaligned(p->scales) || misaligned(p->levels)) return DS_ERR_ALIGN;
        break;
    }
    return DS_OK;
}

// The server's message: the compressor's, or with DS_FLAG_SERVER_IDENTITY the dense average
// (`need_dense` = false: the member may be missing, for the one-call server-and-update).
ds_status_t check_server_payload(const ds_ctx *c, const ds_payload_t *p, bool need_dense = true)
{
    if (!c->sid) return check_payload(c, p);
    if (!p) return DS_ERR_NULL;
    if (!p->dense) return need_dense ? DS_ERR_NULL : DS_OK;
    return misaligned(p->dense) ? DS_ERR_ALIGN : DS_OK;
}

// Binds the calling thread to the context's device for the duration of a call.
struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
        dev_ = dev;
    }
    ~DeviceGuard()
    {
        if (ok && prev != dev_) (void)hipSetDevice(prev);
    }
    int dev_ = -1;
};

}  // namespace

extern "C" {

const char *ds_status_string(ds_status_t s)
{
    switch (s) {
    case DS_OK: return "ok";
    case DS_ERR_NULL: return "a required pointer is NULL";
    case DS_ERR_SHAPE: return "shape out of range";
    case DS_ERR_CONFIG: return "inconsistent configuration";
    case DS_ERR_ALIGN: return "base pointer not 16-byte aligned";
    case DS_ERR_UNSUPPORTED: return "not supported";
    case DS_ERR_DEVICE: return "HIP runtime error";
    }
    return "unknown status";
}

const char *ds_version(void) { return "0.1"; }

ds_status_t ds_create(const ds_config_t *cfg, ds_ctx_t **out)
{
    if (!cfg || !out) return DS_ERR_NULL;
    *out = nullptr;
    if (cfg->n < 1 || cfg->n > 65535) return DS_ERR_SHAPE;
    if (cfg->d < 1 || cfg->d > 0x7FFFFFFFLL) return DS_ERR_SHAPE;
    if (cfg->grad_dtype != DS_F32 && cfg->grad_dtype != DS_BF16) return DS_ERR_CONFIG;
    switch (cfg->comp) {
    case DS_COMP_IDENTITY:
        break;
    case DS_COMP_SIGN:
        if (cfg->scale_mode == DS_SCALE_SEGMENTS) {
            if (!cfg->seg_offsets) return DS_ERR_NULL;
            if (cfg->n_seg < 1) return DS_ERR_CONFIG;
            if (cfg->seg_offsets[0] != 0 || cfg->seg_offsets[cfg->n_seg] != cfg->d) return DS_ERR_CONFIG;
            for (int32_t s = 0; s < cfg->n_seg; ++s)
                if (cfg->seg_offsets[s + 1] <= cfg->seg_offsets[s]) return DS_ERR_CONFIG;
        } else if (cfg->scale_mode == DS_SCALE_CHUNK) {
            if (cfg->chunk < 1) return DS_ERR_CONFIG;
        } else if (cfg->scale_mode != DS_SCALE_WHOLE) {
            return DS_ERR_CONFIG;
        }
        break;
    case DS_COMP_TOPK:
        if (cfg->k < 1 || cfg->k > cfg->d) return DS_ERR_SHAPE;
        if (cfg->topk_max_workgroups < 0 || cfg->topk_spin_limit < -1) return DS_ERR_CONFIG;
        break;
    case DS_COMP_QSGD:
        if (cfg->bucket < 64 || cfg->bucket % 64 != 0) return DS_ERR_CONFIG;
        if (cfg->levels < 1 || cfg->levels > 15) return DS_ERR_CONFIG;
        if (cfg->bucket > 2048 || (cfg->bucket & (cfg->bucket - 1)) != 0) return DS_ERR_UNSUPPORTED;
        break;
    case DS_COMP_CLIP:
        if (cfg->levels < 1 || cfg->levels > 31) return DS_ERR_CONFIG;
        break;
    case DS_COMP_RSPARSE:
        if (cfg->k < 1 || cfg->k > (1 << 24)) return DS_ERR_CONFIG;
        break;
    case DS_COMP_TERNARY:
        break;
    default:
        return DS_ERR_CONFIG;
    }
    {
        const bool nofb = (cfg->flags & DS_FLAG_NO_ERROR_FEEDBACK) != 0, sid = (cfg->flags & DS_FLAG_SERVER_IDENTITY) != 0;
        if ((nofb || sid) && (cfg->comp == DS_COMP_IDENTITY || cfg->comp == DS_COMP_RSPARSE)) return DS_ERR_UNSUPPORTED;
        if (cfg->comp == DS_COMP_TERNARY && !(nofb && sid)) return DS_ERR_UNSUPPORTED;
        if (cfg->comp == DS_COMP_TOPK && nofb && !(sid && cfg->grad_dtype == DS_F32)) return DS_ERR_UNSUPPORTED;
    }
    ds_ctx *c = new (std::nothrow) ds_ctx();
    if (!c) return DS_ERR_DEVICE;
    c->cfg = *cfg;  // cfg.seg_offsets (host) is read by ds_sign_init and cleared after it
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return DS_ERR_DEVICE; }
    c->W = (cfg->d + 63) / 64;
    c->n_tiles = (cfg->d + 2047) / 2048;
    c->S = 0;
    c->inv_n = 1.0f / static_cast<float>(cfg->n);
    c->nofb = (cfg->flags & DS_FLAG_NO_ERROR_FEEDBACK) != 0;
    c->sid = (cfg->flags & DS_FLAG_SERVER_IDENTITY) != 0;
    c->topk = nullptr;
    c->rs = nullptr;
    c->tern = nullptr;
    c->sign_tb_mem = nullptr;
    c->sign_partials = nullptr;
    ds_status_t rc = DS_OK;
    if (cfg->comp == DS_COMP_SIGN) {
        rc = ds_sign_init(c);
    } else if (cfg->comp == DS_COMP_QSGD) {
        c->S = (cfg->d + cfg->bucket - 1) / cfg->bucket;
    } else if (cfg->comp == DS_COMP_TOPK) {
        rc = ds_topk_init(c);
    } else if (cfg->comp == DS_COMP_RSPARSE) {
        rc = ds_rsparse_init(c);
    } else if (cfg->comp == DS_COMP_TERNARY) {
        c->S = 1;
        rc = ds_ternary_init(c);
    }
    c->cfg.seg_offsets = nullptr;
    if (rc != DS_OK) {
        ds_destroy(c);
        return rc;
    }
    *out = c;
    return DS_OK;
}

ds_status_t ds_destroy(ds_ctx_t *c)
{
    if (!c) return DS_OK;
    DeviceGuard guard(c->device);
    ds_sign_fini(c);
    ds_topk_fini(c);
    ds_rsparse_fini(c);
    ds_ternary_fini(c);
    delete c;
    return DS_OK;
}

ds_status_t ds_status(const ds_ctx_t *c)
{
    if (!c) return DS_ERR_NULL;
    return (c->cfg.comp == DS_COMP_TOPK) ? ds_topk_status(c) : DS_OK;
}

ds_status_t ds_payload_sizes(const ds_ctx_t *c, int32_t rows, size_t bytes_out[5])
{
    if (!c || !bytes_out) return DS_ERR_NULL;
    if (rows < 1) return DS_ERR_SHAPE;
    const size_t r = static_cast<size_t>(rows), d = static_cast<size_t>(c->cfg.d);
    for (int i = 0; i < 5; ++i) bytes_out[i] = 0;
    switch (c->cfg.comp) {
    case DS_COMP_IDENTITY:
        bytes_out[4] = r * d * sizeof(float);
        break;
    case DS_COMP_SIGN:
        bytes_out[0] = r * static_cast<size_t>(c->W) * sizeof(uint64_t);
        bytes_out[1] = r * static_cast<size_t>(c->S) * sizeof(float);
        break;
    case DS_COMP_TOPK:
        bytes_out[3] = r * static_cast<size_t>(c->cfg.k) * sizeof(ds_pair_t);
        break;
    case DS_COMP_QSGD:
        bytes_out[0] = r * static_cast<size_t>(c->W) * sizeof(uint64_t);
        bytes_out[1] = r * static_cast<size_t>(c->S) * sizeof(float);
        bytes_out[2] = r * ((d + 1) / 2);
        break;
    case DS_COMP_CLIP:
        bytes_out[2] = r * d * static_cast<size_t>(ds_clip_bytes(c->cfg.levels));
        break;
    case DS_COMP_RSPARSE:
        bytes_out[0] = r * static_cast<size_t>(c->W) * sizeof(uint64_t);
        bytes_out[4] = r * d * sizeof(float);
        break;
    case DS_COMP_TERNARY:
        bytes_out[0] = r * static_cast<size_t>(c->W) * sizeof(uint64_t);
        bytes_out[1] = r * sizeof(float);
        bytes_out[2] = r * static_cast<size_t>(c->W) * sizeof(uint64_t);
        break;
    }
    return DS_OK;
}

ds_status_t ds_worker_compress(ds_ctx_t *c, uint64_t step, const void *g, int64_t g_row_stride, float *delta,
                               int64_t delta_row_stride, const ds_payload_t *out, void *hip_stream)
{
    if (!c || !g) return DS_ERR_NULL;
    if (c->nofb) { delta = nullptr; delta_row_stride = c->cfg.d; }   // no error buffer in this mode
    else if (!delta) return DS_ERR_NULL;
    ds_status_t rc = check_payload(c, out);
    if (rc != DS_OK) return rc;
    if (g_row_stride < c->cfg.d || delta_row_stride < c->cfg.d) return DS_ERR_SHAPE;
    if (misaligned(g) || misaligned(delta)) return DS_ERR_ALIGN;
    DeviceGuard guard(c->device);
    if (!guard.ok) return DS_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    switch (c->cfg.comp) {
    case DS_COMP_IDENTITY: return ds_identity_worker(c, g, g_row_stride, delta, delta_row_stride, out, st);
    case DS_COMP_SIGN: return ds_sign_worker(c, g, g_row_stride, delta, delta_row_stride, out, st);
    case DS_COMP_TOPK: return ds_topk_worker(c, g, g_row_stride, delta, delta_row_stride, out, st);
    case DS_COMP_QSGD: return ds_qsgd_worker(c, step, g, g_row_stride, delta, delta_row_stride, out, st);
    case DS_COMP_CLIP: return ds_clip_worker(c, g, g_row_stride, delta, delta_row_stride, out, st);
    case DS_COMP_RSPARSE: return ds_rsparse_worker(c, step, g, g_row_stride, delta, delta_row_stride, out, st);
    case DS_COMP_TERNARY: return ds_ternary_worker(c, step, g, g_row_stride, out, st);
    }
    return DS_ERR_CONFIG;
}

// Server that does not compress: one kernel per compressor decodes, averages, writes and updates.
static ds_status_t server_identity(ds_ctx *c, const ds_payload_t *in, float *dense_out, ds_update_args u, hipStream_t st)
{
    switch (c->cfg.comp) {
    case DS_COMP_SIGN: return ds_sign_server_identity(c, in, dense_out, u, st);
    case DS_COMP_TOPK: return ds_topk_server_identity(c, in, dense_out, u, st);
    case DS_COMP_QSGD: return ds_qsgd_server_identity(c, in, dense_out, u, st);
    case DS_COMP_CLIP: return ds_clip_server_identity(c, in, dense_out, u, st);
    case DS_COMP_TERNARY: return ds_ternary_server_identity(c, in, dense_out, u, st);
    default: return DS_ERR_UNSUPPORTED;
    }
}

ds_status_t ds_server_aggregate_compress(ds_ctx_t *c, uint64_t step, const ds_payload_t *in, float *delta_s,
                                         const ds_payload_t *out, void *hip_stream)
{
    if (!c) return DS_ERR_NULL;
    if (c->nofb || c->sid) delta_s = nullptr;                         // no server error in these modes
    else if (!delta_s) return DS_ERR_NULL;
    ds_status_t rc = check_payload(c, in);
    if (rc != DS_OK) return rc;
    rc = check_server_payload(c, out);
    if (rc != DS_OK) return rc;
    if (misaligned(delta_s)) return DS_ERR_ALIGN;
    DeviceGuard guard(c->device);
    if (!guard.ok) return DS_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (c->sid) return server_identity(c, in, out->dense, ds_update_args{nullptr, nullptr, 0.f, 0.f}, st);
    switch (c->cfg.comp) {
    case DS_COMP_IDENTITY: return ds_identity_server(c, in, delta_s, out, st);
    case DS_COMP_SIGN: return ds_sign_server(c, in, delta_s, out, st);
    case DS_COMP_TOPK: return ds_topk_server(c, in, delta_s, out, st);
    case DS_COMP_QSGD: return ds_qsgd_server(c, step, in, delta_s, out, st);
    case DS_COMP_CLIP: return ds_clip_server(c, in, delta_s, out, st);
    case DS_COMP_RSPARSE: return ds_rsparse_server(c, step, in, delta_s, out, st);
    case DS_COMP_TERNARY: return DS_ERR_UNSUPPORTED;                  // built with the uncompressed server only
    }
    return DS_ERR_CONFIG;
}

ds_status_t ds_apply_update(ds_ctx_t *c, const ds_payload_t *srv, float *x, float *m, float gamma, float beta,
                            void *hip_stream)
{
    if (!c || !x) return DS_ERR_NULL;
    ds_status_t rc = check_server_payload(c, srv);
    if (rc != DS_OK) return rc;
    if (misaligned(x) || (m && misaligned(m))) return DS_ERR_ALIGN;
    DeviceGuard guard(c->device);
    if (!guard.ok) return DS_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (c->sid) return ds_identity_update(c, srv, x, m, gamma, beta, st);   // the message is the dense average
    switch (c->cfg.comp) {
    case DS_COMP_IDENTITY: return ds_identity_update(c, srv, x, m, gamma, beta, st);
    case DS_COMP_SIGN: return ds_sign_update(c, srv, x, m, gamma, beta, st);
    case DS_COMP_TOPK: return ds_topk_update(c, srv, x, m, gamma, beta, st);
    case DS_COMP_QSGD: return ds_qsgd_update(c, srv, x, m, gamma, beta, st);
    case DS_COMP_CLIP: return ds_clip_update(c, srv, x, m, gamma, beta, st);
    case DS_COMP_RSPARSE: return ds_rsparse_update(c, srv, x, m, gamma, beta, st);
    case DS_COMP_TERNARY: return DS_ERR_UNSUPPORTED;
    }
    return DS_ERR_CONFIG;
}

ds_status_t ds_decompress(ds_ctx_t *c, const ds_payload_t *p, int32_t rows, int32_t row, float *dense_out,
                          void *hip_stream)
{
    if (!c || !dense_out) return DS_ERR_NULL;
    // one message under DS_FLAG_SERVER_IDENTITY with only `dense` set is the server's
    const bool server_dense = c->sid && rows == 1 && p && p->dense && !p->sign_words && !p->levels && !p->pairs;
    ds_status_t rc = server_dense ? check_server_payload(c, p) : check_payload(c, p);
    if (rc != DS_OK) return rc;
    if (rows < 1 || row < 0 || row >= rows) return DS_ERR_SHAPE;
    if (misaligned(dense_out)) return DS_ERR_ALIGN;
    DeviceGuard guard(c->device);
    if (!guard.ok) return DS_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (server_dense) return ds_identity_decode(c, p, 0, dense_out, st);
    switch (c->cfg.comp) {
    case DS_COMP_IDENTITY: return ds_identity_decode(c, p, row, dense_out, st);
    case DS_COMP_SIGN: return ds_sign_decode(c, p, row, dense_out, st);
    case DS_COMP_TOPK: return ds_topk_decode(c, p, row, dense_out, st);
    case DS_COMP_QSGD: return ds_qsgd_decode(c, p, row, dense_out, st);
    case DS_COMP_CLIP: return ds_clip_decode(c, p, row, dense_out, st);
    case DS_COMP_RSPARSE: return ds_rsparse_decode(c, p, row, dense_out, st);
    case DS_COMP_TERNARY: return ds_ternary_decode(c, p, row, dense_out, st);
    }
    return DS_ERR_CONFIG;
}

ds_status_t ds_server_aggregate_compress_update(ds_ctx_t *c, uint64_t step, const ds_payload_t *in, float *delta_s,
                                                const ds_payload_t *out, float *x, float *m, float gamma, float beta,
                                                void *hip_stream)
{
    if (!c || !x) return DS_ERR_NULL;
    if (c->nofb || c->sid) delta_s = nullptr;
    else if (!delta_s) return DS_ERR_NULL;
    ds_status_t rc = check_payload(c, in);
    if (rc != DS_OK) return rc;
    rc = check_server_payload(c, out, false);
    if (rc != DS_OK) return rc;
    if (misaligned(delta_s) || misaligned(x) || (m && misaligned(m))) return DS_ERR_ALIGN;
    if (c->sid) {
        DeviceGuard guard(c->device);
        if (!guard.ok) return DS_ERR_DEVICE;
        return server_identity(c, in, out->dense, ds_update_args{x, m, gamma, beta}, static_cast<hipStream_t>(hip_stream));
    }
    if (c->cfg.comp == DS_COMP_TOPK && !m) {
        // the kept entries of the server's message are the update: applied where they are emitted
        DeviceGuard guard(c->device);
        if (!guard.ok) return DS_ERR_DEVICE;
        return ds_topk_server(c, in, delta_s, out, static_cast<hipStream_t>(hip_stream), x, gamma);
    }
    if (c->cfg.comp == DS_COMP_RSPARSE) {
        DeviceGuard guard(c->device);
        if (!guard.ok) return DS_ERR_DEVICE;
        return ds_rsparse_server_update(c, step, in, delta_s, out, x, m, gamma, beta, static_cast<hipStream_t>(hip_stream));
    }
    if ((c->cfg.comp == DS_COMP_SIGN && c->sign_fused) || c->cfg.comp == DS_COMP_QSGD) {
        // one pass: x (and m) are updated from the registers that hold the server's message
        DeviceGuard guard(c->device);
        if (!guard.ok) return DS_ERR_DEVICE;
        hipStream_t st = static_cast<hipStream_t>(hip_stream);
        return (c->cfg.comp == DS_COMP_SIGN) ? ds_sign_server(c, in, delta_s, out, st, x, m, gamma, beta)
                                             : ds_qsgd_server(c, step, in, delta_s, out, st, x, m, gamma, beta);
    }
    rc = ds_server_aggregate_compress(c, step, in, delta_s, out, hip_stream);
    if (rc != DS_OK) return rc;
    return ds_apply_update(c, out, x, m, gamma, beta, hip_stream);
}

ds_status_t ds_materialize_error(ds_ctx_t *c, float *delta, int64_t delta_row_stride, float *delta_s, void *hip_stream)
{
    if (!c) return DS_ERR_NULL;
    if (delta && delta_row_stride < c->cfg.d) return DS_ERR_SHAPE;
    if ((delta && misaligned(delta)) || (delta_s && misaligned(delta_s))) return DS_ERR_ALIGN;
    if (c->cfg.comp != DS_COMP_SIGN) return DS_OK;   // only the sign compressor has a deferred form
    DeviceGuard guard(c->device);
    if (!guard.ok) return DS_ERR_DEVICE;
    return ds_sign_materialize(c, delta, delta_row_stride, delta_s, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
