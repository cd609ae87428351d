#include "ds_internal.h"
ds_status_t ds_topk_init(ds_ctx *) { return DS_OK; }
void ds_topk_fini(ds_ctx *) {}
ds_status_t ds_topk_worker(ds_ctx *, const void *, int64_t, float *, int64_t, const ds_payload_t *, hipStream_t) { return DS_ERR_UNSUPPORTED; }
ds_status_t ds_topk_server(ds_ctx *, const ds_payload_t *, float *, const ds_payload_t *, hipStream_t) { return DS_ERR_UNSUPPORTED; }
ds_status_t ds_topk_update(ds_ctx *, const ds_payload_t *, float *, float *, float, float, hipStream_t) { return DS_ERR_UNSUPPORTED; }
ds_status_t ds_topk_decode(ds_ctx *, const ds_payload_t *, int32_t, float *, hipStream_t) { return DS_ERR_UNSUPPORTED; }
