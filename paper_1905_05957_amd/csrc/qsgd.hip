#include "ds_internal.h"
ds_status_t ds_qsgd_worker(ds_ctx *, uint64_t, const void *, int64_t, float *, int64_t, const ds_payload_t *, hipStream_t) { return DS_ERR_UNSUPPORTED; }
ds_status_t ds_qsgd_server(ds_ctx *, uint64_t, const ds_payload_t *, float *, const ds_payload_t *, hipStream_t) { return DS_ERR_UNSUPPORTED; }
ds_status_t ds_qsgd_update(ds_ctx *, const ds_payload_t *, float *, float *, float, float, hipStream_t) { return DS_ERR_UNSUPPORTED; }
ds_status_t ds_qsgd_decode(ds_ctx *, const ds_payload_t *, int32_t, float *, hipStream_t) { return DS_ERR_UNSUPPORTED; }
