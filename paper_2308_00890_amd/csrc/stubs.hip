// Entry points declared in tango.h whose kernels have not landed yet.
#include "internal.hip.h"
extern "C" {
size_t tango_qgemm_workspace_bytes(int64_t, int64_t, int64_t) { return 256; }
int tango_qgemm(int64_t, int64_t, int64_t, const float *, const float *, int, uint64_t, uint64_t, uint64_t, int8_t *, float *, int8_t *, float *, float *, float *, void *, size_t, void *) { return TANGO_ERR_UNSUPPORTED; }
size_t tango_qgemm_bwd_workspace_bytes(int64_t, int64_t, int64_t) { return 256; }
int tango_qgemm_bwd(int64_t, int64_t, int64_t, const int8_t *, const float *, const int8_t *, const float *, const float *, int, uint64_t, uint64_t, const float *, int8_t *, float *, float *, float *, void *, size_t, void *) { return TANGO_ERR_UNSUPPORTED; }
int tango_head_proj(int64_t, int, int, const float *, const float *, const float *, float *, float *, float *, float *, void *) { return TANGO_ERR_UNSUPPORTED; }
size_t tango_head_proj_bwd_workspace_bytes(int64_t, int, int) { return 256; }
int tango_head_proj_bwd(int64_t, int, int, const float *, const float *, const float *, const float *, const int8_t *, const float *, const float *, float *, float *, float *, float *, void *, size_t, void *) { return TANGO_ERR_UNSUPPORTED; }
}
