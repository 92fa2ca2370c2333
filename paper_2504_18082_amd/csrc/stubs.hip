// Entry points not yet implemented (removed one by one as the kernels land).
#include "cr_common.h"
#define STUB { cr::set_error("not implemented yet"); return CR_ERR_UNSUPPORTED; }
extern "C" cr_status cr_sage_padded_dims(int32_t, int32_t, int32_t *, int32_t *) STUB
extern "C" cr_status cr_sage_refresh_shadows(const cr_sage_layer *, void *) STUB
extern "C" cr_status cr_sage_linear_fwd(const cr_sage_layer *, const int32_t *, int32_t, const uint16_t *, const uint16_t *, int64_t, int, float *, uint16_t *, void *) STUB
extern "C" cr_status cr_sage_linear_bwd_workspace_bytes(int32_t, int32_t, int32_t, size_t *) STUB
extern "C" cr_status cr_sage_linear_bwd(const cr_sage_layer *, const int32_t *, int32_t, const uint16_t *, const uint16_t *, int64_t, const uint16_t *, float, float, float *, float *, float *, float *, void *, size_t, void *) STUB
extern "C" cr_status cr_softmax_xent(const int32_t *, int32_t, const float *, int64_t, int32_t, const int32_t *, const int32_t *, float *, float *, float *, uint16_t *, void *) STUB
