#include "dbw_internal.h"
size_t dbw_mlp_scratch_floats(const dbw_ctx *) { return 1; }
int dbw_launch_grad_mlp(dbw_ctx *, const float *, const float *, const int32_t *, float *, float *, hipStream_t) { return DBW_ERR_UNSUPPORTED; }
