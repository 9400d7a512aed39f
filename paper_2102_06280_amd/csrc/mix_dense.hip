// placeholder, replaced below
#include "dbw_internal.h"
int dbw_launch_mix_dense(dbw_ctx *, const float *, const float *, float *, float, hipStream_t) { return DBW_ERR_UNSUPPORTED; }
