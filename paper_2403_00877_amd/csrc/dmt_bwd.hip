#include "dmt_internal.h"
extern "C" size_t dmt_bwd_workspace_bytes(const dmt_plan*, int64_t, int64_t) { return 0; }
extern "C" dmt_status dmt_tower_lookup_bwd_update(const dmt_plan*, const int32_t*, const int64_t*, int64_t, int64_t, const float*, float, float, void*, size_t, void*, const dmt_bwd_debug*) { return DMT_ENOTSUP; }
