#include "dmt_internal.h"
extern "C" size_t dmt_tm_workspace_bytes(const dmt_plan*, const dmt_tm_params*, int64_t) { return 0; }
extern "C" dmt_status dmt_tower_module_fwd(const dmt_plan*, const dmt_tm_params*, const void*, int64_t, void*, dmt_dtype, void*, size_t, void*) { return DMT_ENOTSUP; }
