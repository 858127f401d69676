// placeholder until the configuration-evaluation kernels land
#include "kvp_common.h"
extern "C" size_t kvp_eval_workspace_bytes(int64_t, int64_t, int64_t, int64_t, int64_t, int32_t) { return 0; }
extern "C" int32_t kvp_eval_configs(const kvp_view*, const kvp_view*, const kvp_view*, const kvp_config*, int32_t,
                                    float*, float*, void*, size_t, void*) {
  return KVP_ERR_UNSUPPORTED;
}
