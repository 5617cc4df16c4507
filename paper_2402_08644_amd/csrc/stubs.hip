// temporary: entry points not built yet
#include "common.h"
extern "C" {
size_t tandem_project_workspace(const tandem_ff_desc*, int64_t) { return 0; }
int tandem_project(const tandem_ff_desc*, const void*, void*, int64_t, void*, size_t, void*) { return TANDEM_ERR_UNSUPPORTED; }
int tandem_model_create(const tandem_model_desc*, tandem_model**) { return TANDEM_ERR_UNSUPPORTED; }
void tandem_model_destroy(tandem_model*) {}
size_t tandem_decode_step_workspace(const tandem_model*, int32_t, int32_t) { return 0; }
int tandem_decode_step(const tandem_model*, const tandem_state_desc*, int32_t, const int32_t*, int32_t*, int32_t*,
                       const tandem_step_aux*, void*, size_t, void*) { return TANDEM_ERR_UNSUPPORTED; }
}
