// MLP gradients (placeholder until the MFMA path lands).
#include "cada_internal.h"

namespace cada {
size_t mlp_workspace_bytes(const cada_config *, const int64_t) { set_error("MLP model not built yet"); return 0; }
int mlp_plan(Ctx *, const cada_config *, char *, size_t *, int64_t) { set_error("MLP model not built yet"); return CADA_EUNSUPPORTED; }
int mlp_init_state(Ctx *, const float *) { return CADA_EUNSUPPORTED; }
int mlp_gradients(Ctx *, const int32_t *) { set_error("MLP model not built yet"); return CADA_EUNSUPPORTED; }
void mlp_free(Ctx *) {}
}  // namespace cada
