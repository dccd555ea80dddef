// Worker gradients of the fully connected ReLU network (supplement,
// "Simulation details"): placeholder until the MFMA path lands.
#include "laq_internal.h"

namespace laq {

size_t mlp_workspace_bytes(const laq_ctx*, int64_t) { return 256; }

int mlp_worker_grads(laq_ctx* ctx, const float*, float*) {
  return set_error(ctx, LAQ_ESTATE, "MLP gradients are not built into this library yet");
}

}  // namespace laq
