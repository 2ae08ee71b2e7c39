// Softmax-GGN operator (placeholder until the MFMA kernels land).
#include "fosi_internal.h"

namespace fosi {

fosi_status ggn_prepare(fosi_hvp* op) { return fail(op->ctx, FOSI_ERR_INVALID_ARG, "softmax-GGN operator not built yet"); }
fosi_status ggn_apply(fosi_hvp* op, const float*, float*) { return fail(op->ctx, FOSI_ERR_INVALID_ARG, "softmax-GGN operator not built yet"); }
void ggn_release(fosi_hvp*) {}

}  // namespace fosi
