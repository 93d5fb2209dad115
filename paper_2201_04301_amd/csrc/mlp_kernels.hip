// MLP gradients at two iterates (placeholder until the MFMA kernels land).
#include "gcada_internal.h"

namespace gcada {
hipError_t mlp_plan(gcada_ctx*) { return hipErrorNotSupported; }
void mlp_free(gcada_ctx*) {}
hipError_t mlp_gradients(gcada_ctx*, const int32_t*, hipStream_t) { return hipErrorNotSupported; }
hipError_t mlp_refresh_weights(gcada_ctx*, hipStream_t) { return hipErrorNotSupported; }
}  // namespace gcada
