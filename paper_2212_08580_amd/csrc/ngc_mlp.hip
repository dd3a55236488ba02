// Partition gradients of the 2-layer perceptron (placeholder until the MFMA
// route is in place: reports that the loss is not available).
#include "ngc_internal.h"

int ngc_mlp2_grads(ngc_ctx* ctx, const float*, const int*, const float*, int64_t, float*) {
    return ngc_fail(ctx, NGC_ERR_STATE, "NGC_LOSS_MLP2 is not available in this build");
}
