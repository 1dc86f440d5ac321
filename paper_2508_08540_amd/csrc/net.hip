#include "net.h"

int net_score(bls_ctx* ctx, const bls_model*, const float*, const float*, const float*, const int32_t*, int64_t, float*) {
    return bls_fail(ctx, BLS_EUNSUPPORTED, "score_losses is not built yet");
}
int net_local_step(bls_ctx* ctx, const bls_model*, float*, float*, float*, const float*, const int32_t*, int64_t,
                   const int32_t*, int64_t, int64_t, int64_t, const bls_sgd&, float*) {
    return bls_fail(ctx, BLS_EUNSUPPORTED, "local_step is not built yet");
}
void net_release(bls_ctx*) {}
