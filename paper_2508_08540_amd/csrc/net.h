// Network passes behind score_losses and local_step.
#pragma once
#include "common.h"
#include "model.h"

int net_score(bls_ctx* ctx, const bls_model* m, const float* params, const float* buffers, const float* x,
              const int32_t* y, int64_t N, float* losses_out);
int net_local_step(bls_ctx* ctx, const bls_model* m, float* params, float* buffers, float* momentum, const float* x_pool,
                   const int32_t* y_pool, int64_t N, const int32_t* sel, int64_t k, int64_t batch, int64_t tau,
                   const bls_sgd& opt, float* step_losses_out);
void net_release(bls_ctx* ctx);
// The local steps of all workers of a communication round in one launch per layer (networks for which
// net_round_batched_covers): every worker with tau > 0 starts from the global model, trains as in net_local_step and
// leaves its replica, running statistics and momentum in its own storage; the losses of worker number t (counting the
// workers that take a step, in the order given) go to losses_out + loss_off[t] when losses_out is given.
bool net_round_batched_covers(const bls_model* m);
int net_round_batched(bls_ctx* ctx, const bls_model* m, const float* global_params, const float* global_buffers, const bls_worker* workers, int P,
                      const float* x_pool, const int32_t* y_pool, int64_t batch, const bls_sgd& opt, float* losses_out, const int64_t* loss_off);
// the same two passes for the wide residual network (net_wrn.hip)
int wrn_score(bls_ctx* ctx, const bls_model* m, const float* params, const float* buffers, const float* x, const int32_t* y, int64_t N,
              float* losses_out);
int wrn_local_step(bls_ctx* ctx, const bls_model* m, float* params, float* buffers, float* momentum, const float* x_pool,
                   const int32_t* y_pool, int64_t N, const int32_t* sel, int64_t k, int64_t batch, int64_t tau, const bls_sgd& opt,
                   float* step_losses_out);
// the same two passes for the transformer encoder (net_seq.hip); x holds int32 token ids [N][L], y the targets [N][L]
int seq_score(bls_ctx* ctx, const bls_model* m, const float* params, const int32_t* x, const int32_t* y, int64_t N, float* losses_out);
int seq_local_step(bls_ctx* ctx, const bls_model* m, float* params, float* momentum, const int32_t* x_pool, const int32_t* y_pool, int64_t N,
                   const int32_t* sel, int64_t k, int64_t batch, int64_t tau, const bls_sgd& opt, float* step_losses_out);
// Scratch the context grows to for local_step at batch size n (train) or for score_losses over a pool of n samples
size_t net_workspace_bytes(const bls_model* m, int64_t n, bool train);
size_t wrn_workspace_bytes(const bls_model* m, int64_t n, bool train);
size_t seq_workspace_bytes(const bls_model* m, int64_t n, bool train);
