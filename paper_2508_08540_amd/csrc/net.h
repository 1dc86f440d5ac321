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
