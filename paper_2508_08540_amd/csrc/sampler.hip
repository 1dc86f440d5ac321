// Epoch sampler (Section 4.2; the sampling steps that open every epoch of Algorithm 1), composed on the
// device from the top-k selection: the high-loss part is a top-k of the losses, uniform sampling without
// replacement of m items is the top-m of one random key per sample, and "the rest of the data" is
// expressed by overwriting the keys of the already selected samples with -inf before that top-m.
#include "common.h"

__global__ __launch_bounds__(256) void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t n) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void exclude_selected_kernel(const int32_t* __restrict__ sel, int64_t k, float* __restrict__ keys) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < k; i += stride) keys[sel[i]] = -INFINITY;
}

// Round-robin dealing: rank r goes to worker r % P, position r / P of that worker's contiguous segment.
// The first n % P workers hold one element more.
__global__ __launch_bounds__(256) void deal_kernel(const int32_t* __restrict__ ranked, int64_t n, int P, int32_t* __restrict__ out) {
    const int64_t base = n / P, rem = n % P;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n; r += stride) {
        const int64_t p = r % P, j = r / P;
        out[p * base + (p < rem ? p : rem) + j] = ranked[r];
    }
}

static unsigned blocks_for(int64_t n) {
    int64_t b = (n + 255) / 256;
    return (unsigned)(b < 1 ? 1 : (b > 4096 ? 4096 : b));
}

int launch_sample_epoch(bls_ctx* ctx, const float* losses, const float* u_fast, const float* u_slow, int64_t N, int64_t n_fast,
                        int64_t k, int64_t n_slow, int P_f, int P_s, int32_t* fast_out, int32_t* slow_out) {
    // scratch: the selection's own region first (it carves from the arena base), then the masked keys and the ranking
    const size_t topk_bytes = (topk_scratch_bytes(N, N) + 255) & ~size_t(255);
    Carver sizes(nullptr);
    sizes.take<float>(N);
    sizes.take<int32_t>(N);
    int rc = bls_arena_reserve(ctx, topk_bytes + sizes.off);
    if (rc != BLS_OK) return rc;
    Carver c(ctx->arena + topk_bytes);
    float* keys = c.take<float>(N);
    int32_t* ranked = c.take<int32_t>(N);
    hipStream_t s = ctx->stream;
    if (n_fast > 0) {
        if (k > 0) {
            rc = launch_topk(ctx, losses, N, k, ranked, nullptr);
            if (rc != BLS_OK) return rc;
        }
        if (n_fast > k) {
            hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for(N)), dim3(256), 0, s, u_fast, keys, N);
            if (k > 0) hipLaunchKernelGGL(exclude_selected_kernel, dim3(blocks_for(k)), dim3(256), 0, s, ranked, k, keys);
            rc = launch_topk(ctx, keys, N, n_fast - k, ranked + k, nullptr);
            if (rc != BLS_OK) return rc;
        }
        hipLaunchKernelGGL(deal_kernel, dim3(blocks_for(n_fast)), dim3(256), 0, s, ranked, n_fast, P_f, fast_out);
    }
    if (n_slow > 0) {
        rc = launch_topk(ctx, u_slow, N, n_slow, ranked, nullptr);
        if (rc != BLS_OK) return rc;
        hipLaunchKernelGGL(deal_kernel, dim3(blocks_for(n_slow)), dim3(256), 0, s, ranked, n_slow, P_s, slow_out);
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
