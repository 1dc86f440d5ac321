// Epoch sampler (Section 4.2; the sampling steps that open every epoch of Algorithm 1), composed on the
// device from the top-k selection: the high-loss part is a top-k of the losses, uniform sampling without
// replacement of m items is the top-m of one random key per sample, and "the rest of the data" is
// expressed by overwriting the keys of the already selected samples with -inf before that top-m.
#include "common.h"

// Copy of the caller's keys that the exclusion below writes into.  Keys are finite by contract; a key of -inf is lifted
// to the lowest finite value so that it still ranks above the struck entries and a struck sample is never drawn again.
__global__ __launch_bounds__(256) void copy_keys_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t n) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const float v = src[i];
        dst[i] = v == -INFINITY ? -3.402823466e38f : v;
    }
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

// The by-loss group takes the k highest losses, then n_biased - k by its own key from the rest; the other group takes
// n_other by its key from all N (separated) or from what the first group left (unified: the first group's picks are
// struck from the other group's keys as well).
int launch_sample_epoch(bls_ctx* ctx, const float* losses, const float* u_biased, const float* u_other, int64_t N, int64_t n_biased,
                        int64_t k, int64_t n_other, int P_biased, int P_other, bool unified, int32_t* biased_out, int32_t* other_out) {
    // scratch: the selection's own region first (it carves from the arena base), then the masked keys and the ranking
    const size_t topk_bytes = (topk_scratch_bytes(N, N) + 255) & ~size_t(255);
    Carver sizes(nullptr);
    sizes.take<float>(N);
    sizes.take<int32_t>(N);
    sizes.take<int32_t>(N);
    int rc = bls_arena_reserve(ctx, topk_bytes + sizes.off);
    if (rc != BLS_OK) return rc;
    Carver c(ctx->arena + topk_bytes);
    float* keys = c.take<float>(N);
    int32_t* ranked = c.take<int32_t>(N);
    int32_t* ranked_other = c.take<int32_t>(N);
    hipStream_t s = ctx->stream;
    if (n_biased > 0) {
        if (k > 0) {
            rc = launch_topk(ctx, losses, N, k, ranked, nullptr);
            if (rc != BLS_OK) return rc;
        }
        if (n_biased > k) {
            const float* from = u_biased;   // nothing to strike when no sample was taken by loss
            if (k > 0) {
                hipLaunchKernelGGL(copy_keys_kernel, dim3(blocks_for(N)), dim3(256), 0, s, u_biased, keys, N);
                hipLaunchKernelGGL(exclude_selected_kernel, dim3(blocks_for(k)), dim3(256), 0, s, ranked, k, keys);
                from = keys;
            }
            rc = launch_topk(ctx, from, N, n_biased - k, ranked + k, nullptr);
            if (rc != BLS_OK) return rc;
        }
        hipLaunchKernelGGL(deal_kernel, dim3(blocks_for(n_biased)), dim3(256), 0, s, ranked, n_biased, P_biased, biased_out);
    }
    if (n_other > 0) {
        const float* from = u_other;
        if (unified && n_biased > 0) {
            hipLaunchKernelGGL(copy_keys_kernel, dim3(blocks_for(N)), dim3(256), 0, s, u_other, keys, N);
            hipLaunchKernelGGL(exclude_selected_kernel, dim3(blocks_for(n_biased)), dim3(256), 0, s, ranked, n_biased, keys);
            from = keys;
        }
        rc = launch_topk(ctx, from, N, n_other, ranked_other, nullptr);
        if (rc != BLS_OK) return rc;
        hipLaunchKernelGGL(deal_kernel, dim3(blocks_for(n_other)), dim3(256), 0, s, ranked_other, n_other, P_other, other_out);
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
