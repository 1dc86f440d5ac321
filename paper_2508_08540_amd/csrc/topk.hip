// Deterministic loss-based top-k selection (Section 4.2): the k highest-loss samples in rank order.
//
// Every loss is mapped to a 64-bit sort word whose unsigned order is the selection order:
//   high 32 bits: the float's bits made monotone (sign flip), with -0 folded into +0 and every
//                 NaN folded into the largest word, so NaN ranks above +inf;
//   low 32 bits:  ~index, so that among equal losses the smaller index is the larger word.
// All words are distinct, hence exactly one result is correct and no stability argument is needed.
//
// Small pools (N <= TOPK_LDS_MAX) are sorted by one workgroup entirely in LDS with a bitonic
// network.  Larger pools take a multi-workgroup path: radix-select of the k-th word, ordered
// compaction of the selected words, and an LSD radix sort of those k words.
#include "common.h"

#define TOPK_LDS_MAX 16384
#define TOPK_THREADS 1024

__device__ __forceinline__ uint32_t loss_key(float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0xffffffffu;  // NaN: above +inf
    if (u == 0x80000000u) u = 0u;                              // -0 == +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t sort_word(float v, uint32_t idx) {
    return ((uint64_t)loss_key(v) << 32) | (uint64_t)(~idx);
}

// One workgroup; M = power of two >= N words in LDS; sorts descending.
__global__ __launch_bounds__(TOPK_THREADS) void topk_lds_bitonic_kernel(const float* __restrict__ losses, int N, int k,
                                                                        int M, int32_t* __restrict__ idx_out,
                                                                        float* __restrict__ val_out) {
    extern __shared__ uint64_t words[];
    const int tid = threadIdx.x;
    for (int i = tid; i < M; i += TOPK_THREADS) words[i] = i < N ? sort_word(losses[i], (uint32_t)i) : 0ull;
    __syncthreads();
    for (int size = 2; size <= M; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < (M >> 1); t += TOPK_THREADS) {
                int lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                int hi = lo | stride;
                bool descending = (lo & size) == 0;
                uint64_t a = words[lo], b = words[hi];
                if ((a < b) == descending) {
                    words[lo] = b;
                    words[hi] = a;
                }
            }
            __syncthreads();
        }
    }
    for (int r = tid; r < k; r += TOPK_THREADS) {
        uint32_t idx = ~(uint32_t)(words[r] & 0xffffffffull);
        idx_out[r] = (int32_t)idx;
        if (val_out) val_out[r] = losses[idx];
    }
}

size_t topk_scratch_bytes(int64_t N, int64_t k) {
    (void)N;
    (void)k;
    return 0;
}

int launch_topk(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out) {
    if (N <= TOPK_LDS_MAX) {
        int M = 2;
        while (M < N) M <<= 1;
        size_t lds = (size_t)M * sizeof(uint64_t);
        if (lds > ctx->max_lds) return bls_fail(ctx, BLS_EUNSUPPORTED, "top-k needs %zu bytes of LDS, device allows %zu", lds, ctx->max_lds);
        if (lds > 65536)
            BLS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(topk_lds_bitonic_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(topk_lds_bitonic_kernel, dim3(1), dim3(TOPK_THREADS), lds, ctx->stream, losses, (int)N, (int)k,
                           M, idx_out, val_out);
        BLS_HIP(ctx, hipGetLastError());
        return BLS_OK;
    }
    return bls_fail(ctx, BLS_EUNSUPPORTED, "top-k for N > %d is not built yet", TOPK_LDS_MAX);
}
