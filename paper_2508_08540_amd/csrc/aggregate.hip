// Bias-weighted aggregation of P parameter replicas (Section 4.3, Eq. 4): one streaming pass.
//
// HBM-bound: every replica element is read once and the result written once (optionally also
// stored back into each replica).  Each thread owns float4 columns; the P products are
// accumulated in replica order with fused multiply-adds, one rounding per term:
// acc = w_0*x_0; acc = fma(w_i, x_i, acc).
#include "common.h"

#define AGG_MAX_P 64

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct AggArgs {
    const float* src[AGG_MAX_P];
    float w[AGG_MAX_P];
};

__device__ __forceinline__ f32x4 agg_column(const AggArgs& a, int P, int64_t v) {
    f32x4 acc;
    {
        f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.src[0]) + v);
        float w = a.w[0];
        acc.x = __fmul_rn(w, x.x); acc.y = __fmul_rn(w, x.y); acc.z = __fmul_rn(w, x.z); acc.w = __fmul_rn(w, x.w);
    }
    for (int i = 1; i < P; ++i) {
        f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.src[i]) + v);
        float w = a.w[i];
        acc.x = __fmaf_rn(w, x.x, acc.x);
        acc.y = __fmaf_rn(w, x.y, acc.y);
        acc.z = __fmaf_rn(w, x.z, acc.z);
        acc.w = __fmaf_rn(w, x.w, acc.w);
    }
    return acc;
}

__global__ __launch_bounds__(256) void agg_vec4_kernel(AggArgs a, int P, int64_t n_vec, float* out,
                                                       int broadcast) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n_vec; v += stride) {
        f32x4 acc = agg_column(a, P, v);
        reinterpret_cast<f32x4*>(out)[v] = acc;
        if (broadcast)
            for (int i = 0; i < P; ++i) reinterpret_cast<f32x4*>(const_cast<float*>(a.src[i]))[v] = acc;
    }
}

// Scalar path: the tail after the last full float4, or everything when a pointer is not 16-byte aligned.
__global__ __launch_bounds__(256) void agg_scalar_kernel(AggArgs a, int P, int64_t begin, int64_t d,
                                                         float* out, int broadcast) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < d; j += stride) {
        float acc = __fmul_rn(a.w[0], a.src[0][j]);
        for (int i = 1; i < P; ++i) acc = __fmaf_rn(a.w[i], a.src[i][j], acc);
        out[j] = acc;
        if (broadcast)
            for (int i = 0; i < P; ++i) const_cast<float*>(a.src[i])[j] = acc;
    }
}

int launch_weighted_aggregate(bls_ctx* ctx, const float* const* replicas, const float* weights, int P, int64_t d,
                              float* out, bool broadcast) {
    AggArgs a;
    bool aligned = (reinterpret_cast<uintptr_t>(out) & 15) == 0;
    for (int i = 0; i < AGG_MAX_P; ++i) {
        a.src[i] = i < P ? replicas[i] : nullptr;
        a.w[i] = i < P ? weights[i] : 0.f;
        if (i < P && (reinterpret_cast<uintptr_t>(replicas[i]) & 15)) aligned = false;
    }
    int64_t n_vec = aligned ? d / 4 : 0;
    if (n_vec > 0) {
        int64_t blocks = ceil_div(n_vec, 256);
        int64_t cap = (int64_t)ctx->num_cus * 8;
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL(agg_vec4_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, a, P, n_vec, out,
                           broadcast ? 1 : 0);
    }
    int64_t begin = n_vec * 4;
    if (begin < d) {
        int64_t blocks = ceil_div(d - begin, 256);
        int64_t cap = (int64_t)ctx->num_cus * 8;
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL(agg_scalar_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, a, P, begin, d, out,
                           broadcast ? 1 : 0);
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
