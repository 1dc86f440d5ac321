// Classifier head: (average pooling) + linear layer + per-sample softmax cross-entropy, one
// wavefront per sample with shuffle reductions; and the head's weight gradient.
#include "kernels.h"

#define HEAD_MAX_C 64
#define HEAD_MAX_F_PER_LANE 16

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__global__ __launch_bounds__(64) void head_forward_kernel(const float* __restrict__ act, int positions, int F,
                                                          const float* __restrict__ W, const float* __restrict__ bias,
                                                          int C, const int32_t* __restrict__ y, float* __restrict__ loss,
                                                          float* __restrict__ feat, float* __restrict__ dlogits,
                                                          float* __restrict__ dfeat, float grad_scale, int relu_mask) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int per_lane = (F + 63) / 64;
    float f[HEAD_MAX_F_PER_LANE];
    const float inv_pos = 1.f / (float)positions;
    const float* a = act + (int64_t)b * positions * F;
    for (int i = 0; i < per_lane; ++i) {
        int c = lane + 64 * i;
        float acc = 0.f;
        if (c < F)
            for (int p = 0; p < positions; ++p) acc += a[(int64_t)p * F + c];
        f[i] = acc * inv_pos;
        if (feat && c < F) feat[(int64_t)b * F + c] = f[i];
    }
    // logits: every lane ends up with all C values (C <= 64), kept by lane c in z_mine
    float z_mine = -INFINITY;
    for (int c = 0; c < C; ++c) {
        float part = 0.f;
        for (int i = 0; i < per_lane; ++i) {
            int k = lane + 64 * i;
            if (k < F) part = __fmaf_rn(f[i], W[(int64_t)c * F + k], part);
        }
        float z = wave_sum(part) + bias[c];
        if (lane == c) z_mine = z;
    }
    float m = z_mine;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    float e = lane < C ? expf(z_mine - m) : 0.f;
    float sum = wave_sum(e);
    const int label = y[b];
    float z_label = __shfl(z_mine, label, 64);
    if (lane == 0) loss[b] = (m + logf(sum)) - z_label;
    if (!dlogits) return;
    float dz = lane < C ? (e / sum - (lane == label ? 1.f : 0.f)) * grad_scale : 0.f;
    if (lane < C) dlogits[(int64_t)b * C + lane] = dz;
    if (!dfeat) return;
    for (int i = 0; i < per_lane; ++i) {
        int k = lane + 64 * i;
        float acc = 0.f;
        for (int c = 0; c < C; ++c) {
            float d = __shfl(dz, c, 64);
            if (k < F) acc = __fmaf_rn(d, W[(int64_t)c * F + k], acc);
        }
        if (k < F) {
            acc *= inv_pos;
            if (relu_mask && !(f[i] > 0.f)) acc = 0.f;
            dfeat[(int64_t)b * F + k] = acc;
        }
    }
}

void launch_head_forward(hipStream_t s, const float* act, int B, int positions, int F, const float* W, const float* bias,
                         int C, const int32_t* y, float* loss, float* feat, float* dlogits, float* dfeat,
                         float grad_scale, bool relu_mask) {
    hipLaunchKernelGGL(head_forward_kernel, dim3(B), dim3(64), 0, s, act, positions, F, W, bias, C, y, loss, feat, dlogits,
                       dfeat, grad_scale, relu_mask ? 1 : 0);
}

__global__ __launch_bounds__(256) void head_wgrad_kernel(const float* __restrict__ dlogits, const float* __restrict__ feat,
                                                         int B, int C, int F, float* __restrict__ dW, float* __restrict__ db) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < C * F) {
        int c = i / F, k = i - c * F;
        float acc = 0.f;
        for (int b = 0; b < B; ++b) acc = __fmaf_rn(dlogits[(int64_t)b * C + c], feat[(int64_t)b * F + k], acc);
        dW[i] = acc;
    } else if (i < C * F + C) {
        int c = i - C * F;
        float acc = 0.f;
        for (int b = 0; b < B; ++b) acc += dlogits[(int64_t)b * C + c];
        db[c] = acc;
    }
}

void launch_head_wgrad(hipStream_t s, const float* dlogits, const float* feat, int B, int C, int F, float* dW, float* db) {
    int total = C * F + C;
    hipLaunchKernelGGL(head_wgrad_kernel, dim3((total + 255) / 256), dim3(256), 0, s, dlogits, feat, B, C, F, dW, db);
}
