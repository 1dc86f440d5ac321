// Classifier head: (average pooling) + linear layer + per-sample softmax cross-entropy, one
// workgroup of four wavefronts per sample with shuffle reductions; and the head's weight gradient.
#include "act.h"

#define HEAD_MAX_C 128   // two classes per lane

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Average pool, linear layer, softmax cross-entropy and their gradients for one sample per workgroup.  Lane l owns the
// channel quads l, l + 64, ... (channels 4q .. 4q+3): PQ = ceil(F / 256) of them, a template parameter so that the pooled
// features stay in registers; F % 4 == 0.  Four waves per sample (a single one leaves the compute unit nearly empty and
// spends its time waiting for one load after another): wave w pools positions w, w + 4, ..., takes classes w, w + 4, ...
// and, for the feature gradient, sums over those classes; the partial results meet in LDS and are added in wave order.
template <int PQ, typename T>
__global__ __launch_bounds__(256) void head_forward_kernel(const T* __restrict__ act, int positions, int F,
                                                               const float* __restrict__ W, const float* __restrict__ bias,
                                                               int C, const int32_t* __restrict__ y, float* __restrict__ loss,
                                                               float* __restrict__ feat, float* __restrict__ dlogits,
                                                               float* __restrict__ dfeat, float grad_scale, int relu_mask, int64_t rstride) {
    if (rstride) {   // one replica of several: every buffer sits blockIdx.z slots further
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        act = rep_at(act, ro); W = rep_at(W, ro); bias = rep_at(bias, ro); y = rep_at(y, ro); loss = rep_at(loss, ro); feat = rep_at(feat, ro);
        dlogits = rep_at(dlogits, ro); dfeat = rep_at(dfeat, ro);
    }
    __shared__ __attribute__((aligned(16))) float part[4][256 * PQ];   // per wave: pooled sums, later feature-gradient sums
    __shared__ __attribute__((aligned(16))) float fs[256 * PQ];        // pooled features
    __shared__ float zs[HEAD_MAX_C];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float inv_pos = 1.f / (float)positions;
    const T* a = act + (int64_t)b * positions * F;
#pragma unroll
    for (int i = 0; i < PQ; ++i) {
        const int c = 4 * (lane + 64 * i);
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
        if (c < F) {
            int p = wave;
            for (; p + 4 < positions; p += 8) {
                s0 += Act<T>::load4(a + (int64_t)p * F + c);
                s1 += Act<T>::load4(a + (int64_t)(p + 4) * F + c);
            }
            if (p < positions) s0 += Act<T>::load4(a + (int64_t)p * F + c);
        }
        *reinterpret_cast<f32x4*>(&part[wave][c]) = s0 + s1;
    }
    __syncthreads();
    for (int c = 4 * threadIdx.x; c < F; c += 1024) {
        const f32x4 v = ((*reinterpret_cast<const f32x4*>(&part[0][c]) + *reinterpret_cast<const f32x4*>(&part[1][c])) +
                         (*reinterpret_cast<const f32x4*>(&part[2][c]) + *reinterpret_cast<const f32x4*>(&part[3][c]))) * inv_pos;
        *reinterpret_cast<f32x4*>(&fs[c]) = v;
        if (feat) *reinterpret_cast<f32x4*>(feat + (int64_t)b * F + c) = v;
    }
    __syncthreads();
    f32x4 f[PQ];
#pragma unroll
    for (int i = 0; i < PQ; ++i) {
        const int c = 4 * (lane + 64 * i);
        f[i] = c < F ? *reinterpret_cast<const f32x4*>(&fs[c]) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int c = wave; c < C; c += 4) {
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < PQ; ++i) {
            const int k = 4 * (lane + 64 * i);
            if (k < F) {
                const f32x4 w = *reinterpret_cast<const f32x4*>(W + (int64_t)c * F + k);
#pragma unroll
                for (int j = 0; j < 4; ++j) acc = __fmaf_rn(f[i][j], w[j], acc);
            }
        }
        const float z = wave_sum(acc) + bias[c];
        if (lane == 0) zs[c] = z;
    }
    __syncthreads();
    // every wave holds the logits of classes lane and lane + 64 and works out the softmax for itself
    float z_mine[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) z_mine[h] = lane + 64 * h < C ? zs[lane + 64 * h] : -INFINITY;
    float m = fmaxf(z_mine[0], z_mine[1]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    float ex[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) ex[h] = lane + 64 * h < C ? expf(z_mine[h] - m) : 0.f;
    const float sum = wave_sum(ex[0]) + wave_sum(ex[1]);
    const int label = y[b];
    const float z_label = __shfl(label < 64 ? z_mine[0] : z_mine[1], label & 63, 64);
    if (threadIdx.x == 0) loss[b] = (m + logf(sum)) - z_label;
    if (!dlogits) return;
    float dz[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int c = lane + 64 * h;
        dz[h] = c < C ? (ex[h] / sum - (c == label ? 1.f : 0.f)) * grad_scale : 0.f;
        if (wave == 0 && c < C) dlogits[(int64_t)b * C + c] = dz[h];
    }
    if (!dfeat) return;
#pragma unroll
    for (int i = 0; i < PQ; ++i) {
        const int k = 4 * (lane + 64 * i);
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int c = wave; c < C; c += 4) {
            const float d = __shfl(c < 64 ? dz[0] : dz[1], c & 63, 64);
            if (k < F) {
                const f32x4 w = *reinterpret_cast<const f32x4*>(W + (int64_t)c * F + k);
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = __fmaf_rn(d, w[j], acc[j]);
            }
        }
        *reinterpret_cast<f32x4*>(&part[wave][k]) = acc;
    }
    __syncthreads();
    for (int c = 4 * threadIdx.x; c < F; c += 1024) {
        f32x4 v = ((*reinterpret_cast<const f32x4*>(&part[0][c]) + *reinterpret_cast<const f32x4*>(&part[1][c])) +
                   (*reinterpret_cast<const f32x4*>(&part[2][c]) + *reinterpret_cast<const f32x4*>(&part[3][c]))) * inv_pos;
        if (relu_mask) {
            const f32x4 fv = *reinterpret_cast<const f32x4*>(&fs[c]);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (!(fv[j] > 0.f)) v[j] = 0.f;
        }
        *reinterpret_cast<f32x4*>(dfeat + (int64_t)b * F + c) = v;
    }
}

void launch_head_forward(hipStream_t s, int act_type, const void* act, int B, int positions, int F, const float* W, const float* bias,
                         int C, const int32_t* y, float* loss, float* feat, float* dlogits, float* dfeat,
                         float grad_scale, bool relu_mask, Reps reps) {
#define HEAD_LAUNCH(PQ)                                                                                                     \
    ACT_DISPATCH(act_type, hipLaunchKernelGGL((head_forward_kernel<PQ, T>), dim3(B, 1, reps.n), dim3(256), 0, s, (const T*)act, positions, F, W, \
                                              bias, C, y, loss, feat, dlogits, dfeat, grad_scale, relu_mask ? 1 : 0, reps.stride))
    const int quads = (F / 4 + 63) / 64;   // F is a multiple of 16, at most 1024
    if (quads <= 1) HEAD_LAUNCH(1);
    else if (quads <= 2) HEAD_LAUNCH(2);
    else HEAD_LAUNCH(4);
#undef HEAD_LAUNCH
}

// One workgroup per class c: thread (f mod 64, slice) adds every 4th sample for its features, the four
// slices are folded through LDS in order.  db[c] comes from the same workgroup.
__global__ __launch_bounds__(256) void head_wgrad_kernel(const float* __restrict__ dlogits, const float* __restrict__ feat,
                                                         int B, int C, int F, float* __restrict__ dW, float* __restrict__ db, int64_t rstride) {
    if (rstride) {
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        dlogits = rep_at(dlogits, ro); feat = rep_at(feat, ro); dW = rep_at(dW, ro); db = rep_at(db, ro);
    }
    __shared__ float red[4][64];
    const int c = blockIdx.x, fl = threadIdx.x & 63, sl = threadIdx.x >> 6;
    for (int f0 = 0; f0 < F; f0 += 64) {
        const int f = f0 + fl;
        float acc = 0.f;
        if (f < F)
            for (int b = sl; b < B; b += 4) acc = __fmaf_rn(dlogits[(int64_t)b * C + c], feat[(int64_t)b * F + f], acc);
        red[sl][fl] = acc;
        __syncthreads();
        if (sl == 0 && f < F) dW[(int64_t)c * F + f] = (red[0][fl] + red[1][fl]) + (red[2][fl] + red[3][fl]);
        __syncthreads();
    }
    // bias gradient: 256 threads take every 256th sample
    float acc = 0.f;
    for (int b = threadIdx.x; b < B; b += 256) acc += dlogits[(int64_t)b * C + c];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (fl == 0) red[sl][0] = acc;
    __syncthreads();
    if (threadIdx.x == 0) db[c] = (red[0][0] + red[1][0]) + (red[2][0] + red[3][0]);
}

void launch_head_wgrad(hipStream_t s, const float* dlogits, const float* feat, int B, int C, int F, float* dW, float* db, Reps reps) {
    hipLaunchKernelGGL(head_wgrad_kernel, dim3(C, 1, reps.n), dim3(256), 0, s, dlogits, feat, B, C, F, dW, db, reps.stride);
}
