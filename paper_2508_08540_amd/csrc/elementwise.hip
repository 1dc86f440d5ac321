// Small memory-bound kernels around the contractions: batch gather, SGD update, column sums.
#include "act.h"

template <typename T>
__device__ __forceinline__ T to_act(float v);
template <>
__device__ __forceinline__ float to_act<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16_t to_act<bf16_t>(float v) { return f32_to_bf16(v); }

// One image (or row) of one replica's batch per blockIdx.y; see gather_images_kernel.
template <typename T>
__device__ __forceinline__ void gather_one(const float* __restrict__ src, const int32_t* __restrict__ y_src, int64_t img, int b, int pixels,
                                           int c_src, int c_dst, T* __restrict__ dst, int32_t* __restrict__ y_dst) {
    const float* s = src + img * pixels * c_src;
    T* d = dst + (int64_t)b * pixels * c_dst;
    int total = pixels * c_dst;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        int p = i / c_dst, c = i - p * c_dst;
        d[i] = to_act<T>(c < c_src ? s[p * c_src + c] : 0.f);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && y_dst) y_dst[b] = y_src[img];
}

// Several replicas (blockIdx.z), each with its own selection list and its own destination slot.
template <typename T>
__global__ __launch_bounds__(256) void gather_images_reps_kernel(const float* __restrict__ src, const int32_t* __restrict__ y_src, GatherReps lists,
                                                                 int64_t start, int pixels, int c_src, int c_dst, T* __restrict__ dst,
                                                                 int32_t* __restrict__ y_dst, int64_t rstride) {
    const int r = blockIdx.z, b = blockIdx.y;
    const int64_t ro = (int64_t)r * rstride;
    const int64_t img = (int64_t)lists.sel[r][(start + b) % lists.k[r]];
    gather_one<T>(src, y_src, img, b, pixels, c_src, c_dst, rep_at(dst, ro), rep_at(y_dst, ro));
}

template <typename T>
__global__ __launch_bounds__(256) void gather_images_kernel(const float* __restrict__ src, const int32_t* __restrict__ y_src,
                                                            const int32_t* __restrict__ sel, int64_t k, int64_t start,
                                                            int64_t first, int batch, int pixels, int c_src, int c_dst,
                                                            T* __restrict__ dst, int32_t* __restrict__ y_dst) {
    int b = blockIdx.y;
    int64_t img = sel ? (int64_t)sel[(start + b) % k] : first + b;
    gather_one<T>(src, y_src, img, b, pixels, c_src, c_dst, dst, y_dst);
}

void launch_gather_images(hipStream_t s, const float* src, const int32_t* y_src, const int32_t* sel, int64_t k,
                          int64_t start, int64_t first, int batch, int pixels, int c_src, int c_dst, int act, void* dst,
                          int32_t* y_dst) {
    int total = pixels * c_dst;
    int bx = (total + 255) / 256;
    if (bx > 16) bx = 16;
    ACT_DISPATCH(act, hipLaunchKernelGGL(gather_images_kernel<T>, dim3(bx, batch), dim3(256), 0, s, src, y_src, sel, k, start, first,
                                         batch, pixels, c_src, c_dst, (T*)dst, y_dst));
}

void launch_gather_images_reps(hipStream_t s, const float* src, const int32_t* y_src, const GatherReps& lists, int64_t start, int batch,
                               int pixels, int c_src, int c_dst, int act, void* dst, int32_t* y_dst, Reps reps) {
    int total = pixels * c_dst;
    int bx = (total + 255) / 256;
    if (bx > 16) bx = 16;
    ACT_DISPATCH(act, hipLaunchKernelGGL(gather_images_reps_kernel<T>, dim3(bx, batch, reps.n), dim3(256), 0, s, src, y_src, lists, start, pixels,
                                         c_src, c_dst, (T*)dst, y_dst, reps.stride));
}

void launch_gather_rows(hipStream_t s, const float* src, const int32_t* y_src, const int32_t* sel, int64_t k,
                        int64_t start, int batch, int64_t row, float* dst, int32_t* y_dst) {
    launch_gather_images(s, src, y_src, sel, k, start, 0, batch, 1, (int)row, (int)row, ACT_F32, dst, y_dst);
}

// SGD with momentum and coupled weight decay: g += wd*x; buf = mu*buf + g; x -= lr*buf.
__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ params, float* __restrict__ momentum,
                                                  const float* __restrict__ grad, int64_t d, float lr, float mu, float wd) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < d; i += stride) {
        float x = params[i];
        float g = __fmaf_rn(wd, x, grad[i]);
        float buf = __fmaf_rn(mu, momentum[i], g);
        momentum[i] = buf;
        params[i] = __fmaf_rn(-lr, buf, x);
    }
}

void launch_sgd(hipStream_t s, float* params, float* momentum, const float* grad, int64_t d, float lr, float mu,
                float wd) {
    int64_t blocks = (d + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(sgd_kernel, dim3((unsigned)blocks), dim3(256), 0, s, params, momentum, grad, d, lr, mu, wd);
}

__global__ __launch_bounds__(256) void colsum_kernel(const float* __restrict__ in, int rows, int cols, float* __restrict__ out) {
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= cols) return;
    float acc = 0.f;
    for (int b = 0; b < rows; ++b) acc += in[(int64_t)b * cols + n];
    out[n] = acc;
}

void launch_colsum(hipStream_t s, const float* in, int rows, int cols, float* out) {
    hipLaunchKernelGGL(colsum_kernel, dim3((cols + 255) / 256), dim3(256), 0, s, in, rows, cols, out);
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* p, int64_t n, int64_t rstride) {
    p = rep_at(p, (int64_t)blockIdx.z * rstride);
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.f;
}

void launch_fill_zero(hipStream_t s, float* p, int64_t n, Reps reps) {
    if (n <= 0) return;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks, 1, reps.n), dim3(256), 0, s, p, n, reps.stride);
}
