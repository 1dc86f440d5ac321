// fp32 GEMM on the matrix cores for the fully connected layers: C[m][n] = sum_k A(m,k) B(n,k).
//
// One wavefront owns a 16x16 tile of C and walks its K-range in steps of 16 with four
// v_mfma_f32_16x16x4_f32 instructions.  Lane l supplies row (l % 16) and the K-slots of lane
// group g = l / 16; in step j the group contributes k = k0 + 4g + j to both operands, so a
// k-contiguous operand is fetched as one 16-byte load per lane.  The K dimension is split over
// blockIdx.z into partial tiles that a second kernel adds in split order (deterministic), fused
// with bias, ReLU and a ReLU-mask multiply.
#include "kernels.h"

template <bool KMAJOR>
__device__ __forceinline__ void load_k4(const float* __restrict__ P, int ld, int row, int rows, int k, int k_end,
                                        bool vec_ok, float (&v)[4]) {
    if (row >= rows) {
        v[0] = v[1] = v[2] = v[3] = 0.f;
        return;
    }
    if (KMAJOR) {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (k + j < k_end) ? P[(int64_t)(k + j) * ld + row] : 0.f;
    } else {
        const float* p = P + (int64_t)row * ld + k;
        if (vec_ok && k + 3 < k_end) {
            f32x4 t = *reinterpret_cast<const f32x4*>(p);
            v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (k + j < k_end) ? p[j] : 0.f;
        }
    }
}

template <bool A_KMAJOR, bool B_KMAJOR>
__global__ __launch_bounds__(64) void gemm16_kernel(const float* __restrict__ A, int lda, const float* __restrict__ B,
                                                    int ldb, int M, int N, int K, int k_chunk, float* __restrict__ part,
                                                    int a_vec, int b_vec) {
    const int lane = threadIdx.x, r = lane & 15, g = lane >> 4;
    const int m0 = blockIdx.x * 16, n0 = blockIdx.y * 16;
    const int k_begin = blockIdx.z * k_chunk;
    const int k_end = min(K, k_begin + k_chunk);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = k_begin; k0 < k_end; k0 += 16) {
        float a[4], b[4];
        load_k4<A_KMAJOR>(A, lda, m0 + r, M, k0 + 4 * g, k_end, a_vec != 0, a);
        load_k4<B_KMAJOR>(B, ldb, n0 + r, N, k0 + 4 * g, k_end, b_vec != 0, b);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j], b[j], acc, 0, 0, 0);
    }
    // lane holds C[m0 + 4g + i][n0 + r], i = 0..3
    float* out = part + (int64_t)blockIdx.z * M * N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = m0 + 4 * g + i, n = n0 + r;
        if (m < M && n < N) out[(int64_t)m * N + n] = acc[i];
    }
}

__global__ __launch_bounds__(256) void gemm_reduce_kernel(const float* __restrict__ part, int splits, int M, int N,
                                                          float* __restrict__ out, const float* __restrict__ bias,
                                                          int relu, const float* __restrict__ mask) {
    int64_t total = (int64_t)M * N;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        float acc = part[i];
        for (int z = 1; z < splits; ++z) acc += part[(int64_t)z * total + i];
        if (bias) acc += bias[i % N];
        if (relu) acc = relu_keep_nan(acc);
        if (mask) acc = mask[i] > 0.f ? acc : 0.f;
        out[i] = acc;
    }
}

size_t gemm_partial_floats(int M, int N, int splits) { return (size_t)M * N * splits; }

void launch_gemm(hipStream_t s, const float* A, int lda, bool a_kmajor, const float* B, int ldb, bool b_kmajor, int M,
                 int N, int K, int splits, float* part, float* out, const float* bias, bool relu, const float* mask) {
    int k_chunk = ((K + splits - 1) / splits + 15) / 16 * 16;
    splits = (K + k_chunk - 1) / k_chunk;
    dim3 grid((M + 15) / 16, (N + 15) / 16, splits);
    int a_vec = (!a_kmajor && lda % 4 == 0 && (reinterpret_cast<uintptr_t>(A) & 15) == 0) ? 1 : 0;
    int b_vec = (!b_kmajor && ldb % 4 == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0) ? 1 : 0;
#define GEMM_LAUNCH(AK, BK) \
    hipLaunchKernelGGL((gemm16_kernel<AK, BK>), grid, dim3(64), 0, s, A, lda, B, ldb, M, N, K, k_chunk, part, a_vec, b_vec)
    if (a_kmajor && b_kmajor) GEMM_LAUNCH(true, true);
    else if (a_kmajor) GEMM_LAUNCH(true, false);
    else if (b_kmajor) GEMM_LAUNCH(false, true);
    else GEMM_LAUNCH(false, false);
#undef GEMM_LAUNCH
    int64_t total = (int64_t)M * N;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(gemm_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, part, splits, M, N, out, bias,
                       relu ? 1 : 0, mask);
}
