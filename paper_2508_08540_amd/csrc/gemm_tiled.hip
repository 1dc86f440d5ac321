// Tiled fp32 GEMM on the matrix cores for the sequence model: C[m][n] = alpha * sum_k A(m,k) B(n,k) [+ bias[n]] [+ R[m][n]].
//
// With G set the epilogue also stores gelu(C) there (erf form); C itself may then be NULL.
// A(m,k) is A[m*lda + k] or, with a_kmajor, A[k*lda + m]; likewise B(n,k).  With these two flags one kernel serves
// y = x W^T (both k-contiguous), dx = dy W (B k-major), dW = dy^T x (both k-major, contraction over tokens) and the
// attention products.  A batch index z = z1 * inner + z2 adds z1*s1 + z2*s2 to each base pointer (heads inside
// samples).  The contraction can be split over blockIdx.z into partial results that gemm_reduce_kernel adds in split
// order (deterministic).
// Workgroup = 128 x 128 tile of C, four waves as 2 x 2, each 64 x 64 = 4 x 4 blocks of v_mfma_f32_16x16x4_f32.
// K advances 16 at a time through two LDS buffers holding As[k][m] and Bs[k][n] (row pitch 144 floats: a wave's
// read of 16 rows x 4 k-groups touches every bank exactly twice); the next step's global loads are in flight in
// registers while the MFMAs of the current step run.
#include "kernels.h"

#define GT_TILE 128
#define GT_K 16
#define GT_LD 144

template <bool KMAJOR>
__device__ __forceinline__ void gt_fetch(const float* __restrict__ P, int ld, int rows, int K, int row0, int k0, int k_end, bool vec,
                                         f32x4 (&v)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int f = threadIdx.x + 256 * i;
        v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (KMAJOR) {
            const int k = k0 + (f >> 5), r = row0 + 4 * (f & 31);
            if (k < k_end) {
                const float* p = P + (int64_t)k * ld + r;
                if (vec && r + 3 < rows) v[i] = *reinterpret_cast<const f32x4*>(p);
                else
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (r + j < rows) v[i][j] = p[j];
            }
        } else {
            const int r = row0 + (f >> 2), k = k0 + 4 * (f & 3);
            if (r < rows) {
                const float* p = P + (int64_t)r * ld + k;
                if (vec && k + 3 < k_end) v[i] = *reinterpret_cast<const f32x4*>(p);
                else
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (k + j < k_end) v[i][j] = p[j];
            }
        }
    }
    (void)K;
}

template <bool KMAJOR>
__device__ __forceinline__ void gt_put(float* __restrict__ S, const f32x4 (&v)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int f = threadIdx.x + 256 * i;
        if (KMAJOR) {
            *reinterpret_cast<f32x4*>(S + (f >> 5) * GT_LD + 4 * (f & 31)) = v[i];
        } else {
            const int r = f >> 2, k = 4 * (f & 3);
#pragma unroll
            for (int j = 0; j < 4; ++j) S[(k + j) * GT_LD + r] = v[i][j];
        }
    }
}

// Workgroups are handed to the eight XCDs (each with its own L2) round-robin in launch order.  When the tile count of
// one matrix divides by eight, launch slot i takes tile (i % 8) * (tiles / 8) + i / 8, so that an XCD walks a contiguous
// range of tiles, n fastest: the workgroups that share rows of A run on the same L2, one after the other.
__device__ __forceinline__ void gt_tile_of_block(int& tile_x, int& tile_y) {
    const int nx = gridDim.x, tiles = nx * gridDim.y;
    int id = blockIdx.y * nx + blockIdx.x;
    if ((tiles & 7) == 0) id = (id & 7) * (tiles >> 3) + (id >> 3);
    tile_y = id / nx;
    tile_x = id - tile_y * nx;
}

// Writes a wave's 64 x 64 block: lane (r, g) holds C[m = .. + 4g + i][n = .. + r] of every 16 x 16 block.  Blocks that
// lie inside C take the path without bounds checks.
template <bool GUARD>
__device__ __forceinline__ void gt_store_block(const GemmDesc& d, const f32x4 (&acc)[4][4], int m_base, int n_base, float* C, const float* R,
                                               int ldc, bool plain, int r, int g) {
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int n = n_base + nt * 16 + r;
            const float bias = (!plain && d.bias && (!GUARD || n < d.N)) ? d.bias[n] : 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = m_base + mt * 16 + 4 * g + i;
                if (!GUARD || (m < d.M && n < d.N)) {
                    float v = acc[mt][nt][i];
                    if (!plain) {
                        v = v * d.alpha + bias;
                        if (R) v += R[(int64_t)m * ldc + n];
                        if (d.G) d.G[(int64_t)m * ldc + n] = 0.5f * v * (1.f + erff(v * 0.70710678118654752f));
                    }
                    if (C) C[(int64_t)m * ldc + n] = v;
                }
            }
        }
}

__device__ __forceinline__ void gt_store(const GemmDesc& d, const f32x4 (&acc)[4][4], int m_base, int n_base, int z, int z1, int z2, int split,
                                         int r, int g) {
    const bool plain = d.splits > 1;   // partial sums go out as they are; the reduction applies the epilogue
    float* C = plain ? d.part + ((int64_t)z * d.splits + split) * d.part_stride : d.C ? d.C + z1 * d.sc1 + z2 * d.sc2 : nullptr;
    const int ldc = plain ? d.N : d.ldc;
    const float* R = (plain || !d.R) ? nullptr : d.R + z1 * d.sc1 + z2 * d.sc2;
    if (m_base + 64 <= d.M && n_base + 64 <= d.N) gt_store_block<false>(d, acc, m_base, n_base, C, R, ldc, plain, r, g);
    else gt_store_block<true>(d, acc, m_base, n_base, C, R, ldc, plain, r, g);
}

template <bool AK, bool BK>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(GemmDesc d) {
    __shared__ float As[2][GT_K * GT_LD], Bs[2][GT_K * GT_LD];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    int tile_x, tile_y;
    gt_tile_of_block(tile_x, tile_y);
    const int m0 = tile_y * GT_TILE, n0 = tile_x * GT_TILE;
    const int split = blockIdx.z % d.splits, z = blockIdx.z / d.splits;
    const int z1 = z / d.inner, z2 = z - z1 * d.inner;
    const float* A = d.A + z1 * d.sa1 + z2 * d.sa2;
    const float* B = d.B + z1 * d.sb1 + z2 * d.sb2;
    const int k_begin = split * d.k_chunk;
    const int k_end = min(d.K, k_begin + d.k_chunk);
    const bool avec = d.a_vec != 0, bvec = d.b_vec != 0;

    f32x4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    f32x4 pa[2], pb[2];
    gt_fetch<AK>(A, d.lda, d.M, d.K, m0, k_begin, k_end, avec, pa);
    gt_fetch<BK>(B, d.ldb, d.N, d.K, n0, k_begin, k_end, bvec, pb);
    gt_put<AK>(As[0], pa);
    gt_put<BK>(Bs[0], pb);
    __syncthreads();
    int buf = 0;
    for (int k0 = k_begin; k0 < k_end; k0 += GT_K) {
        const bool more = k0 + GT_K < k_end;
        if (more) {
            gt_fetch<AK>(A, d.lda, d.M, d.K, m0, k0 + GT_K, k_end, avec, pa);
            gt_fetch<BK>(B, d.ldb, d.N, d.K, n0, k0 + GT_K, k_end, bvec, pb);
        }
        const float* as = As[buf] + wm * 64 + r;
        const float* bs = Bs[buf] + wn * 64 + r;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a[4], b[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                a[t] = as[(4 * j + g) * GT_LD + 16 * t];
                b[t] = bs[(4 * j + g) * GT_LD + 16 * t];
            }
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
        }
        if (more) {
            gt_put<AK>(As[buf ^ 1], pa);
            gt_put<BK>(Bs[buf ^ 1], pb);
        }
        __syncthreads();
        buf ^= 1;
    }
    gt_store(d, acc, m0 + wm * 64, n0 + wn * 64, z, z1, z2, split, r, g);
}

// out[i] = alpha * sum_z part[z][i] (+ bias) (+ R), in split order
__global__ __launch_bounds__(256) void gemm_split_reduce_kernel(const float* __restrict__ part, int splits, int M, int N, float alpha,
                                                                const float* __restrict__ bias, const float* __restrict__ R, int ldc,
                                                                float* __restrict__ out) {
    const int64_t total = (int64_t)M * N;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        float acc = part[i];
        for (int zz = 1; zz < splits; ++zz) acc += part[(int64_t)zz * total + i];
        const int64_t m = i / N;
        const int n = (int)(i - m * N);
        acc *= alpha;
        if (bias) acc += bias[n];
        if (R) acc += R[m * ldc + n];
        out[m * ldc + n] = acc;
    }
}

size_t gemm_tiled_partial_floats(int M, int N, int splits) { return splits > 1 ? (size_t)M * N * splits : 0; }

// Launch.  Split-K is only supported for a single matrix (batch == 1); d.part must then hold M*N*splits floats.
void launch_gemm_tiled(hipStream_t s, GemmDesc d) {
    if (d.splits < 1) d.splits = 1;
    if (d.inner < 1) d.inner = 1;
    if (d.batch < 1) d.batch = 1;
    const int k_step = GT_K;
    int k_chunk = ((d.K + d.splits - 1) / d.splits + k_step - 1) / k_step * k_step;
    d.splits = (d.K + k_chunk - 1) / k_chunk;
    d.k_chunk = k_chunk;
    d.part_stride = (int64_t)d.M * d.N;
    auto aligned = [](const float* p, int ld, int64_t s1, int64_t s2) {
        return (reinterpret_cast<uintptr_t>(p) & 15) == 0 && ld % 4 == 0 && s1 % 4 == 0 && s2 % 4 == 0;
    };
    d.a_vec = aligned(d.A, d.lda, d.sa1, d.sa2) ? 1 : 0;
    d.b_vec = aligned(d.B, d.ldb, d.sb1, d.sb2) ? 1 : 0;
    dim3 grid((d.N + GT_TILE - 1) / GT_TILE, (d.M + GT_TILE - 1) / GT_TILE, d.batch * d.splits);
    if (d.a_kmajor && d.b_kmajor) hipLaunchKernelGGL((gemm_tiled_kernel<true, true>), grid, dim3(256), 0, s, d);
    else if (d.a_kmajor) hipLaunchKernelGGL((gemm_tiled_kernel<true, false>), grid, dim3(256), 0, s, d);
    else if (d.b_kmajor) hipLaunchKernelGGL((gemm_tiled_kernel<false, true>), grid, dim3(256), 0, s, d);
    else hipLaunchKernelGGL((gemm_tiled_kernel<false, false>), grid, dim3(256), 0, s, d);
    if (d.splits > 1) {
        int64_t total = (int64_t)d.M * d.N;
        int64_t blocks = (total + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(gemm_split_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, d.part, d.splits, d.M, d.N, d.alpha, d.bias, d.R,
                           d.ldc, d.C);
    }
}
