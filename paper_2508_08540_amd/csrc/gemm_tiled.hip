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

// ---- the same product with both operands rounded to bf16 (nearest even) on the way into LDS --------------------
// v_mfma_f32_16x16x32_bf16: lane (r, g) supplies A[r][8g .. 8g+7] and B[8g .. 8g+7][r] as eight bf16 and holds
// C[4g + i][r].  K advances 32 at a time; LDS tiles are bf16 [128 rows][32 k] with a row pitch of 80 bytes, for which
// the 16-byte operand reads of a quarter wave fall into distinct banks.  Accumulation, epilogue and memory stay fp32.
#define GB_K 32
#define GB_PITCH 40   // bf16 elements per LDS row

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){lo, hi}, bf16x2_t));
}

// Global fetch of a 128 x 32 operand tile into four float4 per thread.  Row-major operands: task f = row * 8 + k-quad.
// K-major operands: task f takes two adjacent k for four adjacent rows (v[2i] at k, v[2i+1] at k + 1).
template <bool KMAJOR>
__device__ __forceinline__ void gb_fetch(const float* __restrict__ P, int ld, int rows, int row0, int k0, int k_end, bool vec, f32x4 (&v)[4]) {
    if (KMAJOR) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int kp = (threadIdx.x & 7) + 8 * i, r = row0 + 4 * (threadIdx.x >> 3);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int k = k0 + 2 * kp + h;
                f32x4 t = {0.f, 0.f, 0.f, 0.f};
                if (k < k_end) {
                    const float* p = P + (int64_t)k * ld + r;
                    if (vec && r + 3 < rows) t = *reinterpret_cast<const f32x4*>(p);
                    else
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (r + j < rows) t[j] = p[j];
                }
                v[2 * i + h] = t;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int f = threadIdx.x + 256 * i;
            const int r = row0 + (f >> 3), k = k0 + 4 * (f & 7);
            f32x4 t = {0.f, 0.f, 0.f, 0.f};
            if (r < rows) {
                const float* p = P + (int64_t)r * ld + k;
                if (vec && k + 3 < k_end) t = *reinterpret_cast<const f32x4*>(p);
                else
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (k + j < k_end) t[j] = p[j];
            }
            v[i] = t;
        }
    }
}

// The same fetch without any bounds check, for operands whose rows allow 16-byte loads and whose K is a multiple of
// 32: element offsets of the thread's four loads at k = 0 are fixed before the loop.  Rows past the end of the matrix
// are clamped to the last valid ones: they only feed rows or columns of C that are never stored.
template <bool KMAJOR>
__device__ __forceinline__ void gb_offsets(uint32_t (&off)[4], int ld, int rows, int row0) {
    if (KMAJOR) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kp = (threadIdx.x & 7) + 8 * i, r = min(row0 + 4 * (int)(threadIdx.x >> 3), rows - 4);
                off[2 * i + h] = (uint32_t)((2 * kp + h) * ld + r);
            }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int f = threadIdx.x + 256 * i;
            off[i] = (uint32_t)(min(row0 + (f >> 3), rows - 1) * ld + 4 * (f & 7));
        }
    }
}
template <bool KMAJOR>
__device__ __forceinline__ void gb_fetch_fast(const float* __restrict__ P, const uint32_t (&off)[4], int ld, int k, f32x4 (&v)[4]) {
    const uint32_t step = KMAJOR ? (uint32_t)k * (uint32_t)ld : (uint32_t)k;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = *reinterpret_cast<const f32x4*>(P + (off[i] + step));
}

template <bool KMAJOR>
__device__ __forceinline__ void gb_put(__bf16* __restrict__ S, const f32x4 (&v)[4]) {
    if (KMAJOR) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int kp = (threadIdx.x & 7) + 8 * i, r = 4 * (threadIdx.x >> 3);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<uint32_t*>(S + (r + j) * GB_PITCH + 2 * kp) = pack_bf16(v[2 * i][j], v[2 * i + 1][j]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int f = threadIdx.x + 256 * i;
            *reinterpret_cast<uint2*>(S + (f >> 3) * GB_PITCH + 4 * (f & 7)) = make_uint2(pack_bf16(v[i][0], v[i][1]), pack_bf16(v[i][2], v[i][3]));
        }
    }
}

template <bool AK, bool BK, bool FAST>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmDesc d) {
    __shared__ __attribute__((aligned(16))) __bf16 As[2][GT_TILE * GB_PITCH], Bs[2][GT_TILE * GB_PITCH];
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

    // Rows of a matrix whose pitch is a power of two fall into few memory channels at any one k.  Each tile row of C
    // therefore starts its walk over K at a different step and wraps around, so that the workgroups in flight read
    // different k ranges; tiles that share rows of A keep the same order.
    const int steps = (k_end - k_begin + GB_K - 1) / GB_K;
    const int rot = steps > 0 ? tile_y % steps : 0;
    auto k_of = [&](int i) {
        const int sidx = i + rot < steps ? i + rot : i + rot - steps;
        return k_begin + sidx * GB_K;
    };
    f32x4 pa[4], pb[4];
    uint32_t offa[4], offb[4];
    if (FAST) {
        gb_offsets<AK>(offa, d.lda, d.M, m0);
        gb_offsets<BK>(offb, d.ldb, d.N, n0);
    }
    auto fetch = [&](int k) {
        if (FAST) {
            gb_fetch_fast<AK>(A, offa, d.lda, k, pa);
            gb_fetch_fast<BK>(B, offb, d.ldb, k, pb);
        } else {
            gb_fetch<AK>(A, d.lda, d.M, m0, k, k_end, avec, pa);
            gb_fetch<BK>(B, d.ldb, d.N, n0, k, k_end, bvec, pb);
        }
    };
    fetch(k_of(0));
    gb_put<AK>(As[0], pa);
    gb_put<BK>(Bs[0], pb);
    __syncthreads();
    int buf = 0;
    for (int i = 0; i < steps; ++i) {
        const bool more = i + 1 < steps;
        if (more) fetch(k_of(i + 1));
        const __bf16* as = As[buf] + (wm * 64 + r) * GB_PITCH + 8 * g;
        const __bf16* bs = Bs[buf] + (wn * 64 + r) * GB_PITCH + 8 * g;
        bf16x8_t a[4], b[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            a[t] = *reinterpret_cast<const bf16x8_t*>(as + 16 * t * GB_PITCH);
            b[t] = *reinterpret_cast<const bf16x8_t*>(bs + 16 * t * GB_PITCH);
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
        if (more) {
            gb_put<AK>(As[buf ^ 1], pa);
            gb_put<BK>(Bs[buf ^ 1], pb);
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
    const int k_step = d.bf16 ? GB_K : GT_K;
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
    if (d.bf16) {
        // the unchecked fetch needs 16-byte loads on both operands, whole K steps and 32-bit element offsets
        const int64_t span_a = (int64_t)(d.a_kmajor ? d.K : d.M) * d.lda, span_b = (int64_t)(d.b_kmajor ? d.K : d.N) * d.ldb;
        const bool fast = d.a_vec && d.b_vec && d.K % GB_K == 0 && (!d.a_kmajor || d.M % 4 == 0) && (!d.b_kmajor || d.N % 4 == 0) &&
                          d.M >= 4 && d.N >= 4 && span_a < (int64_t(1) << 30) && span_b < (int64_t(1) << 30);
#define GB_LAUNCH(AKM, BKM)                                                                                   \
    do {                                                                                                      \
        if (fast) hipLaunchKernelGGL((gemm_bf16_kernel<AKM, BKM, true>), grid, dim3(256), 0, s, d);            \
        else hipLaunchKernelGGL((gemm_bf16_kernel<AKM, BKM, false>), grid, dim3(256), 0, s, d);                \
    } while (0)
        if (d.a_kmajor && d.b_kmajor) GB_LAUNCH(true, true);
        else if (d.a_kmajor) GB_LAUNCH(true, false);
        else if (d.b_kmajor) GB_LAUNCH(false, true);
        else GB_LAUNCH(false, false);
#undef GB_LAUNCH
    } else if (d.a_kmajor && d.b_kmajor) hipLaunchKernelGGL((gemm_tiled_kernel<true, true>), grid, dim3(256), 0, s, d);
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
