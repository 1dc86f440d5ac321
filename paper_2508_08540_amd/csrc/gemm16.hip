// Tiled GEMM on the bf16 matrix cores with both operands stored in bf16:
//   C[m][n] = alpha * sum_k A(m,k) B(n,k) [+ bias[n]] [+ R[m][n]],  fp32 sums.
// A(m,k) is A[m*lda + k] or, with a_kmajor, A[k*lda + m]; likewise B(n,k); batch index z = z1 * inner + z2 as in the
// fp32 kernel.  The result goes out as fp32 (C), as bf16 rounded to nearest even (C16), as bf16 gelu(C) (G16), or any
// combination; bias and R are fp32.  With splits > 1 the K range is cut into fp32 partials that
// gemm16_split_reduce_kernel adds in split order.
//
// Workgroup = 128 x 128 tile of C, four waves as 2 x 2, each 64 x 64 = 4 x 4 blocks of v_mfma_f32_16x16x32_bf16.
// K advances 32 at a time through two LDS buffers [128 rows][32 k] with a row pitch of 96 bytes (measured: the 16-byte
// operand reads, 16 rows x 4 k groups per instruction, run at the full LDS rate when the pitch is 32 bytes more than a
// multiple of 64, at half of it with an odd number of 16-byte units such as 80 or 144 bytes); the next two steps'
// global loads (16 bytes = 8 bf16 per lane) are in flight in registers while the matrix instructions run.  The B tile is passed as the first MFMA operand, so
// that lane (r, g) holds C[m = r][n = 4g .. 4g+3] of a block: four adjacent outputs, stored with one 16-byte (fp32)
// or 8-byte (bf16) store.
#include "act.h"
#include "kernels.h"

#define G16_TILE 128
#define G16_K 32
#define G16_PITCH 48   // bf16 elements per LDS row (96 bytes)

typedef __bf16 bf16x2_v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_v __attribute__((ext_vector_type(8)));
typedef float f32x2_v __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_v){lo, hi}, bf16x2_v));
}

// ---- operand fetch: two 16-byte pieces per thread for every 128 rows of an operand tile ------------------------------
// An operand tile has NP * 128 rows (NP = 1 or 2); piece i = 2 * group + sub belongs to rows 128 * group ...
// Row-major operand: f = tid + 256 sub covers row f >> 2, k = 8 (f & 3) .. + 7.
// K-major operand: the thread takes k = 2 kp + sub for the eight rows of chunk c, kp = (tid >> 2) & 15,
// c = 4 (tid >> 6) + (tid & 3); the two pieces of a group are interleaved into (k, k+1) pairs on the way into LDS.
template <bool KMAJOR>
__device__ __forceinline__ void g16_piece(int i, int& row, int& k) {
    const int group = i >> 1, sub = i & 1;
    if (KMAJOR) {
        row = 128 * group + 8 * (4 * (int)(threadIdx.x >> 6) + (int)(threadIdx.x & 3));
        k = 2 * (int)((threadIdx.x >> 2) & 15) + sub;
    } else {
        const int f = threadIdx.x + 256 * sub;
        row = 128 * group + (f >> 2);
        k = 8 * (f & 3);
    }
}

// Checked fetch: any shape and alignment, element by element where a 16-byte load is not possible.
template <bool KMAJOR, int NP>
__device__ __forceinline__ void g16_fetch(const bf16_t* __restrict__ P, int ld, int rows, int row0, int k0, int k_end, bool vec,
                                          u32x4 (&v)[2 * NP]) {
#pragma unroll
    for (int i = 0; i < 2 * NP; ++i) {
        int row, k;
        g16_piece<KMAJOR>(i, row, k);
        row += row0;
        k += k0;
        u32x4 w = {0u, 0u, 0u, 0u};
        if (KMAJOR) {
            if (k < k_end) {
                const bf16_t* p = P + (int64_t)k * ld + row;
                if (vec && row + 7 < rows) {
                    w = *reinterpret_cast<const u32x4*>(p);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (row + j < rows) w[j >> 1] |= (uint32_t)p[j] << (16 * (j & 1));
                }
            }
        } else {
            if (row < rows) {
                const bf16_t* p = P + (int64_t)row * ld + k;
                if (vec && k + 7 < k_end) {
                    w = *reinterpret_cast<const u32x4*>(p);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (k + j < k_end) w[j >> 1] |= (uint32_t)p[j] << (16 * (j & 1));
                }
            }
        }
        v[i] = w;
    }
}

// Unchecked fetch: element offsets of the two pieces at k = 0 are fixed before the loop.  Rows past the end of the
// matrix are clamped to valid ones; they only feed rows or columns of C that are never stored.
template <bool KMAJOR, int NP>
__device__ __forceinline__ void g16_offsets(uint32_t (&off)[2 * NP], int ld, int rows, int row0) {
#pragma unroll
    for (int i = 0; i < 2 * NP; ++i) {
        int row, k;
        g16_piece<KMAJOR>(i, row, k);
        if (KMAJOR) off[i] = (uint32_t)(k * ld + min(row0 + row, rows - 8));
        else off[i] = (uint32_t)(min(row0 + row, rows - 1) * ld + k);
    }
}
template <bool KMAJOR, int NP>
__device__ __forceinline__ void g16_fetch_fast(const bf16_t* __restrict__ P, const uint32_t (&off)[2 * NP], int ld, int k, u32x4 (&v)[2 * NP]) {
    const uint32_t step = KMAJOR ? (uint32_t)k * (uint32_t)ld : (uint32_t)k;
#pragma unroll
    for (int i = 0; i < 2 * NP; ++i) v[i] = *reinterpret_cast<const u32x4*>(P + (off[i] + step));
}

template <bool KMAJOR, int NP>
__device__ __forceinline__ void g16_put(bf16_t* __restrict__ S, const u32x4 (&v)[2 * NP]) {
    if (KMAJOR) {
#pragma unroll
        for (int grp = 0; grp < NP; ++grp) {
            int row, k;
            g16_piece<true>(2 * grp, row, k);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // rows row + 2j and row + 2j + 1: the low and the high halves of word j of both pieces
                *reinterpret_cast<uint32_t*>(S + (row + 2 * j) * G16_PITCH + k) = __builtin_amdgcn_perm(v[2 * grp + 1][j], v[2 * grp][j], 0x05040100u);
                *reinterpret_cast<uint32_t*>(S + (row + 2 * j + 1) * G16_PITCH + k) = __builtin_amdgcn_perm(v[2 * grp + 1][j], v[2 * grp][j], 0x07060302u);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 2 * NP; ++i) {
            int row, k;
            g16_piece<false>(i, row, k);
            *reinterpret_cast<u32x4*>(S + row * G16_PITCH + k) = v[i];
        }
    }
}

__device__ __forceinline__ void g16_tile_of_block(int& tile_x, int& tile_y) {
    // launch slot -> tile such that each of the eight XCDs (round-robin over launch slots) walks a contiguous tile range
    const int nx = gridDim.x, tiles = nx * gridDim.y;
    int id = blockIdx.y * nx + blockIdx.x;
    if ((tiles & 7) == 0) id = (id & 7) * (tiles >> 3) + (id >> 3);
    tile_y = id / nx;
    tile_x = id - tile_y * nx;
}

// Stores a wave's 64 x 64 block; lane (r, g) holds acc[mt][nt][i] = C[m_base + 16 mt + r][n_base + 16 nt + 4 g + i].
template <bool VEC, int MB, bool GELU>
__device__ __forceinline__ void g16_store_block(const Gemm16Desc& d, const f32x4 (&acc)[MB][4], int m_base, int n_base, float* C, bf16_t* C16,
                                                bf16_t* G16, const float* R, const float* bias, int ldc, bool plain, int r, int g) {
#pragma unroll
    for (int mt = 0; mt < MB; ++mt) {
        const int m = m_base + 16 * mt + r;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int n = n_base + 16 * nt + 4 * g;
            if (VEC) {
                // the block lies inside C and rows allow 16-byte accesses
                f32x4 v = acc[mt][nt];
                const int64_t at = (int64_t)m * ldc + n;
                if (!plain) {
                    v *= d.alpha;
                    if (bias) v += *reinterpret_cast<const f32x4*>(bias + n);
                    if (R) v += *reinterpret_cast<const f32x4*>(R + at);
                }
                if (C) *reinterpret_cast<f32x4*>(C + at) = v;
                if (C16) *reinterpret_cast<u32x2*>(C16 + at) = u32x2{pack2_bf16(v[0], v[1]), pack2_bf16(v[2], v[3])};
                if (GELU && G16) {
                    f32x4 q;
#pragma unroll
                    for (int i = 0; i < 4; ++i) q[i] = 0.5f * v[i] * (1.f + erff(v[i] * 0.70710678118654752f));
                    *reinterpret_cast<u32x2*>(G16 + at) = u32x2{pack2_bf16(q[0], q[1]), pack2_bf16(q[2], q[3])};
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (m < d.M && n + i < d.N) {
                        float v = acc[mt][nt][i];
                        const int64_t at = (int64_t)m * ldc + n + i;
                        if (!plain) {
                            v *= d.alpha;
                            if (bias) v += bias[n + i];
                            if (R) v += R[at];
                        }
                        if (C) C[at] = v;
                        if (C16) C16[at] = (bf16_t)(pack2_bf16(v, 0.f) & 0xffffu);
                        if (GELU && G16) G16[at] = (bf16_t)(pack2_bf16(0.5f * v * (1.f + erff(v * 0.70710678118654752f)), 0.f) & 0xffffu);
                    }
                }
            }
        }
    }
}

// Softmax statistics of a wave's 64 columns for each of its 64 rows: ce_part[2 * tile_x + wn][m] = (max, sum of
// exp(v - max)) over the columns that exist, and the value in column ce_targets[m] goes to ce_tlogit[m] when this wave
// holds it.  A later pass folds the pairs of a row in index order.  The product is taken without bias.
template <int MB>
__device__ __forceinline__ void g16_ce_block(const Gemm16Desc& d, const f32x4 (&acc)[MB][4], int m_base, int n_base, int part_idx, int r, int g) {
    const bool full = n_base + 64 <= d.N;   // uniform: every column of the block exists
#pragma unroll
    for (int mt = 0; mt < MB; ++mt) {
        const int m = m_base + 16 * mt + r;
        const int tgt = m < d.M ? d.ce_targets[m] : -1;
        const int t_local = tgt - n_base - 4 * g;   // column of the target among this lane's 16, as 16 nt + i
        float v[16];
        float mx = -INFINITY, at_target = 0.f;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float q = acc[mt][nt][i] * d.alpha;
                if (!full && n_base + 16 * nt + 4 * g + i >= d.N) q = -INFINITY;
                v[4 * nt + i] = q;
                mx = fmaxf(mx, q);
                at_target = t_local == 16 * nt + i ? q : at_target;
            }
        if (t_local >= 0 && t_local < 64 && (t_local & 12) == 0) d.ce_tlogit[m] = at_target;
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float sum = 0.f;
        if (mx > -INFINITY)
#pragma unroll
            for (int j = 0; j < 16; ++j) sum += __expf(v[j] - mx);   // hardware exponential: 64 per lane, the accurate one would double the tile time
        sum += __shfl_xor(sum, 16, 64);
        sum += __shfl_xor(sum, 32, 64);
        if (g == 0 && m < d.M) *reinterpret_cast<f32x2_v*>(d.ce_part + 2 * ((int64_t)part_idx * d.M + m)) = f32x2_v{mx, sum};
    }
}

// MB = 16-row blocks per wave in m: 4 (128 x 128 tile per workgroup) or 8 (256 x 128: a third less operand traffic
// per flop, for products with enough tiles to fill the chip that way).
// EPI: 0 plain epilogue, 1 also writes gelu(C) (its erf code stays out of the other instantiations), 2 softmax statistics
template <bool AK, bool BK, bool FAST, int EPI, int MB>
__global__ __launch_bounds__(256, MB == 8 ? 2 : 3) void gemm16_kernel(Gemm16Desc d) {
    constexpr int NPA = MB / 4, TILE_M = 32 * MB;
    __shared__ __attribute__((aligned(16))) bf16_t As[2][TILE_M * G16_PITCH], Bs[2][G16_TILE * G16_PITCH];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    int tile_x, tile_y;
    g16_tile_of_block(tile_x, tile_y);
    const int m0 = tile_y * TILE_M, n0 = tile_x * G16_TILE;
    const int split = blockIdx.z % d.splits, z = blockIdx.z / d.splits;
    const int z1 = z / d.inner, z2 = z - z1 * d.inner;
    const bf16_t* A = d.A + z1 * d.sa1 + z2 * d.sa2;
    const bf16_t* B = d.B + z1 * d.sb1 + z2 * d.sb2;
    const int k_begin = split * d.k_chunk;
    const int k_end = min(d.K, k_begin + d.k_chunk);
    const bool avec = d.a_vec != 0, bvec = d.b_vec != 0;

    f32x4 acc[MB][4];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // each tile row of C starts its walk over K at a different step and wraps around, so that workgroups in flight
    // read different k ranges (rows with a power-of-two pitch otherwise meet in few memory channels)
    const int steps = (k_end - k_begin + G16_K - 1) / G16_K;
    const int rot = steps > 0 ? tile_y % steps : 0;
    auto k_of = [&](int i) {
        const int sidx = i + rot < steps ? i + rot : i + rot - steps;
        return k_begin + sidx * G16_K;
    };
    // Two K steps of global loads are in flight (register sets 0 and 1, used in turn) while a third is multiplied
    // out of LDS: with one to three workgroups per compute unit it is the bytes in flight that bound the rate.
    u32x4 pa0[2 * NPA], pb0[2], pa1[2 * NPA], pb1[2];
    uint32_t offa[2 * NPA], offb[2];
    if (FAST) {
        g16_offsets<AK, NPA>(offa, d.lda, d.M, m0);
        g16_offsets<BK, 1>(offb, d.ldb, d.N, n0);
    }
    auto fetch = [&](int k, u32x4 (&pa)[2 * NPA], u32x4 (&pb)[2]) {
        if (FAST) {
            g16_fetch_fast<AK, NPA>(A, offa, d.lda, k, pa);
            g16_fetch_fast<BK, 1>(B, offb, d.ldb, k, pb);
        } else {
            g16_fetch<AK, NPA>(A, d.lda, d.M, m0, k, k_end, avec, pa);
            g16_fetch<BK, 1>(B, d.ldb, d.N, n0, k, k_end, bvec, pb);
        }
    };
    auto compute = [&](int buf) {
        const bf16_t* as = As[buf] + (wm * 16 * MB + r) * G16_PITCH + 8 * g;
        const bf16_t* bs = Bs[buf] + (wn * 64 + r) * G16_PITCH + 8 * g;
        bf16x8_v a[MB], b[4];
#pragma unroll
        for (int t = 0; t < MB; ++t) a[t] = *reinterpret_cast<const bf16x8_v*>(as + 16 * t * G16_PITCH);
#pragma unroll
        for (int t = 0; t < 4; ++t) b[t] = *reinterpret_cast<const bf16x8_v*>(bs + 16 * t * G16_PITCH);
#pragma unroll
        for (int mt = 0; mt < MB; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[nt], a[mt], acc[mt][nt], 0, 0, 0);
    };
    if (steps > 0) {
        fetch(k_of(0), pa0, pb0);
        g16_put<AK, NPA>(As[0], pa0);
        g16_put<BK, 1>(Bs[0], pb0);
    }
    if (steps > 1) fetch(k_of(1), pa0, pb0);
    __syncthreads();
    int i = 0;
    // steady state, two steps per turn: every fetch and store is unconditional here, so that the wait before a store
    // into LDS counts the younger set's loads as still in flight
    for (; i + 3 < steps; i += 2) {
        fetch(k_of(i + 2), pa1, pb1);
        compute(0);
        g16_put<AK, NPA>(As[1], pa0);
        g16_put<BK, 1>(Bs[1], pb0);
        __syncthreads();
        fetch(k_of(i + 3), pa0, pb0);
        compute(1);
        g16_put<AK, NPA>(As[0], pa1);
        g16_put<BK, 1>(Bs[0], pb1);
        __syncthreads();
    }
    // the last (up to three) steps
    while (i < steps) {
        // LDS buffer 0 holds step i, register set 0 step i + 1
        if (i + 2 < steps) fetch(k_of(i + 2), pa1, pb1);
        compute(0);
        if (i + 1 < steps) {
            g16_put<AK, NPA>(As[1], pa0);
            g16_put<BK, 1>(Bs[1], pb0);
        }
        __syncthreads();
        if (++i >= steps) break;
        // LDS buffer 1 holds step i, register set 1 step i + 1
        if (i + 2 < steps) fetch(k_of(i + 2), pa0, pb0);
        compute(1);
        if (i + 1 < steps) {
            g16_put<AK, NPA>(As[0], pa1);
            g16_put<BK, 1>(Bs[0], pb1);
        }
        __syncthreads();
        ++i;
    }

    const bool plain = d.splits > 1;   // partial sums go out as they are; the reduction applies the epilogue
    const int64_t zoff = z1 * d.sc1 + z2 * d.sc2;
    float* C = plain ? d.part + ((int64_t)z * d.splits + split) * d.part_stride : d.C ? d.C + zoff : nullptr;
    bf16_t* C16 = (plain || !d.C16) ? nullptr : d.C16 + zoff;
    bf16_t* G16 = (plain || !d.G16) ? nullptr : d.G16 + zoff;
    const float* R = (plain || !d.R) ? nullptr : d.R + zoff;
    const float* bias = (plain || !d.bias) ? nullptr : d.bias + z1 * d.sbias1;
    const int ldc = plain ? d.N : d.ldc;
    const int m_base = m0 + wm * 16 * MB, n_base = n0 + wn * 64;
    if (EPI == 2) g16_ce_block<MB>(d, acc, m_base, n_base, 2 * tile_x + wn, r, g);   // its own instantiation: the statistics cost registers
    const bool vec = (plain ? (d.N & 3) == 0 : d.c_vec != 0) && m_base + 16 * MB <= d.M && n_base + 64 <= d.N;
    if (vec) g16_store_block<true, MB, EPI == 1>(d, acc, m_base, n_base, C, C16, G16, R, bias, ldc, plain, r, g);
    else g16_store_block<false, MB, EPI == 1>(d, acc, m_base, n_base, C, C16, G16, R, bias, ldc, plain, r, g);
}

// out[i] = alpha * sum_z part[z][i] (+ bias) (+ R), in split order (weight gradients: fp32 output only); blockIdx.y is the
// matrix of a batch (outer batch index only), whose output starts sc1 floats after the previous one
__global__ __launch_bounds__(256) void gemm16_split_reduce_kernel(const float* __restrict__ part, int splits, int M, int N, float alpha,
                                                                  const float* __restrict__ bias, const float* __restrict__ R, int ldc,
                                                                  float* __restrict__ out, int64_t sc1) {
    const int64_t total = (int64_t)M * N;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    part += (int64_t)blockIdx.y * splits * total;
    out += (int64_t)blockIdx.y * sc1;
    if (R) R += (int64_t)blockIdx.y * sc1;
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

// Launch.  Split-K writes an fp32 output only and, with a batch, needs inner == 1; d.part must then hold
// batch*M*N*splits floats.
void launch_gemm16(hipStream_t s, Gemm16Desc d) {
    if (d.splits < 1) d.splits = 1;
    if (d.inner < 1) d.inner = 1;
    if (d.batch < 1) d.batch = 1;
    int k_chunk = ((d.K + d.splits - 1) / d.splits + G16_K - 1) / G16_K * G16_K;
    d.splits = (d.K + k_chunk - 1) / k_chunk;
    d.k_chunk = k_chunk;
    d.part_stride = (int64_t)d.M * d.N;
    auto al = [](const void* p, int bytes) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0; };
    d.a_vec = (al(d.A, 16) && d.lda % 8 == 0 && d.sa1 % 8 == 0 && d.sa2 % 8 == 0) ? 1 : 0;
    d.b_vec = (al(d.B, 16) && d.ldb % 8 == 0 && d.sb1 % 8 == 0 && d.sb2 % 8 == 0) ? 1 : 0;
    d.c_vec = (al(d.C, 16) && al(d.R, 16) && al(d.bias, 16) && al(d.C16, 8) && al(d.G16, 8) && d.ldc % 4 == 0 && d.sc1 % 4 == 0 && d.sc2 % 4 == 0 && d.sbias1 % 4 == 0) ? 1 : 0;
    // the unchecked fetch needs 16-byte loads on both operands, whole K steps and 32-bit element offsets
    const int64_t span_a = (int64_t)(d.a_kmajor ? d.K : d.M) * d.lda, span_b = (int64_t)(d.b_kmajor ? d.K : d.N) * d.ldb;
    const bool fast = d.a_vec && d.b_vec && d.K % G16_K == 0 && (!d.a_kmajor || d.M % 8 == 0) && (!d.b_kmajor || d.N % 8 == 0) && d.M >= 8 &&
                      d.N >= 8 && span_a < (int64_t(1) << 31) && span_b < (int64_t(1) << 31);
    // 256-row tiles where the product still has at least 512 of them (two per compute unit); they need the unchecked fetch
    const bool tall = fast && !d.a_kmajor && (int64_t)((d.M + 255) / 256) * ((d.N + G16_TILE - 1) / G16_TILE) * d.batch * d.splits >= 512 && d.M >= 256;
    const int tile_m = tall ? 256 : G16_TILE;
    dim3 grid((d.N + G16_TILE - 1) / G16_TILE, (d.M + tile_m - 1) / tile_m, d.batch * d.splits);
#define G16_LAUNCH(AKM, BKM, EPI, TALL_OK)                                                                     \
    do {                                                                                                       \
        if (TALL_OK && tall) hipLaunchKernelGGL((gemm16_kernel<AKM, BKM, true, EPI, TALL_OK ? 8 : 4>), grid, dim3(256), 0, s, d); \
        else if (fast) hipLaunchKernelGGL((gemm16_kernel<AKM, BKM, true, EPI, 4>), grid, dim3(256), 0, s, d);   \
        else hipLaunchKernelGGL((gemm16_kernel<AKM, BKM, false, EPI, 4>), grid, dim3(256), 0, s, d);            \
    } while (0)
    if (d.ce_part) G16_LAUNCH(false, false, 2, true);   // row statistics: row-major factors, one matrix, no split
    else if (d.G16 && !d.a_kmajor && !d.b_kmajor) G16_LAUNCH(false, false, 1, true);
    else if (d.a_kmajor && d.b_kmajor) G16_LAUNCH(true, true, 0, false);
    else if (d.a_kmajor) G16_LAUNCH(true, false, 0, false);
    else if (d.b_kmajor) G16_LAUNCH(false, true, 0, true);
    else G16_LAUNCH(false, false, 0, true);
#undef G16_LAUNCH
    if (d.splits > 1) {
        int64_t total = (int64_t)d.M * d.N;
        int64_t blocks = (total + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(gemm16_split_reduce_kernel, dim3((unsigned)blocks, (unsigned)d.batch), dim3(256), 0, s, d.part, d.splits, d.M, d.N, d.alpha,
                           d.bias, d.R, d.ldc, d.C, d.sc1);
    }
}
