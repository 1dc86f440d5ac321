// Kernels of the sequence model around the GEMMs: embedding lookup and its gradient, layer norm, row softmax,
// the GELU derivative (the forward GELU lives in the GEMM epilogue), per-token cross-entropy over a large vocabulary, and column sums.  All activations are fp32 [tokens][D].
// Column sums over tokens (bias and layer-norm gradients, the position-embedding gradient) are taken in two stages
// with a fixed order: per-workgroup partial rows, then one pass over those.  The token-embedding gradient scatters by
// token id through 64-bit fixed-point integer atomics (scale 2^44), which do not depend on the order of arrival;
// fix_finalize_kernel turns them into floats.
#include "kernels.h"

#define LN_EPS 1e-5f

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
typedef __bf16 sq_bf16x2 __attribute__((ext_vector_type(2)));
typedef float sq_f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t sq_u32x2 __attribute__((ext_vector_type(2)));
// two floats -> two bf16 (nearest even) in one word, the first in the low half
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((sq_f32x2){lo, hi}, sq_bf16x2));
}
__device__ __forceinline__ uint16_t to_bf16(float v) { return (uint16_t)(pack_bf16x2(v, 0.f) & 0xffffu); }
__device__ __forceinline__ void store_bf16x4(uint16_t* p, f32x4 v) {
    *reinterpret_cast<sq_u32x2*>(p) = sq_u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
}

// h[t][:] = tok_emb[token[t]][:] + pos_emb[t % L][:]; one wave per token, D % 4 == 0
__global__ __launch_bounds__(256) void embed_kernel(const int32_t* __restrict__ tokens, int64_t T, int L, int D, const float* __restrict__ tok,
                                                    const float* __restrict__ pos, float* __restrict__ h, uint16_t* __restrict__ h16) {
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int lane = threadIdx.x & 63;
    const float* e = tok + (int64_t)tokens[t] * D;
    const float* p = pos + (int64_t)(t % L) * D;
    for (int c = 4 * lane; c < D; c += 256) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(e + c) + *reinterpret_cast<const f32x4*>(p + c);
        *reinterpret_cast<f32x4*>(h + t * D + c) = v;
        if (h16) store_bf16x4(h16 + t * D + c, v);
    }
}

// acc_tok[token[t]][:] += dh[t][:] (fixed point, 2^-44).  Every token of the batch may hit the same row, so a single
// contribution must stay below `limit` = 2^61 / T in scaled units (16 in real units for 8192 tokens; the single word
// of a row is read on its own, so it may use the whole range below the poison value); beyond that, or
// for a value that is not finite, the word is poisoned and the gradient comes out as NaN.
__global__ __launch_bounds__(256) void embed_grad_kernel(const int32_t* __restrict__ tokens, int64_t T, int D, const float* __restrict__ dh,
                                                         fixsum_t* __restrict__ acc_tok, double limit) {
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int lane = threadIdx.x & 63;
    fixsum_t* a = acc_tok + (int64_t)tokens[t] * D;
    for (int c = lane; c < D; c += 64) fixsum_add(a + c, (double)dh[t * D + c] * FIX_BWD_SCALE, limit);
}

// part[blockIdx.y][n] = sum of X[m][n] over the 64 rows of the block
__global__ __launch_bounds__(256) void colsum_partial_kernel(const float* __restrict__ X, int64_t M, int N, float* __restrict__ part) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const int64_t m0 = (int64_t)blockIdx.y * 64, m1 = m0 + 64 < M ? m0 + 64 : M;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int64_t m = m0;
    for (; m + 3 < m1; m += 4) {
        s0 += X[m * N + n];
        s1 += X[(m + 1) * N + n];
        s2 += X[(m + 2) * N + n];
        s3 += X[(m + 3) * N + n];
    }
    for (; m < m1; ++m) s0 += X[m * N + n];
    part[(int64_t)blockIdx.y * N + n] = (s0 + s1) + (s2 + s3);
}

// out[n] = sum over rows of X[r][n]: 64 columns per workgroup, four row slices folded through LDS in a fixed order
__global__ __launch_bounds__(256) void colsum_rows_kernel(const float* __restrict__ X, int rows, int N, float* __restrict__ out) {
    __shared__ float red[4][64];
    const int c = threadIdx.x & 63, sl = threadIdx.x >> 6, n = blockIdx.x * 64 + c;
    float a0 = 0.f, a1 = 0.f;
    if (n < N) {
        int r = sl;
        for (; r + 4 < rows; r += 8) {
            a0 += X[(int64_t)r * N + n];
            a1 += X[(int64_t)(r + 4) * N + n];
        }
        if (r < rows) a0 += X[(int64_t)r * N + n];
    }
    red[sl][c] = a0 + a1;
    __syncthreads();
    if (sl == 0 && n < N) out[n] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
}

// The same for a table of jobs (blockIdx.y): out[out_off + n] = sum over the job's rows of part[part_off + r * pitch + n]
__global__ __launch_bounds__(256) void colsum_table_kernel(ColsumTable tab, const float* __restrict__ part, float* __restrict__ out) {
    __shared__ float red[4][64];
    const ColsumJob job = tab.j[blockIdx.y];
    const int c = threadIdx.x & 63, sl = threadIdx.x >> 6, n = blockIdx.x * 64 + c;
    if (blockIdx.x * 64 >= job.N) return;
    const float* X = part + job.part_off;
    float a0 = 0.f, a1 = 0.f;
    if (n < job.N) {
        int r = sl;
        for (; r + 4 < job.rows; r += 8) {
            a0 += X[(int64_t)r * job.pitch + n];
            a1 += X[(int64_t)(r + 4) * job.pitch + n];
        }
        if (r < job.rows) a0 += X[(int64_t)r * job.pitch + n];
    }
    red[sl][c] = a0 + a1;
    __syncthreads();
    if (sl == 0 && n < job.N) out[job.out_off + n] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
}

// out[i] = acc[i] / 2^44, acc[i] = 0; blockIdx.y selects a range
__global__ __launch_bounds__(256) void fix_finalize_kernel(FixRangeTable tab, fixsum_t* __restrict__ acc, float* __restrict__ grad) {
    const FixRange r = tab.r[blockIdx.y];
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < r.n; i += (int64_t)gridDim.x * 256) {
        const long long w = (long long)acc[r.acc_off + i];
        grad[r.grad_off + i] = w >= FIX_POISON_MIN ? FIX_NAN : (float)((double)w * (1.0 / FIX_BWD_SCALE));
        acc[r.acc_off + i] = 0ull;
    }
}

// y = (x - mean) * invstd * g + b per row; stats[row] = (mean, invstd); one wave per row, D <= 1024, D % 4 == 0
__global__ __launch_bounds__(256) void layernorm_kernel(const float* __restrict__ x, int64_t T, int D, const float* __restrict__ g,
                                                        const float* __restrict__ b, float* __restrict__ y, uint16_t* __restrict__ y16,
                                                        float* __restrict__ stats) {
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int lane = threadIdx.x & 63;
    f32x4 v[4];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = 4 * (lane + 64 * i);
        v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (c < D) v[i] = *reinterpret_cast<const f32x4*>(x + t * D + c);
        s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
    }
    const float mean = wsum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = 4 * (lane + 64 * i);
        if (c < D)
#pragma unroll
            for (int j = 0; j < 4; ++j) q += (v[i][j] - mean) * (v[i][j] - mean);
    }
    const float inv = 1.f / sqrtf(wsum(q) / (float)D + LN_EPS);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = 4 * (lane + 64 * i);
        if (c < D) {
            const f32x4 gg = *reinterpret_cast<const f32x4*>(g + c), bb = *reinterpret_cast<const f32x4*>(b + c);
            f32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = (v[i][j] - mean) * inv * gg[j] + bb[j];
            *reinterpret_cast<f32x4*>(y + t * D + c) = o;
            if (y16) store_bf16x4(y16 + t * D + c, o);
        }
    }
    if (stats && lane == 0) {
        stats[2 * t] = mean;
        stats[2 * t + 1] = inv;
    }
}

// dx = inv * (dxh - mean(dxh) - xhat * mean(dxh * xhat)), dxh = dy * g.  A wave walks `rows_per_wave` rows and keeps
// the column sums of dy * xhat and dy for its channels in registers; the four waves fold theirs through LDS and the
// workgroup writes one row part[blockIdx.x][0 .. D) = sum dy * xhat, [D .. 2D) = sum dy and, with sum_dx, [2D .. 3D) = sum dx
// (the gradient of a bias added just before the normalised tensor).
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const float* __restrict__ dy, const float* __restrict__ x,
                                                            const float* __restrict__ stats, int64_t T, int D, const float* __restrict__ g,
                                                            float* __restrict__ dx, uint16_t* __restrict__ dx16, float* __restrict__ part,
                                                            int rows_per_wave, int sum_dx) {
    __shared__ float red[4][3 * 1024];
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t t0 = w * rows_per_wave, t1 = t0 + rows_per_wave < T ? t0 + rows_per_wave : T;
    f32x4 sg[4], sb[4], sx[4], gg[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        sg[i] = sb[i] = sx[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int c = 4 * (lane + 64 * i);
        gg[i] = c < D ? *reinterpret_cast<const f32x4*>(g + c) : sg[i];
    }
    for (int64_t t = t0; t < t1; ++t) {
        const float mean = stats[2 * t], inv = stats[2 * t + 1];
        f32x4 xh[4], dh[4];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = 4 * (lane + 64 * i);
            xh[i] = dh[i] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (c < D) {
                const f32x4 xv = *reinterpret_cast<const f32x4*>(x + t * D + c), dv = *reinterpret_cast<const f32x4*>(dy + t * D + c);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    xh[i][j] = (xv[j] - mean) * inv;
                    dh[i][j] = dv[j] * gg[i][j];
                    s1 += dh[i][j];
                    s2 += dh[i][j] * xh[i][j];
                    sg[i][j] += dv[j] * xh[i][j];
                    sb[i][j] += dv[j];
                }
            }
        }
        const float m1 = wsum(s1) / (float)D, m2 = wsum(s2) / (float)D;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = 4 * (lane + 64 * i);
            if (c < D) {
                f32x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = inv * (dh[i][j] - m1 - xh[i][j] * m2);
                sx[i] += o;
                *reinterpret_cast<f32x4*>(dx + t * D + c) = o;
                if (dx16) store_bf16x4(dx16 + t * D + c, o);
            }
        }
    }
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = 4 * (lane + 64 * i);
        if (c < D)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                red[wave][c + j] = sg[i][j];
                red[wave][D + c + j] = sb[i][j];
                red[wave][2 * D + c + j] = sx[i][j];
            }
    }
    __syncthreads();
    const int width = (sum_dx ? 3 : 2) * D;
    for (int c = threadIdx.x; c < width; c += 256) part[(int64_t)blockIdx.x * width + c] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
}

// row <- softmax(row), in place when store_f32 is set, and/or as bf16 into p16; one wave per row of length n <= 1024
__global__ __launch_bounds__(256) void softmax_rows_kernel(float* __restrict__ s, uint16_t* __restrict__ p16, int store_f32, int64_t rows,
                                                           int n) {
    const int64_t rrow = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (rrow >= rows) return;
    const int lane = threadIdx.x & 63;
    float* p = s + rrow * n;
    float v[16];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = lane + 64 * i;
        v[i] = c < n ? p[c] : -INFINITY;
        m = fmaxf(m, v[i]);
    }
    m = wmax(m);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        v[i] = lane + 64 * i < n ? expf(v[i] - m) : 0.f;
        sum += v[i];
    }
    sum = wsum(sum);
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (lane + 64 * i < n) {
            const float q = v[i] / sum;
            if (store_f32) p[lane + 64 * i] = q;
            if (p16) p16[rrow * n + lane + 64 * i] = to_bf16(q);
        }
}

// The same for rows of n <= 4 * LPR values with n % 4 == 0: LPR lanes per row, one 16-byte load each, 64 / LPR rows per wave.
template <int LPR>
__global__ __launch_bounds__(256) void softmax_short_rows_kernel(float* __restrict__ s, uint16_t* __restrict__ p16, int store_f32, int64_t rows,
                                                                 int n) {
    const int lane = threadIdx.x & 63, sub = lane % LPR;
    const int64_t rrow = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * (64 / LPR) + lane / LPR;
    const bool live = rrow < rows && 4 * sub < n;
    f32x4 v = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    if (live) v = *reinterpret_cast<const f32x4*>(s + rrow * n + 4 * sub);
    float m = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        v[j] = live ? expf(v[j] - m) : 0.f;
        sum += v[j];
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (!live) return;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = v[j] / sum;
    if (store_f32) *reinterpret_cast<f32x4*>(s + rrow * n + 4 * sub) = v;
    if (p16) store_bf16x4(p16 + rrow * n + 4 * sub, v);
}

// ds = p * (dp - sum_j dp_j p_j) * scale, in place on dp, or as bf16 into ds16 when that is given
__global__ __launch_bounds__(256) void softmax_bwd_rows_kernel(float* __restrict__ dp, const float* __restrict__ p, uint16_t* __restrict__ ds16,
                                                               int64_t rows, int n, float scale) {
    const int64_t rrow = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (rrow >= rows) return;
    const int lane = threadIdx.x & 63;
    float a[16], d[16];
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = lane + 64 * i;
        a[i] = c < n ? p[rrow * n + c] : 0.f;
        d[i] = c < n ? dp[rrow * n + c] : 0.f;
        dot += a[i] * d[i];
    }
    dot = wsum(dot);
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (lane + 64 * i < n) {
            const float q = a[i] * (d[i] - dot) * scale;
            if (ds16) ds16[rrow * n + lane + 64 * i] = to_bf16(q);
            else dp[rrow * n + lane + 64 * i] = q;
        }
}

__device__ __forceinline__ float gelu_df(float x) {
    return 0.5f * (1.f + erff(x * 0.70710678118654752f)) + x * 0.3989422804014327f * expf(-0.5f * x * x);
}
// in place on dg: du = dg * gelu'(u)
__global__ __launch_bounds__(256) void gelu_bwd_kernel(float* __restrict__ dg, const float* __restrict__ u, uint16_t* __restrict__ du16,
                                                       int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const float q = dg[i] * gelu_df(u[i]);
        dg[i] = q;
        if (du16) du16[i] = to_bf16(q);
    }
}

// The same with the column sums of du on the way (the gradient of the bias added before the activation): a workgroup
// owns GB_ROWS rows of 1024 adjacent columns, a thread four of those columns; part[blockIdx.y][n] = its rows' sum.
#define GB_ROWS 32
__global__ __launch_bounds__(256) void gelu_bwd_colsum_kernel(float* __restrict__ dg, const float* __restrict__ u, uint16_t* __restrict__ du16,
                                                              int64_t M, int N, float* __restrict__ part) {
    const int n = 4 * (blockIdx.x * 256 + threadIdx.x);
    if (n >= N) return;
    const int64_t m0 = (int64_t)blockIdx.y * GB_ROWS, m1 = m0 + GB_ROWS < M ? m0 + GB_ROWS : M;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int64_t m = m0; m < m1; ++m) {
        const f32x4 d = *reinterpret_cast<const f32x4*>(dg + m * N + n), uu = *reinterpret_cast<const f32x4*>(u + m * N + n);
        f32x4 q;
#pragma unroll
        for (int j = 0; j < 4; ++j) q[j] = d[j] * gelu_df(uu[j]);
        *reinterpret_cast<f32x4*>(dg + m * N + n) = q;
        if (du16) store_bf16x4(du16 + m * N + n, q);
        sum += q;
    }
    *reinterpret_cast<f32x4*>(part + (int64_t)blockIdx.y * N + n) = sum;
}

// Running (max, sum of exp(z - max)) pairs: fold one value or another pair in.
struct MaxSum {
    float m, s;
};
__device__ __forceinline__ MaxSum fold(MaxSum a, MaxSum b) {
    const float M = fmaxf(a.m, b.m);
    const float fa = a.m == M ? 1.f : expf(a.m - M), fb = b.m == M ? 1.f : expf(b.m - M);
    return {M, a.s * fa + b.s * fb};
}

// One workgroup per token row of logits [T][V]: tok_loss[t] = logsumexp(z) - z[target], with the maximum and the sum
// taken in one pass over the row (each thread keeps a running pair, pairs are folded in a fixed order).  With
// grad_scale != 0 the gradient (softmax(z) - onehot(target)) * grad_scale then overwrites the row, or goes to d16 as bf16
// when that is given (the logits stay).
__global__ __launch_bounds__(256) void token_ce_kernel(float* __restrict__ logits, const int32_t* __restrict__ targets, int V,
                                                       float* __restrict__ tok_loss, float grad_scale, uint16_t* __restrict__ d16) {
    __shared__ MaxSum red[4];
    const int64_t t = blockIdx.x;
    float* z = logits + t * (int64_t)V;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    MaxSum acc = {-INFINITY, 0.f};
    const bool vec = (V & 3) == 0;   // rows then start on 16-byte boundaries
    if (vec) {
        // four loads in flight per thread; the running pair takes them in order
        auto take = [&](f32x4 v) {
            const float m4 = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
            if (m4 > acc.m) {
                acc.s *= expf(acc.m - m4);
                acc.m = m4;
            }
            acc.s += (expf(v[0] - acc.m) + expf(v[1] - acc.m)) + (expf(v[2] - acc.m) + expf(v[3] - acc.m));
        };
        int c = 4 * threadIdx.x;
        for (; c + 3072 < V; c += 4096) {
            const f32x4 v0 = *reinterpret_cast<const f32x4*>(z + c), v1 = *reinterpret_cast<const f32x4*>(z + c + 1024),
                        v2 = *reinterpret_cast<const f32x4*>(z + c + 2048), v3 = *reinterpret_cast<const f32x4*>(z + c + 3072);
            take(v0);
            take(v1);
            take(v2);
            take(v3);
        }
        for (; c < V; c += 1024) take(*reinterpret_cast<const f32x4*>(z + c));
    } else {
        for (int c = threadIdx.x; c < V; c += 256) acc = fold(acc, MaxSum{z[c], 1.f});
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc = fold(acc, MaxSum{__shfl_xor(acc.m, o, 64), __shfl_xor(acc.s, o, 64)});
    if (lane == 0) red[wave] = acc;
    __syncthreads();
    acc = fold(fold(red[0], red[1]), fold(red[2], red[3]));
    const float m = acc.m, s = acc.s;
    const int tgt = targets[t];
    if (threadIdx.x == 0) tok_loss[t] = (m + logf(s)) - z[tgt];
    if (grad_scale != 0.f) {
        __syncthreads();  // z[tgt] has been read
        const float inv = 1.f / s;
        if (vec) {
            for (int c = 4 * threadIdx.x; c < V; c += 1024) {
                f32x4 v = *reinterpret_cast<const f32x4*>(z + c);
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = (expf(v[j] - m) * inv - (c + j == tgt ? 1.f : 0.f)) * grad_scale;
                if (d16) store_bf16x4(d16 + t * (int64_t)V + c, v);
                else *reinterpret_cast<f32x4*>(z + c) = v;
            }
        } else {
            for (int c = threadIdx.x; c < V; c += 256) {
                const float q = (expf(z[c] - m) * inv - (c == tgt ? 1.f : 0.f)) * grad_scale;
                if (d16) d16[t * (int64_t)V + c] = to_bf16(q);
                else z[c] = q;
            }
        }
    }
}

// Folds the n_parts (max, sum) pairs part[i][t] of every row t: a workgroup takes 64 rows, thread (row, slice) folds the
// pairs slice, slice + 4, ... in order, and the four slices are folded in order through LDS.
__global__ __launch_bounds__(256) void ce_combine_kernel(const float* __restrict__ part, int n_parts, const float* __restrict__ tlogit, int64_t T,
                                                         float* __restrict__ tok_loss, float* __restrict__ row_stats) {
    __shared__ MaxSum red[4][64];
    const int row = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int64_t t = (int64_t)blockIdx.x * 64 + row;
    MaxSum acc = {-INFINITY, 0.f};
    if (t < T)
        for (int i = slice; i < n_parts; i += 4) {
            const sq_f32x2 p = *reinterpret_cast<const sq_f32x2*>(part + 2 * ((int64_t)i * T + t));
            acc = fold(acc, MaxSum{p[0], p[1]});
        }
    red[slice][row] = acc;
    __syncthreads();
    if (slice == 0 && t < T) {
        acc = fold(fold(red[0][row], red[1][row]), fold(red[2][row], red[3][row]));
        tok_loss[t] = (acc.m + logf(acc.s)) - tlogit[t];
        if (row_stats) {
            row_stats[2 * t] = acc.m;
            row_stats[2 * t + 1] = acc.s;
        }
    }
}

__global__ __launch_bounds__(256) void ce_grad_kernel(const float* __restrict__ logits, const int32_t* __restrict__ targets,
                                                      const float* __restrict__ row_stats, int V, float grad_scale, uint16_t* __restrict__ d16) {
    const int64_t t = blockIdx.x;
    const float* z = logits + t * (int64_t)V;
    const float m = row_stats[2 * t], inv = 1.f / row_stats[2 * t + 1];
    const int tgt = targets[t];
    if ((V & 3) == 0) {
        for (int c = 4 * threadIdx.x; c < V; c += 1024) {
            f32x4 v = *reinterpret_cast<const f32x4*>(z + c);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (expf(v[j] - m) * inv - (c + j == tgt ? 1.f : 0.f)) * grad_scale;
            store_bf16x4(d16 + t * (int64_t)V + c, v);
        }
    } else {
        for (int c = threadIdx.x; c < V; c += 256) d16[t * (int64_t)V + c] = to_bf16((expf(z[c] - m) * inv - (c == tgt ? 1.f : 0.f)) * grad_scale);
    }
}

// loss[b] = mean of tok_loss[b*L .. b*L + L); one wave per sample, fixed order
__global__ __launch_bounds__(64) void sample_mean_kernel(const float* __restrict__ tok_loss, int L, float* __restrict__ loss) {
    const int b = blockIdx.x, lane = threadIdx.x;
    float s = 0.f;
    for (int l = lane; l < L; l += 64) s += tok_loss[(int64_t)b * L + l];
    s = wsum(s);
    if (lane == 0) loss[b] = s / (float)L;
}

// out[i] = bf16(in[i]), nearest even: the bf16 copies of the weights
__global__ __launch_bounds__(256) void to_bf16_kernel(const float* __restrict__ in, uint16_t* __restrict__ out, int64_t n4) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256)
        store_bf16x4(out + 4 * i, *reinterpret_cast<const f32x4*>(in + 4 * i));
}

// ---- launchers ---------------------------------------------------------------------------------------
static unsigned nblk(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

void launch_embed(hipStream_t s, const int32_t* tokens, int64_t T, int L, int D, const float* tok, const float* pos, float* h, uint16_t* h16) {
    hipLaunchKernelGGL(embed_kernel, dim3(nblk(T, 4)), dim3(256), 0, s, tokens, T, L, D, tok, pos, h, h16);
}
// n must be a multiple of 4 and both pointers 16- / 8-byte aligned
void launch_to_bf16(hipStream_t s, const float* in, uint16_t* out, int64_t n) {
    unsigned b = nblk(n / 4, 256);
    hipLaunchKernelGGL(to_bf16_kernel, dim3(b > 8192 ? 8192 : b), dim3(256), 0, s, in, out, n / 4);
}
void launch_embed_grad(hipStream_t s, const int32_t* tokens, int64_t T, int D, const float* dh, fixsum_t* acc_tok) {
    double limit = 2305843009213693952.0;   // 2^61
    for (int64_t n = 1; n < T; n <<= 1) limit *= 0.5;
    hipLaunchKernelGGL(embed_grad_kernel, dim3(nblk(T, 4)), dim3(256), 0, s, tokens, T, D, dh, acc_tok, limit);
}
size_t colsum_partial_floats(int64_t M, int N) { return (size_t)nblk(M, 64) * N; }
// out[n] = sum_m X[m][n]; part holds colsum_partial_floats(M, N) floats
void launch_colsum_tokens(hipStream_t s, const float* X, int64_t M, int N, float* part, float* out) {
    if (M <= 64) {
        hipLaunchKernelGGL(colsum_rows_kernel, dim3(nblk(N, 64)), dim3(256), 0, s, X, (int)M, N, out);
        return;
    }
    hipLaunchKernelGGL(colsum_partial_kernel, dim3(nblk(N, 256), nblk(M, 64)), dim3(256), 0, s, X, M, N, part);
    hipLaunchKernelGGL(colsum_rows_kernel, dim3(nblk(N, 64)), dim3(256), 0, s, part, (int)nblk(M, 64), N, out);
}
// First half only: part[r][n] = sum over the 64 rows of chunk r; returns the number of chunks
int launch_colsum_partial(hipStream_t s, const float* X, int64_t M, int N, float* part) {
    hipLaunchKernelGGL(colsum_partial_kernel, dim3(nblk(N, 256), nblk(M, 64)), dim3(256), 0, s, X, M, N, part);
    return (int)nblk(M, 64);
}
// Second half of up to COLSUM_TABLE_MAX column sums in one launch
void launch_colsum_table(hipStream_t s, const ColsumTable& tab, const float* part, float* out) {
    int widest = 1;
    for (int i = 0; i < tab.n; ++i) widest = tab.j[i].N > widest ? tab.j[i].N : widest;
    if (tab.n > 0) hipLaunchKernelGGL(colsum_table_kernel, dim3(nblk(widest, 64), tab.n), dim3(256), 0, s, tab, part, out);
}
void launch_fix_finalize(hipStream_t s, const FixRangeTable& tab, fixsum_t* acc, float* grad) {
    int64_t longest = 1;
    for (int i = 0; i < tab.n; ++i) longest = tab.r[i].n > longest ? tab.r[i].n : longest;
    unsigned bx = nblk(longest, 256);
    if (bx > 2048) bx = 2048;
    hipLaunchKernelGGL(fix_finalize_kernel, dim3(bx, tab.n), dim3(256), 0, s, tab, acc, grad);
}
void launch_layernorm(hipStream_t s, const float* x, int64_t T, int D, const float* g, const float* b, float* y, uint16_t* y16, float* stats) {
    hipLaunchKernelGGL(layernorm_kernel, dim3(nblk(T, 4)), dim3(256), 0, s, x, T, D, g, b, y, y16, stats);
}
#define LN_BWD_ROWS_PER_WAVE 4
size_t layernorm_bwd_partial_floats(int64_t T, int D) { return (size_t)nblk(T, 4 * LN_BWD_ROWS_PER_WAVE) * 3 * D; }
// dgb[0 .. D) = gradient of the scale, dgb[D .. 2D) = gradient of the shift; part holds layernorm_bwd_partial_floats(T, D)
void launch_layernorm_bwd(hipStream_t s, const float* dy, const float* x, const float* stats, int64_t T, int D, const float* g, float* dx,
                          uint16_t* dx16, float* part, float* dgb) {
    const unsigned wgs = nblk(T, 4 * LN_BWD_ROWS_PER_WAVE);
    hipLaunchKernelGGL(layernorm_bwd_kernel, dim3(wgs), dim3(256), 0, s, dy, x, stats, T, D, g, dx, dx16, part, LN_BWD_ROWS_PER_WAVE, 0);
    hipLaunchKernelGGL(colsum_rows_kernel, dim3(nblk(2 * D, 64)), dim3(256), 0, s, part, (int)wgs, 2 * D, dgb);
}
// Without the final sum: part takes one row of (scale, shift, column sum of dx) partials, 3 D floats, per workgroup;
// returns the number of rows
int launch_layernorm_bwd_partial(hipStream_t s, const float* dy, const float* x, const float* stats, int64_t T, int D, const float* g, float* dx,
                                 uint16_t* dx16, float* part) {
    const unsigned wgs = nblk(T, 4 * LN_BWD_ROWS_PER_WAVE);
    hipLaunchKernelGGL(layernorm_bwd_kernel, dim3(wgs), dim3(256), 0, s, dy, x, stats, T, D, g, dx, dx16, part, LN_BWD_ROWS_PER_WAVE, 1);
    return (int)wgs;
}
void launch_softmax_rows(hipStream_t s, float* sc, uint16_t* p16, bool store_f32, int64_t rows, int n) {
    const int f = store_f32 ? 1 : 0;
    if (n % 4 == 0 && n <= 128 && n > 64)
        hipLaunchKernelGGL(softmax_short_rows_kernel<32>, dim3(nblk(rows, 8)), dim3(256), 0, s, sc, p16, f, rows, n);
    else if (n % 4 == 0 && n <= 64)
        hipLaunchKernelGGL(softmax_short_rows_kernel<16>, dim3(nblk(rows, 16)), dim3(256), 0, s, sc, p16, f, rows, n);
    else
        hipLaunchKernelGGL(softmax_rows_kernel, dim3(nblk(rows, 4)), dim3(256), 0, s, sc, p16, f, rows, n);
}
void launch_softmax_bwd_rows(hipStream_t s, float* dp, const float* p, uint16_t* ds16, int64_t rows, int n, float scale) {
    hipLaunchKernelGGL(softmax_bwd_rows_kernel, dim3(nblk(rows, 4)), dim3(256), 0, s, dp, p, ds16, rows, n, scale);
}
void launch_gelu_bwd(hipStream_t s, float* dg, const float* u, uint16_t* du16, int64_t n) {
    unsigned b = nblk(n, 256);
    hipLaunchKernelGGL(gelu_bwd_kernel, dim3(b > 8192 ? 8192 : b), dim3(256), 0, s, dg, u, du16, n);
}
size_t gelu_bwd_colsum_floats(int64_t M, int N) { return (size_t)nblk(M, GB_ROWS) * N; }
// dg[M][N] in place and the partial column sums of the result, gelu_bwd_colsum_floats(M, N) floats; N % 4 == 0 and 16-byte
// aligned pointers (8 for du16) or nothing is launched and 0 comes back; otherwise the number of rows of part
int launch_gelu_bwd_colsum(hipStream_t s, float* dg, const float* u, uint16_t* du16, int64_t M, int N, float* part) {
    auto al = [](const void* p, int bytes) { return (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0; };
    if (N % 4 != 0 || !al(dg, 16) || !al(u, 16) || !al(du16, 8) || !al(part, 16)) return 0;
    hipLaunchKernelGGL(gelu_bwd_colsum_kernel, dim3(nblk(N, 1024), nblk(M, GB_ROWS)), dim3(256), 0, s, dg, u, du16, M, N, part);
    return (int)nblk(M, GB_ROWS);
}
void launch_token_ce(hipStream_t s, float* logits, const int32_t* targets, int64_t T, int V, float* tok_loss, float grad_scale, uint16_t* d16) {
    hipLaunchKernelGGL(token_ce_kernel, dim3((unsigned)T), dim3(256), 0, s, logits, targets, V, tok_loss, grad_scale, d16);
}
void launch_ce_combine(hipStream_t s, const float* ce_part, int n_parts, const float* tlogit, int64_t T, float* tok_loss, float* row_stats) {
    hipLaunchKernelGGL(ce_combine_kernel, dim3(nblk(T, 64)), dim3(256), 0, s, ce_part, n_parts, tlogit, T, tok_loss, row_stats);
}
void launch_ce_grad(hipStream_t s, const float* logits, const int32_t* targets, const float* row_stats, int64_t T, int V, float grad_scale,
                    uint16_t* d16) {
    hipLaunchKernelGGL(ce_grad_kernel, dim3((unsigned)T), dim3(256), 0, s, logits, targets, row_stats, V, grad_scale, d16);
}
void launch_sample_mean(hipStream_t s, const float* tok_loss, int B, int L, float* loss) {
    hipLaunchKernelGGL(sample_mean_kernel, dim3(B), dim3(64), 0, s, tok_loss, L, loss);
}
