// Self-attention of one (sample, head) per workgroup with bf16 factors: scores, softmax and the weighted sum of the
// values without a round trip of the L x L scores through memory.
//   S = alpha * Q K^T (fp32 sums),  P = softmax over each row of S,  ctx = bf16(P) V (fp32 sums), stored as bf16.
// Q, K, V are bf16 slices [L][dh] of [tokens][ld] tensors (head h at column h * dh); L <= 128, L % 8 == 0, dh = 32 or 64.
// The probabilities can be kept for the backward pass as fp32 (P) and bf16 (P16), both [B][H][L][L].
//
// Four waves; wave w owns rows 32 w .. 32 w + 31.  v_mfma_f32_16x16x32_bf16 with the key (value) tile as first operand,
// so that lane (r, g) holds row r, columns 4 g .. 4 g + 3 of a 16 x 16 block: a row of S lives in four lanes and its
// softmax needs two shuffles.  LDS: Q and K as [row][dh + 16] (row pitches of 32 bytes more than a multiple of 64 let the
// 16-byte operand reads run at the full LDS rate), V transposed to [d][128 + 16] (pairs of rows interleaved on the way
// in), and P as [row][128 + 16] in the space Q and K occupied.
#include "act.h"
#include "kernels.h"

typedef __bf16 at_bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 at_bf16x8 __attribute__((ext_vector_type(8)));
typedef float at_f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t at_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t at_u32x2 __attribute__((ext_vector_type(2)));

#define AT_L 128          // rows and columns of the padded score tile
#define AT_PP (AT_L + 16) // pitch of P and of the transposed V, in bf16 elements: 288 bytes

__device__ __forceinline__ uint32_t at_pack(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((at_f32x2){lo, hi}, at_bf16x2));
}

template <int DH>
__global__ __launch_bounds__(256) void attention16_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                          int ld, int H, int L, float alpha, bf16_t* __restrict__ ctx, int ldc,
                                                          float* __restrict__ P, bf16_t* __restrict__ P16) {
    constexpr int PQ = DH + 16;                                   // pitch of Q and K
    constexpr int QK_ELEMS = 2 * AT_L * PQ, P_ELEMS = AT_L * AT_PP;
    constexpr int R0 = QK_ELEMS > P_ELEMS ? QK_ELEMS : P_ELEMS;
    __shared__ __attribute__((aligned(16))) bf16_t lds[R0 + DH * AT_PP];
    bf16_t* Qs = lds;
    bf16_t* Ks = lds + AT_L * PQ;
    bf16_t* Ps = lds;                                             // after the scores are done
    bf16_t* Vt = lds + R0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int b = blockIdx.x / H, h = blockIdx.x - b * H;
    const int64_t row0 = (int64_t)b * L;                          // first token of the sample
    const bf16_t* qh = q + row0 * ld + h * DH;
    const bf16_t* kh = k + row0 * ld + h * DH;
    const bf16_t* vh = v + row0 * ld + h * DH;

    // ---- stage Q, K (rows past L are zero) and V transposed ----------------------------------------------------------
    constexpr int CH = DH / 8;                                    // 16-byte pieces per row
    for (int i = threadIdx.x; i < AT_L * CH; i += 256) {
        const int row = i / CH, c = i - row * CH;
        at_u32x4 a = {0u, 0u, 0u, 0u}, bb = {0u, 0u, 0u, 0u};
        if (row < L) {
            a = *reinterpret_cast<const at_u32x4*>(qh + (int64_t)row * ld + 8 * c);
            bb = *reinterpret_cast<const at_u32x4*>(kh + (int64_t)row * ld + 8 * c);
        }
        *reinterpret_cast<at_u32x4*>(Qs + row * PQ + 8 * c) = a;
        *reinterpret_cast<at_u32x4*>(Ks + row * PQ + 8 * c) = bb;
    }
    for (int i = threadIdx.x; i < (AT_L / 2) * CH; i += 256) {
        const int pair = i / CH, c = i - pair * CH, l2 = 2 * pair;
        at_u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
        if (l2 < L) lo = *reinterpret_cast<const at_u32x4*>(vh + (int64_t)l2 * ld + 8 * c);
        if (l2 + 1 < L) hi = *reinterpret_cast<const at_u32x4*>(vh + (int64_t)(l2 + 1) * ld + 8 * c);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // features 8c + 2j and 8c + 2j + 1: the low and high halves of word j of both rows
            *reinterpret_cast<uint32_t*>(Vt + (8 * c + 2 * j) * AT_PP + l2) = __builtin_amdgcn_perm(hi[j], lo[j], 0x05040100u);
            *reinterpret_cast<uint32_t*>(Vt + (8 * c + 2 * j + 1) * AT_PP + l2) = __builtin_amdgcn_perm(hi[j], lo[j], 0x07060302u);
        }
    }
    __syncthreads();

    // ---- scores: rows 32 wave + 16 mt + r, columns 16 nt + 4 g + i -------------------------------------------------------
    f32x4 s[2][8];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) s[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < DH / 32; ++kk) {
        at_bf16x8 a[2], kb[8];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) a[mt] = *reinterpret_cast<const at_bf16x8*>(Qs + (32 * wave + 16 * mt + r) * PQ + 32 * kk + 8 * g);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) kb[nt] = *reinterpret_cast<const at_bf16x8*>(Ks + (16 * nt + r) * PQ + 32 * kk + 8 * g);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) s[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[nt], a[mt], s[mt][nt], 0, 0, 0);
    }
    // ---- softmax of each row (its 128 columns sit in the four lanes r, r + 16, r + 32, r + 48) ------------------------------
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        float mx = -INFINITY;
#pragma unroll
        for (int nt = 0; nt < 8; ++nt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float z = 16 * nt + 4 * g + i < L ? s[mt][nt][i] * alpha : -INFINITY;
                s[mt][nt][i] = z;
                mx = fmaxf(mx, z);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float sum = 0.f;
#pragma unroll
        for (int nt = 0; nt < 8; ++nt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float e = __expf(s[mt][nt][i] - mx);
                s[mt][nt][i] = e;
                sum += e;
            }
        sum += __shfl_xor(sum, 16, 64);
        sum += __shfl_xor(sum, 32, 64);
        const float inv = 1.f / sum;
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) s[mt][nt] = s[mt][nt] * inv;
    }
    __syncthreads();   // every wave has read Q and K: their space takes P
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int m = 32 * wave + 16 * mt + r;
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
            const int n = 16 * nt + 4 * g;
            const at_u32x2 packed = {at_pack(s[mt][nt][0], s[mt][nt][1]), at_pack(s[mt][nt][2], s[mt][nt][3])};
            *reinterpret_cast<at_u32x2*>(Ps + m * AT_PP + n) = packed;
            if (m < L && n < L) {   // L % 8 == 0, so a quad is inside or outside as a whole
                const int64_t at = ((int64_t)blockIdx.x * L + m) * L + n;
                if (P) *reinterpret_cast<f32x4*>(P + at) = s[mt][nt];
                if (P16) *reinterpret_cast<at_u32x2*>(P16 + at) = packed;
            }
        }
    }
    __syncthreads();

    // ---- ctx = P V: rows as above, columns 16 nt + 4 g + i of the head ------------------------------------------------------
    f32x4 o[2][DH / 16];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < DH / 16; ++nt) o[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < AT_L / 32; ++kk) {
        at_bf16x8 a[2], vb[DH / 16];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) a[mt] = *reinterpret_cast<const at_bf16x8*>(Ps + (32 * wave + 16 * mt + r) * AT_PP + 32 * kk + 8 * g);
#pragma unroll
        for (int nt = 0; nt < DH / 16; ++nt) vb[nt] = *reinterpret_cast<const at_bf16x8*>(Vt + (16 * nt + r) * AT_PP + 32 * kk + 8 * g);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < DH / 16; ++nt) o[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vb[nt], a[mt], o[mt][nt], 0, 0, 0);
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int m = 32 * wave + 16 * mt + r;
        if (m < L)
#pragma unroll
            for (int nt = 0; nt < DH / 16; ++nt) {
                const at_u32x2 packed = {at_pack(o[mt][nt][0], o[mt][nt][1]), at_pack(o[mt][nt][2], o[mt][nt][3])};
                *reinterpret_cast<at_u32x2*>(ctx + (row0 + m) * ldc + h * DH + 16 * nt + 4 * g) = packed;
            }
    }
}

// ---- backward -----------------------------------------------------------------------------------------------------------
// Gradients of one (sample, head) from dctx (bf16) and the probabilities the forward pass kept (fp32):
//   dv = bf16(P)^T dctx,   dP = dctx v^T,   dS = alpha * P * (dP - rowsum(dP * P)),   dq = bf16(dS) k,   dk = bf16(dS)^T q,
// each product with bf16 factors and fp32 sums; dq, dk, dv go out as fp32 and as bf16 ([tokens][ld] slices like q, k, v).
// Same wave and lane layout as the forward kernel.  dP and dS live in registers; bf16(P) and bf16(dS) pass through
// LDS once row-major or transposed, as the product that reads them needs, in the space the dctx and v tiles occupied;
// the [L][dh] factor of each product is transposed on its way into a second LDS region (its global loads are issued
// one product ahead).

template <int DH>
struct AtT {   // a transposed [dh][128 + 16] operand: pieces of two rows per thread
    static constexpr int CH = DH / 8, TASKS = (AT_L / 2) * CH / 256;
    at_u32x4 lo[TASKS], hi[TASKS];
    __device__ __forceinline__ void load(const bf16_t* __restrict__ src, int ld, int L) {
#pragma unroll
        for (int t = 0; t < TASKS; ++t) {
            const int i = threadIdx.x + 256 * t, pair = i / CH, c = i - pair * CH, l2 = 2 * pair;
            lo[t] = at_u32x4{0u, 0u, 0u, 0u};
            hi[t] = at_u32x4{0u, 0u, 0u, 0u};
            if (l2 < L) lo[t] = *reinterpret_cast<const at_u32x4*>(src + (int64_t)l2 * ld + 8 * c);
            if (l2 + 1 < L) hi[t] = *reinterpret_cast<const at_u32x4*>(src + (int64_t)(l2 + 1) * ld + 8 * c);
        }
    }
    __device__ __forceinline__ void put(bf16_t* __restrict__ dst) const {
#pragma unroll
        for (int t = 0; t < TASKS; ++t) {
            const int i = threadIdx.x + 256 * t, pair = i / CH, c = i - pair * CH, l2 = 2 * pair;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                *reinterpret_cast<uint32_t*>(dst + (8 * c + 2 * j) * AT_PP + l2) = __builtin_amdgcn_perm(hi[t][j], lo[t][j], 0x05040100u);
                *reinterpret_cast<uint32_t*>(dst + (8 * c + 2 * j + 1) * AT_PP + l2) = __builtin_amdgcn_perm(hi[t][j], lo[t][j], 0x07060302u);
            }
        }
    }
};

// out[row][16 nt + 4 g + i] = sum_k X[row][k] Yt[16 nt + ..][k] over the 128 (padded) k, rows 32 wave + 16 mt + r; stored as fp32 and bf16
template <int DH>
__device__ __forceinline__ void at_product_store(const bf16_t* __restrict__ X, const bf16_t* __restrict__ Yt, int wave, int r, int g, int L,
                                                 float* __restrict__ out, bf16_t* __restrict__ out16, int ldo, float* __restrict__ colsum) {
    f32x4 o[2][DH / 16];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < DH / 16; ++nt) o[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < AT_L / 32; ++kk) {
        at_bf16x8 a[2], yb[DH / 16];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) a[mt] = *reinterpret_cast<const at_bf16x8*>(X + (32 * wave + 16 * mt + r) * AT_PP + 32 * kk + 8 * g);
#pragma unroll
        for (int nt = 0; nt < DH / 16; ++nt) yb[nt] = *reinterpret_cast<const at_bf16x8*>(Yt + (16 * nt + r) * AT_PP + 32 * kk + 8 * g);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < DH / 16; ++nt) o[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(yb[nt], a[mt], o[mt][nt], 0, 0, 0);
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int row = 32 * wave + 16 * mt + r;
        if (row < L)
#pragma unroll
            for (int nt = 0; nt < DH / 16; ++nt) {
                const int64_t at = (int64_t)row * ldo + 16 * nt + 4 * g;
                *reinterpret_cast<f32x4*>(out + at) = o[mt][nt];
                *reinterpret_cast<at_u32x2*>(out16 + at) = at_u32x2{at_pack(o[mt][nt][0], o[mt][nt][1]), at_pack(o[mt][nt][2], o[mt][nt][3])};
            }
    }
    if (colsum) {
        // sum over the wave's 32 rows (rows past L are exact zeros): the two row blocks, then the 16 lanes of a column quad
#pragma unroll
        for (int nt = 0; nt < DH / 16; ++nt) {
            f32x4 c = o[0][nt] + o[1][nt];
#pragma unroll
            for (int sh = 1; sh < 16; sh <<= 1)
#pragma unroll
                for (int i = 0; i < 4; ++i) c[i] += __shfl_xor(c[i], sh, 64);
            if (r == 0) *reinterpret_cast<f32x4*>(colsum + 16 * nt + 4 * g) = c;
        }
    }
}

template <int DH>
__global__ __launch_bounds__(256, 2) void attention16_bwd_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                              const bf16_t* __restrict__ dctx, const float* __restrict__ P, int ld, int H, int L,
                                                              float alpha, float* __restrict__ dq, float* __restrict__ dk, float* __restrict__ dv,
                                                              bf16_t* __restrict__ dq16, bf16_t* __restrict__ dk16, bf16_t* __restrict__ dv16,
                                                              float* __restrict__ colsum) {
    constexpr int PQ = DH + 16;
    constexpr int RC_ELEMS = 2 * AT_L * PQ, P_ELEMS = AT_L * AT_PP;
    constexpr int R0 = RC_ELEMS > P_ELEMS ? RC_ELEMS : P_ELEMS;
    __shared__ __attribute__((aligned(16))) bf16_t lds[R0 + DH * AT_PP];
    bf16_t* dCs = lds;                 // dctx and v rows, for dP
    bf16_t* Vs = lds + AT_L * PQ;
    bf16_t* X = lds;                   // then bf16(P)^T, bf16(dS), bf16(dS)^T in turn
    bf16_t* Yt = lds + R0;             // dctx^T, k^T, q^T in turn
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int b = blockIdx.x / H, h = blockIdx.x - b * H;
    const int64_t head = ((int64_t)b * L) * ld + h * DH;   // first element of the head's slice in a [tokens][ld] tensor
    const float* Ph = P + (int64_t)blockIdx.x * L * L;
    // partial column sums: [3][4 B][H DH], this wave's row and this head's columns
    const int64_t cs_plane = (int64_t)4 * (gridDim.x / H) * H * DH;
    float* cs = colsum ? colsum + ((int64_t)4 * b + wave) * H * DH + h * DH : nullptr;

    constexpr int CH = DH / 8;
    for (int i = threadIdx.x; i < AT_L * CH; i += 256) {
        const int row = i / CH, c = i - row * CH;
        at_u32x4 a = {0u, 0u, 0u, 0u}, bb = {0u, 0u, 0u, 0u};
        if (row < L) {
            a = *reinterpret_cast<const at_u32x4*>(dctx + head + (int64_t)row * ld + 8 * c);
            bb = *reinterpret_cast<const at_u32x4*>(v + head + (int64_t)row * ld + 8 * c);
        }
        *reinterpret_cast<at_u32x4*>(dCs + row * PQ + 8 * c) = a;
        *reinterpret_cast<at_u32x4*>(Vs + row * PQ + 8 * c) = bb;
    }
    AtT<DH> yt;
    yt.load(dctx + head, ld, L);
    yt.put(Yt);
    __syncthreads();
    yt.load(k + head, ld, L);          // in flight until dv is done

    // ---- dP (rows 32 wave + 16 mt + r, columns 16 nt + 4 g + i), then dS and bf16(P), both packed --------------------------
    at_u32x2 p16[2][8], ds16[2][8];
    {
        f32x4 s[2][8];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) s[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < DH / 32; ++kk) {
            at_bf16x8 a[2], vb[8];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) a[mt] = *reinterpret_cast<const at_bf16x8*>(dCs + (32 * wave + 16 * mt + r) * PQ + 32 * kk + 8 * g);
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) vb[nt] = *reinterpret_cast<const at_bf16x8*>(Vs + (16 * nt + r) * PQ + 32 * kk + 8 * g);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) s[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vb[nt], a[mt], s[mt][nt], 0, 0, 0);
        }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const int m = 32 * wave + 16 * mt + r;
            f32x4 p[8];
            float dot = 0.f;
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) {
                const int n = 16 * nt + 4 * g;
                p[nt] = (m < L && n < L) ? *reinterpret_cast<const f32x4*>(Ph + (int64_t)m * L + n) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < 4; ++i) dot += p[nt][i] * s[mt][nt][i];
            }
            dot += __shfl_xor(dot, 16, 64);
            dot += __shfl_xor(dot, 32, 64);
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) {
                const f32x4 d = p[nt] * (s[mt][nt] - dot) * alpha;
                p16[mt][nt] = at_u32x2{at_pack(p[nt][0], p[nt][1]), at_pack(p[nt][2], p[nt][3])};
                ds16[mt][nt] = at_u32x2{at_pack(d[0], d[1]), at_pack(d[2], d[3])};
            }
        }
    }
    // element (m, n + i) of a packed quad into a transposed [n][m] tile
    auto put_transposed = [&](const at_u32x2 (&w)[2][8]) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const int m = 32 * wave + 16 * mt + r;
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) {
                const int n = 16 * nt + 4 * g;
                X[(n + 0) * AT_PP + m] = (bf16_t)(w[mt][nt][0] & 0xffffu);
                X[(n + 1) * AT_PP + m] = (bf16_t)(w[mt][nt][0] >> 16);
                X[(n + 2) * AT_PP + m] = (bf16_t)(w[mt][nt][1] & 0xffffu);
                X[(n + 3) * AT_PP + m] = (bf16_t)(w[mt][nt][1] >> 16);
            }
        }
    };
    __syncthreads();                   // dctx and v rows are no longer read
    // ---- dv[n][d] = sum_m P[m][n] dctx[m][d] -------------------------------------------------------------------------------
    put_transposed(p16);
    __syncthreads();
    at_product_store<DH>(X, Yt, wave, r, g, L, dv + head, dv16 + head, ld, cs ? cs + 2 * cs_plane : nullptr);
    __syncthreads();
    // ---- dq[m][d] = sum_n dS[m][n] k[n][d] ---------------------------------------------------------------------------------
    yt.put(Yt);
    yt.load(q + head, ld, L);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) *reinterpret_cast<at_u32x2*>(X + (32 * wave + 16 * mt + r) * AT_PP + 16 * nt + 4 * g) = ds16[mt][nt];
    __syncthreads();
    at_product_store<DH>(X, Yt, wave, r, g, L, dq + head, dq16 + head, ld, cs);
    __syncthreads();
    // ---- dk[n][d] = sum_m dS[m][n] q[m][d] ---------------------------------------------------------------------------------
    yt.put(Yt);
    put_transposed(ds16);
    __syncthreads();
    at_product_store<DH>(X, Yt, wave, r, g, L, dk + head, dk16 + head, ld, cs ? cs + cs_plane : nullptr);
}

// Returns false (and launches nothing) for shapes or alignments the kernel does not take.
bool launch_attention16(hipStream_t s, const uint16_t* q, const uint16_t* k, const uint16_t* v, int ld, int B, int H, int L, int dh, float alpha,
                        uint16_t* ctx, int ldc, float* P, uint16_t* P16) {
    auto al = [](const void* p, int bytes) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0; };
    if (L < 8 || L > AT_L || L % 8 != 0 || (dh != 32 && dh != 64) || ld % 8 != 0 || ldc % 4 != 0) return false;
    if (!al(q, 16) || !al(k, 16) || !al(v, 16) || !al(ctx, 8) || !al(P, 16) || !al(P16, 8)) return false;
    if (dh == 64) hipLaunchKernelGGL(attention16_kernel<64>, dim3(B * H), dim3(256), 0, s, q, k, v, ld, H, L, alpha, ctx, ldc, P, P16);
    else hipLaunchKernelGGL(attention16_kernel<32>, dim3(B * H), dim3(256), 0, s, q, k, v, ld, H, L, alpha, ctx, ldc, P, P16);
    return true;
}

bool launch_attention16_bwd(hipStream_t s, const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* dctx, const float* P, int ld, int B,
                            int H, int L, int dh, float alpha, float* dq, float* dk, float* dv, uint16_t* dq16, uint16_t* dk16, uint16_t* dv16,
                            float* colsum) {
    auto al = [](const void* p, int bytes) { return p != nullptr && (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0; };
    if (L < 8 || L > AT_L || L % 8 != 0 || (dh != 32 && dh != 64) || ld % 8 != 0) return false;
    if (!al(q, 16) || !al(k, 16) || !al(v, 16) || !al(dctx, 16) || !al(P, 16) || !al(dq, 16) || !al(dk, 16) || !al(dv, 16) || !al(dq16, 8) ||
        !al(dk16, 8) || !al(dv16, 8) || (reinterpret_cast<uintptr_t>(colsum) & 15) != 0)
        return false;
    if (dh == 64)
        hipLaunchKernelGGL(attention16_bwd_kernel<64>, dim3(B * H), dim3(256), 0, s, q, k, v, dctx, P, ld, H, L, alpha, dq, dk, dv, dq16, dk16, dv16, colsum);
    else
        hipLaunchKernelGGL(attention16_bwd_kernel<32>, dim3(B * H), dim3(256), 0, s, q, k, v, dctx, P, ld, H, L, alpha, dq, dk, dv, dq16, dk16, dv16, colsum);
    return true;
}
