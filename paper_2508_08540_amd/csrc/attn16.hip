// Self-attention of one (sample, head) per workgroup with bf16 factors: scores, softmax and the weighted sum of the
// values without a round trip of the L x L scores through memory.
//   S = alpha * Q K^T (fp32 sums),  P = softmax over each row of S,  ctx = bf16(P) V (fp32 sums), stored as bf16.
// Q, K, V are bf16 slices [L][dh] of [tokens][ld] tensors (head h at column h * dh); L <= 128, L % 8 == 0, dh = 32 or 64.
// The probabilities can be kept for the backward pass as fp32 (P) and bf16 (P16), both [B][H][L][L].
//
// Four waves; wave w owns rows 32 w .. 32 w + 31.  v_mfma_f32_16x16x32_bf16 with the key (value) tile as first operand,
// so that lane (r, g) holds row r, columns 4 g .. 4 g + 3 of a 16 x 16 block: a row of S lives in four lanes and its
// softmax needs two shuffles.  LDS: Q and K as [row][dh + 8] (the padding spreads the 16-byte operand reads over the
// banks), V transposed to [d][128 + 8] (pairs of rows interleaved on the way in), and P as [row][128 + 8] in the space
// Q and K occupied.
#include "act.h"
#include "kernels.h"

typedef __bf16 at_bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 at_bf16x8 __attribute__((ext_vector_type(8)));
typedef float at_f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t at_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t at_u32x2 __attribute__((ext_vector_type(2)));

#define AT_L 128          // rows and columns of the padded score tile
#define AT_PP (AT_L + 8)  // pitch of P and of the transposed V, in bf16 elements

__device__ __forceinline__ uint32_t at_pack(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((at_f32x2){lo, hi}, at_bf16x2));
}

template <int DH>
__global__ __launch_bounds__(256) void attention16_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                          int ld, int H, int L, float alpha, bf16_t* __restrict__ ctx, int ldc,
                                                          float* __restrict__ P, bf16_t* __restrict__ P16) {
    constexpr int PQ = DH + 8;                                    // pitch of Q and K
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
                const float e = expf(s[mt][nt][i] - mx);
                s[mt][nt][i] = e;
                sum += e;
            }
        sum += __shfl_xor(sum, 16, 64);
        sum += __shfl_xor(sum, 32, 64);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) s[mt][nt] = s[mt][nt] / sum;
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
