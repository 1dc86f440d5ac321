// 3x3 convolutions (padding 1, stride 1 or 2) as implicit GEMMs on the fp32 matrix cores, NHWC.
//
// Forward / input gradient (conv_kernel).  A workgroup owns 4 consecutive output rows (all columns; more rows when maps are narrower than 8)
// and stages the input rows they touch, with a zero halo, into LDS as [row][col][C_in + 4]; the
// 4-float pad spreads consecutive pixels over all LDS banks for 16-byte reads.  Each wavefront keeps
// the weights of one block of 16 output channels in registers for the whole kernel (9*C_in/4 VGPRs)
// and walks 16-pixel tiles: v_mfma_f32_16x16x4_f32 with A = weights (row = output channel) and
// B = pixels (column = pixel), so lane l ends with 4 consecutive channels of pixel (l % 16) and
// stores them with one 16-byte write.  Lane group g = l / 16 supplies input channels 16s+4g .. +3
// of a tap as one 16-byte LDS read that feeds four MFMAs (the K order inside a tap is free as long
// as both operands agree).  The epilogue optionally reduces per-channel sum and sum of squares of
// the tile for batch normalisation (fixed shuffle tree, fixed wave order, then order-independent
// fixed-point integer atomics across workgroups).
// The input gradient of a stride-1 layer is the same kernel with weights read transposed and
// flipped; for a stride-2 layer the upstream gradient is staged with zeros inserted between
// samples, which turns the transposed convolution into a stride-1 one.
//
// Weight gradient (wgrad_kernel).  dW[o][tap][i] = sum_pixels dy[p][o] * x[p + tap][i] is a GEMM with
// K = B*H*W: see the comment above that kernel.
//
// Storage type.  All kernels are templates on the type T activations are stored in.  With bf16 the tile
// in LDS and the packed weights are bf16 too (half the bytes everywhere), the same lane-to-channel
// assignment feeds v_mfma_f32_16x16x16_bf16 (one instruction per tap and 16 input channels instead of four),
// accumulation stays fp32 and results are rounded to bf16 once, at the store; the reductions of the epilogue
// see the rounded values, i.e. exactly what later kernels read back.  The weight gradient converts
// bf16 operands to fp32 while staging and runs the fp32 instruction, so master-weight gradients keep fp32
// products.
#include "conv_tile.h"

// The same staging split in two for software pipelining: tile_load issues the global loads of a tile into
// registers (column per thread, up to PRE_ROWS rows), tile_store writes them to an LDS buffer later.
#define PRE_ROWS 12
template <typename T, int CIN>
__device__ __forceinline__ void tile_load(typename Tile<T>::vec16 (&v)[PRE_ROWS], const T* __restrict__ x, const ConvGeom& g, int tile) {
    constexpr int CQ = CIN / 4 / Tile<T>::VQ;  // 16-byte columns per pixel
    constexpr int CQ_LOG2 = clog2(CQ);
    constexpr int pitch = CIN;
    const int rpi = 1 << g.rpi_log2;
    const int row0 = tile * g.rows_tile;
    const int rows_total = g.imgs * g.in_rows;
    const int src_h = g.ups ? (g.h_in >> 1) : g.h_in;
    const int col = threadIdx.x;
    const int cq = col & (CQ - 1), lc = col >> CQ_LOG2;
    const int wi = lc - g.pad;
    bool wok = col < g.lw * CQ && (unsigned)wi < (unsigned)g.h_in;
    int wsrc = wi;
    if (g.ups) {
        wok = wok && ((wi & 1) == 0);
        wsrc = wi >> 1;
    }
    const T* colp = x + (int64_t)(wok ? wsrc : 0) * pitch + cq * (4 * Tile<T>::VQ);
#pragma unroll
    for (int r = 0; r < PRE_ROWS; ++r) {
        const int part = r / g.in_rows, li = r - part * g.in_rows;  // wave-uniform
        const int grow = row0 + part * rpi;
        const int n = grow >> g.wout_log2;
        const int hi = (grow & (g.h_out - 1)) * g.stride - g.pad + li;
        bool ok = r < rows_total && n < g.B && (unsigned)hi < (unsigned)g.h_in && wok;
        int hsrc = hi;
        if (g.ups) {
            ok = ok && ((hi & 1) == 0);
            hsrc = hi >> 1;
        }
        v[r] = Tile<T>::zero16();
        if (ok) v[r] = *reinterpret_cast<const typename Tile<T>::vec16*>(colp + ((int64_t)n * src_h + hsrc) * src_h * pitch);
    }
}

template <typename T, int CIN>
__device__ __forceinline__ void tile_store(const typename Tile<T>::vec16 (&v)[PRE_ROWS], typename Tile<T>::quad* __restrict__ ldsq,
                                           const ConvGeom& g) {
    constexpr int CPQ = CIN / 4 + 1, CQ = CIN / 4 / Tile<T>::VQ;
    constexpr int CQ_LOG2 = clog2(CQ);
    const int col = threadIdx.x;
    if (col >= g.lw * CQ) return;
    const int rows_total = g.imgs * g.in_rows;
    typename Tile<T>::quad* dst = ldsq + (col >> CQ_LOG2) * CPQ + (col & (CQ - 1)) * Tile<T>::VQ;
#pragma unroll
    for (int r = 0; r < PRE_ROWS; ++r)
        if (r < rows_total) Tile<T>::store16(dst + r * g.lw * CPQ, v[r]);
}

// MFMAs, epilogue and store of one staged tile for this wave.
// ---- batch norm + ReLU of the layer below applied while staging (training forward) ------------------------------------
// s_bn[0..3][c] = mean, 1/std, scale, shift of input channel c.  The arithmetic is bn_apply_kernel's, so the staged and
// the stored values are the ones that kernel would have written.
__device__ __forceinline__ f32x4 bn_relu4(f32x4 v, f32x4 res, const float (&k)[4][4]) {
    f32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float t = __fmaf_rn((v[j] - k[0][j]) * k[1][j], k[2][j], k[3][j]) + res[j];
        o[j] = relu_keep_nan(t);
    }
    return o;
}
// stage_input with that transform: rows and columns outside the image stay zero; the rows the tile's own output rows
// sit on (everything but the halo) also go to a_out, so that every pixel of the activation is written exactly once.
template <typename T, int CIN, int THREADS, bool RES, int R>
__device__ __forceinline__ void stage_input_bn(typename Tile<T>::quad* __restrict__ lds4, const T* __restrict__ x, const T* __restrict__ res,
                                               const ConvGeom& g, int tile, const float (*s_bn)[64], T* __restrict__ a_out,
                                               int res_c, int res_lo, int res_stride) {
    typedef typename Act<T>::raw4 raw4;
    constexpr int CP4 = (CIN + 4) / 4, CQ = CIN / 4;
    constexpr int CQ_LOG2 = clog2(CQ);
    const int res_h = g.h_in * res_stride;
    const int rpi = 1 << g.rpi_log2;
    const int row0 = tile * g.rows_tile;
    const int n_cols = g.lw * CQ;
    const int rows_total = g.imgs * g.in_rows;
    for (int col = threadIdx.x; col < n_cols; col += THREADS) {
        const int cq = col & (CQ - 1), lc = col >> CQ_LOG2;
        const int wi = lc - g.pad;
        const bool wok = (unsigned)wi < (unsigned)g.h_in;
        const int64_t colo = (int64_t)(wok ? wi : 0) * CIN + cq * 4;
        // the shortcut covers channels res_lo .. res_lo + res_c of x and is read at every res_stride-th pixel
        const bool rch = RES && cq * 4 >= res_lo && cq * 4 < res_lo + res_c;
        const int64_t rcolo = (int64_t)(wok ? wi : 0) * res_stride * res_c + (cq * 4 - res_lo);
        typename Tile<T>::quad* dst = lds4 + lc * CP4 + cq;
        float k_bn[4][4];   // the column's four channels' constants, read once
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int j = 0; j < 4; ++j) k_bn[a][j] = s_bn[a][cq * 4 + j];
        int part0 = 0, li0 = 0;   // image part and row inside it of row r0
        for (int r0 = 0; r0 < rows_total; r0 += R, li0 += R) {
            while (li0 >= g.in_rows) {
                li0 -= g.in_rows;
                ++part0;
            }
            raw4 v[R], vr[R];
            int64_t at[R];
            bool ok[R], inner[R];
            int part = part0, li = li0;                              // of row r0 + r, without a division per row
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int lr = r0 + r;                               // wave-uniform
                const int grow = row0 + part * rpi;
                const int n = grow >> g.wout_log2;
                const int hi = (grow & (g.h_out - 1)) * g.stride - g.pad + li;
                ok[r] = lr < rows_total && n < g.B && (unsigned)hi < (unsigned)g.h_in && wok;
                inner[r] = li >= g.pad && li < g.pad + rpi * g.stride;
                at[r] = ((int64_t)n * g.h_in + hi) * g.h_in * CIN + colo;
                if (++li == g.in_rows) {
                    li = 0;
                    ++part;
                }
                v[r] = vr[r] = Act<T>::zero();
                if (ok[r]) {
                    v[r] = Act<T>::load_raw(x + at[r]);
                    if (rch) vr[r] = Act<T>::load_raw(res + ((int64_t)n * res_h + (int64_t)hi * res_stride) * res_h * res_c + rcolo);
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (r0 + r < rows_total) {
                    raw4 o = v[r];
                    if (ok[r]) {
                        const f32x4 t = bn_relu4(Act<T>::widen(o), Act<T>::widen(vr[r]), k_bn);
                        if constexpr (sizeof(T) == 4) o = t;
                        else o = Act<T>::narrow(t);
                        if (inner[r]) *reinterpret_cast<raw4*>(a_out + at[r]) = o;
                    }
                    dst[(r0 + r) * g.lw * CP4] = o;
                }
        }
    }
}

// ---- batch-norm backward of the layer applied while its input gradient stages dy -----------------------------------------
// s_bw[0..4][c] = sum of g, sum of g * xhat, mean, 1/std, scale of channel c; the expression is bn_bwd_apply_kernel's.
// g is the upstream gradient as the launch of the layer above stored it: already zero where this layer's ReLU is.
__device__ __forceinline__ f32x4 bn_bwd4(f32x4 g, f32x4 v, const float (&k)[5][4], float inv_count) {
    f32x4 r;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float xhat = (v[j] - k[2][j]) * k[3][j];
        r[j] = k[4][j] * k[3][j] * (g[j] - k[0][j] * inv_count - xhat * (k[1][j] * inv_count));
    }
    return r;
}

// Stages dy = batch-norm backward of (dout, y) for the tile, zero outside the image; the rows that are not halo are
// stored to dy_out, every pixel exactly once.
// R rows of loads are in flight per thread and round: five (the 10 rows of an 8-row tile in two rounds), or three for the
// 64-channel launches over several replicas, which have the fewest registers to spare (measured: + 3.5 % on the
// eight-worker round, - 1.5 % on a single worker, which keeps five).
template <typename T, int CIN, int THREADS, int R>
__device__ __forceinline__ void stage_input_bwd(typename Tile<T>::quad* __restrict__ lds4, const T* __restrict__ dout, const T* __restrict__ y,
                                                const ConvGeom& g, int tile, const float (*s_bw)[64], float inv_count, T* __restrict__ dy_out) {
    typedef typename Act<T>::raw4 raw4;
    constexpr int CP4 = (CIN + 4) / 4, CQ = CIN / 4;
    constexpr int CQ_LOG2 = clog2(CQ);
    const int rpi = 1 << g.rpi_log2;
    const int row0 = tile * g.rows_tile;
    const int n_cols = g.lw * CQ;
    const int rows_total = g.imgs * g.in_rows;
    for (int col = threadIdx.x; col < n_cols; col += THREADS) {
        const int cq = col & (CQ - 1), lc = col >> CQ_LOG2;
        const int wi = lc - g.pad;
        // stride-2 layers: dy is read with zeros inserted (g.ups), only even virtual coordinates hold a pixel
        const bool wok = (unsigned)wi < (unsigned)g.h_in && !(g.ups && (wi & 1));
        const int src_h = g.ups ? (g.h_in >> 1) : g.h_in;
        const int64_t colo = (int64_t)(wok ? (g.ups ? wi >> 1 : wi) : 0) * CIN + cq * 4;
        typename Tile<T>::quad* dst = lds4 + lc * CP4 + cq;
        // bf16 storage: the column's four channels' constants are read once (fp32 launches have no registers to spare for
        // them: measured, 1.5 % slower) and once per row otherwise
        float k_col[5][4];
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int a = 0; a < 5; ++a)
#pragma unroll
                for (int j = 0; j < 4; ++j) k_col[a][j] = s_bw[a][cq * 4 + j];
        }
        int part0 = 0, li0 = 0;   // image part and row inside it of row r0
        for (int r0 = 0; r0 < rows_total; r0 += R, li0 += R) {
            while (li0 >= g.in_rows) {
                li0 -= g.in_rows;
                ++part0;
            }
            raw4 vd[R], vy[R];
            int64_t at[R];
            bool ok[R], inner[R];
            int part = part0, li = li0;                              // of row r0 + r, without a division per row
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int lr = r0 + r;                               // wave-uniform
                const int grow = row0 + part * rpi;
                const int n = grow >> g.wout_log2;
                const int hi = (grow & (g.h_out - 1)) - g.pad + li;
                ok[r] = lr < rows_total && n < g.B && (unsigned)hi < (unsigned)g.h_in && wok && !(g.ups && (hi & 1));
                inner[r] = li >= g.pad && li < g.pad + rpi;
                at[r] = ((int64_t)n * src_h + (g.ups ? hi >> 1 : hi)) * src_h * CIN + colo;
                if (++li == g.in_rows) {
                    li = 0;
                    ++part;
                }
                vd[r] = vy[r] = Act<T>::zero();
                if (ok[r]) {
                    vd[r] = Act<T>::load_raw(dout + at[r]);
                    vy[r] = Act<T>::load_raw(y + at[r]);
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (r0 + r < rows_total) {
                    raw4 o = Act<T>::zero();
                    if (ok[r]) {
                        float k_row[5][4];
                        if constexpr (sizeof(T) != 2) {
#pragma unroll
                            for (int a = 0; a < 5; ++a)
#pragma unroll
                                for (int j = 0; j < 4; ++j) k_row[a][j] = s_bw[a][cq * 4 + j];
                        }
                        const f32x4 t = bn_bwd4(Act<T>::widen(vd[r]), Act<T>::widen(vy[r]), sizeof(T) == 2 ? k_col : k_row, inv_count);
                        if constexpr (sizeof(T) == 4) o = t;
                        else o = Act<T>::narrow(t);
                        if (inner[r]) *reinterpret_cast<raw4*>(dy_out + at[r]) = o;
                    }
                    dst[(r0 + r) * g.lw * CP4] = o;
                }
        }
    }
}

// The epilogue's pointers as replica blockIdx.z sees them (`ro` bytes further).
__device__ __forceinline__ void epi_at(ConvEpi& e, int64_t ro) {
    e.sums = rep_at(e.sums, ro); e.sc_g = rep_at(e.sc_g, ro); e.a_prev = rep_at(e.a_prev, ro); e.y_prev = rep_at(e.y_prev, ro);
    e.mean_prev = rep_at(e.mean_prev, ro); e.invstd_prev = rep_at(e.invstd_prev, ro); e.gamma = rep_at(e.gamma, ro); e.beta = rep_at(e.beta, ro);
    e.in_sums = rep_at(e.in_sums, ro); e.in_mean = rep_at(e.in_mean, ro); e.in_invstd = rep_at(e.in_invstd, ro);
    e.in_rmean = rep_at(e.in_rmean, ro); e.in_rvar = rep_at(e.in_rvar, ro); e.in_gamma = rep_at(e.in_gamma, ro); e.in_beta = rep_at(e.in_beta, ro);
    e.in_res = rep_at(e.in_res, ro); e.a_out = rep_at(e.a_out, ro);
    e.bw_dout = rep_at(e.bw_dout, ro); e.bw_y = rep_at(e.bw_y, ro); e.bw_mean = rep_at(e.bw_mean, ro);
    e.bw_invstd = rep_at(e.bw_invstd, ro); e.bw_gamma = rep_at(e.bw_gamma, ro); e.bw_sums = rep_at(e.bw_sums, ro);
    e.bw_dgamma = rep_at(e.bw_dgamma, ro); e.bw_dbeta = rep_at(e.bw_dbeta, ro); e.bw_dy_out = rep_at(e.bw_dy_out, ro);
}

template <typename T, int CIN, int MT, int NW, int EPI>
__device__ __forceinline__ void conv_tile(const typename Tile<T>::quad* __restrict__ lds4, const typename Tile<T>::quad (&wr)[9][CIN / 16],
                                          T* __restrict__ y, const ConvEpi& e, const ConvGeom& g, int tile, f32x4& ssum, f32x4& ssq) {
    typedef typename Tile<T>::quad quad;
    constexpr int CP = CIN + 4, S = CIN / 16;
    const T* sc_g = static_cast<const T*>(e.sc_g);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, grp = lane >> 4;
    const int NO = g.c_out, NOB = NO >> 4;
    const int ob = wave % NOB;
    const int tile_pixels = g.rows_tile << g.wout_log2;
    const int n_groups = tile_pixels / (16 * MT);
    const int64_t pix0 = (int64_t)tile * tile_pixels;
    const int64_t total_pixels = (int64_t)g.total_rows << g.wout_log2;
    // per-channel constants of the epilogue: this lane always owns channels c0 .. c0+3
    const int c0 = ob * 16 + 4 * grp;
    f32x4 ch_mu = {0.f, 0.f, 0.f, 0.f}, ch_is = ch_mu, ch_ga = ch_mu, ch_be = ch_mu;
    if (EPI == 2 || EPI == 3) {
        ch_mu = *reinterpret_cast<const f32x4*>(e.mean_prev + c0);
        ch_is = *reinterpret_cast<const f32x4*>(e.invstd_prev + c0);
    }
    if (EPI == 3) {
        // invstd_prev holds the running variance here
#pragma unroll
        for (int j = 0; j < 4; ++j) ch_is[j] = (float)(1.0 / sqrt((double)ch_is[j] + 1e-5));
        ch_ga = *reinterpret_cast<const f32x4*>(e.gamma + c0);
        ch_be = *reinterpret_cast<const f32x4*>(e.beta + c0);
    }
    for (int mg = wave / NOB; mg < n_groups; mg += NW / NOB) {
        int base[MT];
        f32x4 acc[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            base[m] = pixel_lds_base<CIN>(g, (mg * MT + m) * 16 + r16) / 4 + grp;  // float4 units
            acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        // input gradient: the epilogue's operands (activation and convolution output of the layer below, shortcut
        // gradient) are requested before the MFMA loop so that their latency hides behind it
        typename Act<T>::raw4 pre_a[MT], pre_y[MT], pre_s[MT];
        if (EPI == 2) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const int64_t p = pix0 + (mg * MT + m) * 16 + r16;
                pre_a[m] = pre_y[m] = pre_s[m] = Act<T>::zero();
                if (p < total_pixels) {
                    pre_a[m] = Act<T>::load_raw(static_cast<const T*>(e.a_prev) + p * NO + c0);
                    pre_y[m] = Act<T>::load_raw(static_cast<const T*>(e.y_prev) + p * NO + c0);
                    if (sc_g) {
                        if (e.sc_stride == 1) {
                            pre_s[m] = Act<T>::load_raw(sc_g + p * e.sc_c + c0);
                        } else {
                            const int wq = (int)(p & (g.h_out - 1));
                            const int64_t row = p >> g.wout_log2;
                            const int hq = (int)(row & (g.h_out - 1));
                            if (((wq | hq) & 1) == 0) {
                                const int64_t n = row >> g.wout_log2;
                                const int hs = g.h_out >> 1;
                                pre_s[m] = Act<T>::load_raw(sc_g + ((n * hs + (hq >> 1)) * hs + (wq >> 1)) * e.sc_c + e.sc_lo + c0);
                            }
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int tap_off = ((t / 3) * g.lw + (t % 3)) * (CP / 4);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                quad b[MT];
#pragma unroll
                for (int m = 0; m < MT; ++m) b[m] = lds4[base[m] + tap_off + 4 * s];
                if constexpr (sizeof(T) == 4) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int m = 0; m < MT; ++m)
                            acc[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr[t][s][j], b[m][j], acc[m], 0, 0, 0);
                } else {
                    // K = 16: lane group g supplies channels 16s + 4g .. +3 of both operands
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        acc[m] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, wr[t][s]),
                                                                           __builtin_bit_cast(s16x4, b[m]), acc[m], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            int64_t p = pix0 + (mg * MT + m) * 16 + r16;
            if (p < total_pixels) {
                f32x4 v = acc[m];
                if (EPI == 2) {
                    // gradient that bypassed the block below through its shortcut (zero when there is none)
                    v += Act<T>::widen(pre_s[m]);
                    v = Act<T>::rounded(v);  // the sums below see what later kernels read back
                    const f32x4 av = Act<T>::widen(pre_a[m]);
                    const f32x4 yv = Act<T>::widen(pre_y[m]);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float gq = av[j] > 0.f ? v[j] : 0.f;
                        v[j] = gq;
                        ssum[j] += gq;
                        ssq[j] = __fmaf_rn(gq, (yv[j] - ch_mu[j]) * ch_is[j], ssq[j]);
                    }
                    // what goes out is the gradient behind the ReLU of the layer below: that layer's batch-norm backward, its
                    // block's shortcut and nothing else read it, and none of them has to look the activation up again
                    Act<T>::store4(y + p * NO + c0, v);
                } else if (EPI == 3) {
                    // inference: batch norm with running statistics, shortcut, ReLU
                    f32x4 r = {0.f, 0.f, 0.f, 0.f};
                    if (e.sc_g && c0 >= e.sc_lo && c0 < e.sc_lo + e.sc_c) {
                        int64_t rp = p;
                        if (e.sc_stride != 1) {
                            const int wq = (int)(p & (g.h_out - 1));
                            const int64_t row = p >> g.wout_log2;
                            const int hq = (int)(row & (g.h_out - 1));
                            const int64_t n = row >> g.wout_log2;
                            const int hr = g.h_out * e.sc_stride;
                            rp = (n * hr + (int64_t)hq * e.sc_stride) * hr + (int64_t)wq * e.sc_stride;
                        }
                        r = Act<T>::load4(sc_g + rp * e.sc_c + (c0 - e.sc_lo));
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[j] = relu_keep_nan(__fmaf_rn((v[j] - ch_mu[j]) * ch_is[j], ch_ga[j], ch_be[j]) + r[j]);
                    Act<T>::store4(y + p * NO + c0, v);
                } else {
                    v = Act<T>::rounded(v);
                    Act<T>::store4(y + p * NO + c0, v);
                    ssum += v;
                    ssq += v * v;
                }
            }
        }
    }
}

// `w` is the packed copy of the layer's weights made by pack_weights_kernel (forward or input-gradient form).
// EPI 0: plain store.  EPI 1: also per-channel sum / sum of squares of the output (batch-norm statistics).
// EPI 2 (input gradient): the shortcut gradient is added before the store, and the output is masked by
// the ReLU of the layer below and reduced to the two sums of that layer's batch-norm backward pass.
// For EPI 1 and 2 every workgroup adds its sums into per-channel fixed-point accumulators (integer atomics).
// EPI 3 (inference): batch norm with the running statistics, shortcut add and ReLU are applied before the store.
//
// The grid is persistent: workgroup b handles tiles b, b + gridDim.x, ...  While the MFMAs of one tile
// run from one LDS buffer, the global loads of the next tile are in flight into registers and are then
// written to the other buffer (one barrier per tile).
// XF 1, 2: the input is the raw convolution output of the layer below; its batch norm (XF == 2: plus an identity
// shortcut) and ReLU are applied while staging (ConvEpi::in_sums and the fields after it).  XF 3 (input gradient): the
// input dy is computed while staging, by the layer's batch-norm backward (ConvEpi::bw_dout and the fields after it).
// MULTI: a workgroup may own several tiles; the sums of the epilogue are then folded and converted tile by tile.
template <typename T, int CIN, int MT, int NW, int EPI, int XF, bool MULTI>
__global__ __launch_bounds__(NW * 64, (MULTI && CIN == 64) ? 2 : 1) void conv_kernel(const T* __restrict__ x, const void* __restrict__ w,
                                                            T* __restrict__ y, ConvEpi e, ConvGeom g, int pipelined, int64_t rstride) {
    __builtin_amdgcn_s_setprio(2);   // ahead of the weight-gradient kernels of the side stream, which only the update waits for
    if (rstride) {   // one replica of several: every buffer sits blockIdx.z slots further
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        x = rep_at(x, ro); w = rep_at(w, ro); y = rep_at(y, ro);
        epi_at(e, ro);
    }
    typedef typename Tile<T>::quad quad;
    __shared__ float s_bn[XF == 3 ? 5 : XF ? 4 : 1][64];
    if constexpr (XF == 3) {
        const int c = threadIdx.x;
        if (c < CIN) {
            s_bn[0][c] = (float)((double)fixsum_read(e.bw_sums, CIN, 0, c) * (1.0 / FIX_BWD_SCALE));
            s_bn[1][c] = (float)((double)fixsum_read(e.bw_sums, CIN, 1, c) * (1.0 / FIX_BWD_SCALE));
            s_bn[2][c] = e.bw_mean[c];
            s_bn[3][c] = e.bw_invstd[c];
            s_bn[4][c] = e.bw_gamma[c];
            if (blockIdx.x == 0) {
                const bool bad = fixsum_poisoned(e.bw_sums, CIN, c);   // out of range or not finite: NaN, as a float sum would end
                e.bw_dbeta[c] = bad ? FIX_NAN : s_bn[0][c];
                e.bw_dgamma[c] = bad ? FIX_NAN : s_bn[1][c];
            }
        }
        __syncthreads();
    } else if constexpr (XF != 0) {
        // statistics of the input's batch norm, exactly as bn_apply_kernel derives them
        const int c = threadIdx.x;
        if (c < CIN) {
            const double s1 = (double)fixsum_read(e.in_sums, CIN, 0, c) * (1.0 / FIX_FWD_SCALE);
            const double s2 = (double)fixsum_read(e.in_sums, CIN, 1, c) * (1.0 / FIX_FWD_SCALE);
            double mu = s1 / e.in_count;
            double var = s2 / e.in_count - mu * mu;
            if (var < 0.0) var = 0.0;
            s_bn[0][c] = (float)mu;
            s_bn[1][c] = (float)(1.0 / sqrt(var + BN_EPS));
            s_bn[2][c] = e.in_gamma[c];
            s_bn[3][c] = e.in_beta[c];
            if (blockIdx.x == 0) {
                if (fixsum_poisoned(e.in_sums, CIN, c)) {   // out of range or not finite: NaN, as a float sum would end
                    s_bn[0][c] = s_bn[1][c] = FIX_NAN;
                    mu = var = (double)FIX_NAN;
                }
                e.in_mean[c] = s_bn[0][c];
                e.in_invstd[c] = s_bn[1][c];
                const double unbiased = e.in_count > 1.0 ? var * e.in_count / (e.in_count - 1.0) : var;
                e.in_rmean[c] = (float)((1.0 - BN_MOMENTUM) * (double)e.in_rmean[c] + BN_MOMENTUM * mu);
                e.in_rvar[c] = (float)((1.0 - BN_MOMENTUM) * (double)e.in_rvar[c] + BN_MOMENTUM * unbiased);
            }
        }
        __syncthreads();
    }
    T* a_out = static_cast<T*>(e.a_out);
    const T* in_res = static_cast<const T*>(e.in_res);
    constexpr bool RES = XF == 2;
    extern __shared__ f32x4 lds_raw[];  // vector-typed so that tile reads and writes are single 16- or 8-byte LDS accesses
    quad* lds4 = reinterpret_cast<quad*>(lds_raw);
    constexpr int S = CIN / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, grp = lane >> 4;
    const int NO = g.c_out, NOB = NO >> 4;
    const int ob = wave % NOB;

    // weights of output-channel block `ob` into registers: wr[tap][s] holds input channels 16s+4grp .. +3 of
    // output channel 16*ob + r16, read from the lane-major packed copy (one contiguous 1 KB load each)
    quad wr[9][S];
    {
        const quad* wp = reinterpret_cast<const quad*>(w) + (int64_t)ob * 9 * S * 64 + lane;
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int s = 0; s < S; ++s) wr[t][s] = wp[(t * S + s) * 64];
    }
    f32x4 ssum = {0.f, 0.f, 0.f, 0.f}, ssq = {0.f, 0.f, 0.f, 0.f};
    // Per-channel sums of the epilogue (EPI 1, 2): after every tile the waves fold their lanes (fixed shuffle tree) into
    // red[parity], and after the next barrier thread (which, c) adds the waves in wave order, converts the tile's partial to
    // fixed point and keeps the integer sum; one atomic per thread leaves the workgroup at the end.
    __shared__ float red[2][NW * 2 * 16];
    long long fx_sum = 0;
    bool fx_poisoned = false;
    auto fold_write = [&](int par) {
        // lanes of one group hold the same 4 channels for 16 different pixels: fold the pixels
#pragma unroll
        for (int o = 1; o < 16; o <<= 1)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ssum[j] += __shfl_xor(ssum[j], o, 64);
                ssq[j] += __shfl_xor(ssq[j], o, 64);
            }
        if (r16 == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                red[par][(wave * 2 + 0) * 16 + 4 * grp + j] = ssum[j];
                red[par][(wave * 2 + 1) * 16 + 4 * grp + j] = ssq[j];
            }
        }
        ssum = ssq = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto fold_read = [&](int par) {
        if (threadIdx.x < 2 * NO) {
            const int which = threadIdx.x / NO, c = threadIdx.x % NO;
            const int cb = c >> 4;
            float acc = 0.f;
            for (int wv = cb; wv < NW; wv += NOB) acc += red[par][(wv * 2 + which) * 16 + (c & 15)];
            fixsum_collect(fx_sum, fx_poisoned, (double)acc * e.scale, e.tile_limit);
        }
    };

    // the transforming variants stage without prefetching: their launches have at most one or two tiles per workgroup
    // at the batch sizes of a local step, and the prefetch registers would cost them a wave of occupancy
    if (XF == 0 && pipelined) {
        const int buf_f4 = g.imgs * g.in_rows * g.lw * ((CIN + 4) / 4);
        typename Tile<T>::vec16 pre[PRE_ROWS];
        int tile = blockIdx.x;
        tile_load<T, CIN>(pre, x, g, tile);
        tile_store<T, CIN>(pre, lds4, g);
        __syncthreads();
        for (int it = 0; tile < g.n_tiles; ++it, tile += gridDim.x) {
            const int next = tile + gridDim.x;
            if (next < g.n_tiles) tile_load<T, CIN>(pre, x, g, next);
            conv_tile<T, CIN, MT, NW, EPI>(lds4 + (it & 1) * buf_f4, wr, y, e, g, tile, ssum, ssq);
            if (MULTI && (EPI == 1 || EPI == 2)) fold_write(it & 1);
            if (next < g.n_tiles) tile_store<T, CIN>(pre, lds4 + ((it + 1) & 1) * buf_f4, g);
            __syncthreads();
            if (MULTI && (EPI == 1 || EPI == 2)) fold_read(it & 1);
        }
    } else {
        int it = 0;
        for (int tile = blockIdx.x; tile < g.n_tiles; tile += gridDim.x, ++it) {
            if constexpr (XF == 3)
                stage_input_bwd<T, CIN, NW * 64, (MULTI && CIN == 64) ? 3 : 5>(lds4, static_cast<const T*>(e.bw_dout), static_cast<const T*>(e.bw_y), g, tile, s_bn, e.bw_inv_count,
                                                 static_cast<T*>(e.bw_dy_out));
            else if constexpr (XF != 0) stage_input_bn<T, CIN, NW * 64, RES, (MULTI && CIN == 64) ? 3 : 6>(lds4, x, in_res, g, tile, s_bn, a_out, e.in_res_c, e.in_res_lo, e.in_res_stride);
            else stage_input<T, quad, CIN, NW * 64>(lds4, x, g, tile);
            __syncthreads();
            conv_tile<T, CIN, MT, NW, EPI>(lds4, wr, y, e, g, tile, ssum, ssq);
            if (MULTI && (EPI == 1 || EPI == 2)) fold_write(it & 1);
            __syncthreads();
            if (MULTI && (EPI == 1 || EPI == 2)) fold_read(it & 1);   // the next write into this half of red is two barriers away
        }
    }

    if (!MULTI && (EPI == 1 || EPI == 2)) {   // one tile: its sums are still in the lanes
        fold_write(0);
        __syncthreads();
        fold_read(0);
    }
    // order-independent accumulation across workgroups: 64-bit fixed point, integer atomic add
    if ((EPI == 1 || EPI == 2) && threadIdx.x < 2 * NO) {
        const int which = threadIdx.x / NO, c = threadIdx.x % NO;
        fixsum_flush(e.sums + ((blockIdx.x % FIX_REPLICAS) * 2 + which) * NO + c, fx_sum, fx_poisoned);
    }
}

// Workgroups per launch: at most CONV_GRID_CAP (two per compute unit on a 256-CU part).  With several replicas in one
// launch the cap is shared: a workgroup then walks several tiles of its replica with one set of weights and one prologue
// (and, without a transform on load, with the next tile prefetched), which is where launches of 2048 and more one-tile
// workgroups lost their time.  The sums do not depend on the split (fixsum_collect).
#define CONV_GRID_CAP 512
static int conv_grid(const ConvGeom& g, int replicas) {
    int cap = CONV_GRID_CAP / (replicas < 1 ? 1 : replicas);
    if (cap < 1) cap = 1;
    return g.n_tiles < cap ? g.n_tiles : cap;
}
// One tile's scaled partial sum may reach 2^54 in a launch of up to CONV_GRID_CAP tiles: a word then holds less than 2^59
// and the sum of its FIX_REPLICAS replicas, which the readers take in 64-bit integers, less than 2^63.  Launches of more
// tiles lower the bound per tile in proportion (the same rms per tile, as their tiles are smaller or their batches larger).
static double conv_tile_limit(const ConvGeom& g) {
    double limit = 2.0 * FIX_PARTIAL_LIMIT;
    for (int t = CONV_GRID_CAP; t < g.n_tiles; t *= 2) limit *= 0.5;
    return limit;
}

template <typename T, int CIN, int EPI>
static void launch_conv_t(hipStream_t s, const ConvGeom& g, const T* x, const void* w, T* y, const ConvEpi& e_in,
                          const KernelTiming* kt, Reps reps) {
    constexpr int MT = CONV_MT, NW = CONV_NW;
    ConvEpi e = e_in;
    e.tile_limit = conv_tile_limit(g);
    const int grid = conv_grid(g, reps.n);
    // prefetching needs the whole tile in PRE_ROWS registers per thread, one column per thread, and more
    // than one tile per workgroup to pay off
    bool transforming = false;   // batch norm applied while staging: no prefetching path
    if constexpr (EPI == 1) transforming = e.in_sums != nullptr;
    if constexpr (EPI == 2) transforming = e.bw_dout != nullptr;
    const bool fused_bwd = EPI == 2 && transforming;
    const int pipelined = (!transforming && g.imgs * g.in_rows <= PRE_ROWS && g.lw * (CIN / 4 / Tile<T>::VQ) <= NW * 64 && g.n_tiles > grid) ? 1 : 0;
    size_t lds = input_lds_bytes<T, CIN>(g) * (pipelined ? 2 : 1);
    if ((EPI == 1 || EPI == 2) && lds < 1024) lds = 1024;  // per-wave partial sums
    // a workgroup that owns one tile keeps the epilogue's sums in its lanes until the end; one that owns several folds them
    // tile by tile (inference and plain launches have no sums: one instantiation)
    const bool multi = (EPI == 1 || EPI == 2) && g.n_tiles > grid;
    auto kern = multi ? conv_kernel<T, CIN, MT, NW, EPI, 0, true> : conv_kernel<T, CIN, MT, NW, EPI, 0, false>;
    if constexpr (EPI == 1) {
        if (e.in_sums && e.in_res) kern = multi ? conv_kernel<T, CIN, MT, NW, EPI, 2, true> : conv_kernel<T, CIN, MT, NW, EPI, 2, false>;
        else if (e.in_sums) kern = multi ? conv_kernel<T, CIN, MT, NW, EPI, 1, true> : conv_kernel<T, CIN, MT, NW, EPI, 1, false>;
    }
    if constexpr (EPI == 2) {
        if (fused_bwd) kern = multi ? conv_kernel<T, CIN, MT, NW, EPI, 3, true> : conv_kernel<T, CIN, MT, NW, EPI, 3, false>;
    }
    if (lds > 65536) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    // with timing events the dispatch itself is stamped (start and end of this kernel only)
    hipExtLaunchKernelGGL(kern, dim3(grid, 1, reps.n), dim3(NW * 64), lds, s, kt ? kt->start : nullptr, kt ? kt->stop : nullptr, 0, x, w, y, e, g,
                          pipelined, reps.stride);
}

template <typename T, int EPI>
static void launch_conv_ct(hipStream_t s, int c_in, const ConvGeom& g, const void* x, const void* w, void* y, const ConvEpi& e,
                           const KernelTiming* kt, Reps reps) {
    switch (c_in) {
        case 16: launch_conv_t<T, 16, EPI>(s, g, (const T*)x, w, (T*)y, e, kt, reps); break;
        case 32: launch_conv_t<T, 32, EPI>(s, g, (const T*)x, w, (T*)y, e, kt, reps); break;
        default: launch_conv_t<T, 64, EPI>(s, g, (const T*)x, w, (T*)y, e, kt, reps); break;
    }
}

template <int EPI>
static void launch_conv_c(hipStream_t s, int act, int c_in, const ConvGeom& g, const void* x, const void* w, void* y, const ConvEpi& e,
                          const KernelTiming* kt, Reps reps) {
    if (act == ACT_BF16) launch_conv_ct<bf16_t, EPI>(s, c_in, g, x, w, y, e, kt, reps);
    else launch_conv_ct<float, EPI>(s, c_in, g, x, w, y, e, kt, reps);
}

// ---- weight packing -----------------------------------------------------------------------------------
//
// Lane-major copies of every convolution's weights, rebuilt after each parameter update.  For a layer
// with (padded) input channels CI and output channels CO the forward copy holds, as quad (4 values of the storage type) number
// ((ob*taps + t)*(CI/16) + s)*64 + lane, the values w[16*ob + lane%16][t][16*s + 4*(lane/16) + 0..3] (zero
// beyond the real input channels; taps = 9 for 3x3 and 1 for 1x1 filters).  The input-gradient copy describes
// the transposed convolution: roles of CI and CO swap and the taps are flipped,
// value j = w[16*s + 4*(lane/16) + j][taps - 1 - t][16*ob + lane%16].

template <typename T>
__global__ __launch_bounds__(256) void pack_weights_kernel(const float* __restrict__ params, typename Tile<T>::quad* __restrict__ packed,
                                                           PackTable tab, int64_t rstride) {
    params = rep_at(params, (int64_t)blockIdx.z * rstride);
    packed = rep_at(packed, (int64_t)blockIdx.z * rstride);
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // quad index
    if (i >= tab.total_vec4) return;
    int l = 0;
    while (l + 1 < tab.n && i >= tab.e[l + 1].pack_off) ++l;
    const PackEntry e = tab.e[l];
    int64_t r = i - e.pack_off;
    const int lane = (int)(r & 63);
    r >>= 6;
    const int r16 = lane & 15, grp = lane >> 4;
    const float* w = params + e.w_off;
    f32x4 v;
    const int taps = e.taps;
    if (!e.dgrad) {
        const int S = e.c_in >> 4;
        const int s = (int)(r % S), t = (int)((r / S) % taps), ob = (int)(r / (S * taps));
        const int o = ob * 16 + r16, i0 = 16 * s + 4 * grp;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (i0 + j < e.c_in_real) ? w[((int64_t)o * taps + t) * e.c_in_real + i0 + j] : 0.f;
    } else {
        // transposed convolution: its input channels are the layer's outputs, its outputs the layer's inputs
        const int S = e.c_out >> 4;
        const int s = (int)(r % S), t = (int)((r / S) % taps), ob = (int)(r / (S * taps));
        const int o = ob * 16 + r16, i0 = 16 * s + 4 * grp;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = w[((int64_t)(i0 + j) * taps + (taps - 1 - t)) * e.c_in_real + o];
    }
    Act<T>::store4(reinterpret_cast<T*>(packed + i), v);
}

void launch_pack_weights(hipStream_t s, int act, const float* params, void* packed, const PackTable& tab, Reps reps) {
    int64_t blocks = (tab.total_vec4 + 255) / 256;
    ACT_DISPATCH(act, hipLaunchKernelGGL(pack_weights_kernel<T>, dim3((unsigned)blocks, 1, reps.n), dim3(256), 0, s, params,
                                         (typename Tile<T>::quad*)packed, tab, reps.stride));
}

int conv_fwd_tiles(const ConvShape& cs) {
    int h_out = (cs.h_in - 1) / cs.stride + 1;
    return make_geom(cs.B, cs.h_in, h_out, cs.c_out, cs.stride, 0, cs.c_in_real).n_tiles;
}

#define TALL_MIN_TILES 256
#define FWD_TALL_MIN_H 32
void launch_conv_fwd(hipStream_t s, int act, const ConvShape& cs, const void* x, const void* w, void* y, const ConvEpi* stats,
                     const KernelTiming* kt, Reps reps) {
    int h_out = (cs.h_in - 1) / cs.stride + 1;
    // normalise-on-load and inference launches on the large images: taller tiles, fewer halo rows re-read
    // (only while the launch keeps at least TALL_MIN_TILES workgroups)
    const int rows = (stats && (stats->in_sums || stats->gamma) && cs.stride == 1 && h_out >= FWD_TALL_MIN_H && cs.B * h_out >= 8 * TALL_MIN_TILES) ? 8 : 0;
    ConvGeom g = make_geom(cs.B, cs.h_in, h_out, cs.c_out, cs.stride, 0, cs.c_in_real, rows);
    if (stats && stats->gamma) launch_conv_c<3>(s, act, cs.c_in, g, x, w, y, *stats, kt, reps);
    else if (stats) launch_conv_c<1>(s, act, cs.c_in, g, x, w, y, *stats, kt, reps);
    else launch_conv_c<0>(s, act, cs.c_in, g, x, w, y, ConvEpi{}, kt, reps);
}

#define DGRAD_TALL_MIN_H 16
void launch_conv_dgrad(hipStream_t s, int act, const ConvShape& cs, const void* dy, const void* w, void* dx, const ConvEpi* bn_below,
                       const KernelTiming* kt, Reps reps) {
    // The gradient with respect to the input is a stride-1 convolution whose input channels are the
    // layer's output channels and whose output channels are the layer's input channels.
    int ups = cs.stride == 2 ? 1 : 0;
    // with the batch-norm backward in the staging three tensors are read per tile: taller tiles on the large images
    // (halo rows 2 in 10 instead of 2 in 6)
    const int rows = (bn_below && bn_below->bw_dout && cs.h_in >= DGRAD_TALL_MIN_H && cs.B * cs.h_in >= 8 * TALL_MIN_TILES) ? 8 : 0;
    ConvGeom g = make_geom(cs.B, cs.h_in, cs.h_in, cs.c_in, 1, ups, cs.c_in, rows);
    if (bn_below) launch_conv_c<2>(s, act, cs.c_out, g, dy, w, dx, *bn_below, kt, reps);
    else launch_conv_c<0>(s, act, cs.c_out, g, dy, w, dx, ConvEpi{}, kt, reps);
}

// ---- weight gradient ------------------------------------------------------------------------------
//
// Workgroup (pg, ob, ib) owns the 16x16 block (output channels 16*ob.., input channels 16*ib..) of dW
// for all 9 taps over pixel group pg.  It stages only those 16-channel slices of x and dy, its four
// waves take output rows in turn (9 MFMAs per pixel quad), fold their 9 accumulators through LDS in
// wave order and add the 2304 sums into replicated 64-bit fixed-point accumulators with integer atomics
// (order-independent, hence reproducible).  All layer shapes run the same code; the grid has
// groups * (C_out/16) * (C_in/16) workgroups.

#define WG_BLOCK_FLOATS (16 * 9 * 16)   // one 16x16 channel block of a 3x3 filter; a 1x1 filter has 16 * 16
#define WGRAD_REPLICAS 8
#define FIX_WGRAD_SCALE 1099511627776.0  // 2^40: |dW| < 2^23, resolution 2^-40

#define WGRAD_THREADS 512
#define WG_WAVES (WGRAD_THREADS / 64)
#define WGRAD_GROUP_CAP 512

// PIPE: a thread owns up to WG_XK fixed 4-channel slots of the x tile and WG_DK of the dy tile; the next tile's slots are
// loaded into registers while the current tile multiplies (tiles small enough for that, see wgrad_geom).
#define WG_XK 4
#define WG_XK_STRIDE2 10   // stride-2 layers stage (2 rows + 1) x (2 columns + 2) input pixels per output pixel
#define WG_DK 2
#define WG_PIPE_PIXELS (WGRAD_THREADS / 2)

// MULTI (launches over several replicas): a workgroup takes `groups_per_wg` consecutive pixel groups.  At the end of each
// it folds and converts its sums exactly as a one-group workgroup does and keeps them as integers in registers, the
// prefetch of the next tile runs across the boundary, and one set of atomics leaves at the end: the same bits from an
// eighth of the workgroups, first loads and atomics.
// (the unroll request on the loop over pixel quads is declined in the instantiations where the row width is not known:
// expected, not worth a line per instantiation in every build)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wpass-failed"
template <typename T, int TAPS, bool PIPE, bool MULTI, int XK = WG_XK>
__global__ __launch_bounds__(WGRAD_THREADS) void wgrad_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                              fixsum_t* __restrict__ gacc, ConvGeom g, int tiles_per_group,
                                                              int NI, int NO, int replicas, int64_t rstride, int groups_per_wg) {
    if (rstride) {   // one replica of several: every buffer sits blockIdx.z slots further
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        x = rep_at(x, ro); dy = rep_at(dy, ro); gacc = rep_at(gacc, ro);
    }
    extern __shared__ f32x4 lds4[];
    float* lds = reinterpret_cast<float*>(lds4);
    // pixel pitch 16 floats: the four lane groups of a read (4 consecutive pixels x 16 channels) cover the
    // 32 banks exactly twice, the minimum for 256 bytes
    constexpr int CP = 16, DP = 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, grp = lane >> 4;
    const int NIB = NI >> 4;
    const int ob = blockIdx.y / NIB, ib = blockIdx.y - ob * NIB;
    const int w_out = g.h_out;
    const int tile_pixels = g.rows_tile << g.wout_log2;
    const int64_t total_pixels = (int64_t)g.total_rows << g.wout_log2;
    float* lds_x = lds;
    float* lds_dy = lds + (size_t)g.imgs * g.in_rows * g.lw * CP;

    constexpr int BLOCK_FLOATS = 16 * TAPS * 16;
    f32x4 acc[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int tile_begin = blockIdx.x * tiles_per_group * (MULTI ? groups_per_wg : 1);
    const int tile_end = min(g.n_tiles, tile_begin + tiles_per_group * (MULTI ? groups_per_wg : 1));
    typedef typename Act<T>::raw4 raw4;
    // MULTI: fixed-point sums of the pixel groups finished so far, element threadIdx.x + i * WGRAD_THREADS of the block
    constexpr int FX = (BLOCK_FLOATS + WGRAD_THREADS - 1) / WGRAD_THREADS;
    long long fx_sum[MULTI ? FX : 1];
    bool fx_poisoned = false;
#pragma unroll
    for (int i = 0; i < (MULTI ? FX : 1); ++i) fx_sum[i] = 0;
    // Fold the waves in wave order.  LDS and the partial are lane-major, element (t*4 + j)*64 + lane
    // holds dW[o = 4*(lane/16) + j][t][i = lane%16] of the block: conflict-free writes, coalesced stores.
    auto fold_group = [&]() {
        __syncthreads();   // the tile in LDS is consumed
#pragma unroll
        for (int t = 0; t < TAPS; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                lds[wave * BLOCK_FLOATS + (t * 4 + j) * 64 + lane] = acc[t][j];
                acc[t][j] = 0.f;
            }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < FX; ++i) {
            const int e = threadIdx.x + i * WGRAD_THREADS;
            if (e < BLOCK_FLOATS) {
                float v = lds[e];
#pragma unroll
                for (int wv = 1; wv < WG_WAVES; ++wv) v += lds[wv * BLOCK_FLOATS + e];
                fixsum_collect(fx_sum[MULTI ? i : 0], fx_poisoned, (double)v * FIX_WGRAD_SCALE, FIX_PARTIAL_LIMIT);
            }
        }
    };
    // slot k of this thread: element threadIdx.x + k * WGRAD_THREADS of the tile (rows x columns x 4 channel quads)
    int x_dst[XK], x_part[XK], x_li[XK], x_off[XK];
    raw4 xv[XK], dv[WG_DK];
    if constexpr (PIPE) {
        const int n_cols = g.lw * 4, slots = g.imgs * g.in_rows * n_cols;
#pragma unroll
        for (int k = 0; k < XK; ++k) {
            const int e = threadIdx.x + k * WGRAD_THREADS;
            const int lr = e / n_cols, col = e - lr * n_cols;
            const int lc = col >> 2, cq = col & 3, wi = lc - g.pad;
            x_dst[k] = e < slots ? (lr * g.lw + lc) * (CP / 4) + cq : -1;
            x_part[k] = lr / g.in_rows;
            x_li[k] = lr - x_part[k] * g.in_rows;
            x_off[k] = (e < slots && (unsigned)wi < (unsigned)g.h_in) ? wi * NI + ib * 16 + cq * 4 : -1;
        }
    }
    auto load_tile = [&](int tile) {
        const int rpi = 1 << g.rpi_log2;
        const int row0 = tile * g.rows_tile;
#pragma unroll
        for (int k = 0; k < XK; ++k) {
            xv[k] = Act<T>::zero();
            if (x_off[k] >= 0) {
                const int grow = row0 + x_part[k] * rpi;
                const int n = grow >> g.wout_log2;
                const int hi = (grow & (g.h_out - 1)) * g.stride - g.pad + x_li[k];
                if (n < g.B && (unsigned)hi < (unsigned)g.h_in) xv[k] = Act<T>::load_raw(x + ((int64_t)n * g.h_in + hi) * g.h_in * NI + x_off[k]);
            }
        }
        const int64_t pix0 = (int64_t)tile * tile_pixels;
#pragma unroll
        for (int k = 0; k < WG_DK; ++k) {
            const int i = threadIdx.x + k * WGRAD_THREADS;
            const int q = i >> 2, c4 = i & 3;
            dv[k] = Act<T>::zero();
            if (i < tile_pixels * 4 && pix0 + q < total_pixels) dv[k] = Act<T>::load_raw(dy + (pix0 + q) * NO + ob * 16 + c4 * 4);
        }
    };
    if constexpr (PIPE) {
        if (tile_begin < tile_end) load_tile(tile_begin);
    }
    for (int tile = tile_begin; tile < tile_end; ++tile) {
        __syncthreads();  // previous tile fully consumed
        if constexpr (PIPE) {
#pragma unroll
            for (int k = 0; k < XK; ++k)
                if (x_dst[k] >= 0) lds4[x_dst[k]] = Act<T>::widen(xv[k]);
#pragma unroll
            for (int k = 0; k < WG_DK; ++k) {
                const int i = threadIdx.x + k * WGRAD_THREADS;
                if (i < tile_pixels * 4) reinterpret_cast<f32x4*>(lds_dy)[i] = Act<T>::widen(dv[k]);
            }
            __syncthreads();
            if (tile + 1 < tile_end) load_tile(tile + 1);
        } else {
            stage_input<T, f32x4, 16, WGRAD_THREADS, 0>(lds4, x, g, tile, NI, ib * 16);
            const int64_t pix0 = (int64_t)tile * tile_pixels;
            for (int i = threadIdx.x; i < tile_pixels * 4; i += WGRAD_THREADS) {
                int q = i >> 2, c4 = i & 3;
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (pix0 + q < total_pixels) v = Act<T>::load4(dy + (pix0 + q) * NO + ob * 16 + c4 * 4);
                reinterpret_cast<f32x4*>(lds_dy)[q * (DP / 4) + c4] = v;
            }
            __syncthreads();
        }
        // One MFMA consumes 4 pixels (one per lane group).
        if (w_out >= 4) {
            // a quad lies inside one output row: the waves take rows in turn and the row base is wave-uniform
            const int lane_x = grp * g.stride * CP + r16, lane_dy = grp * DP + r16;
            for (int row = wave; row < g.rows_tile; row += WG_WAVES) {
                const int part = row >> g.rpi_log2, r = row & ((1 << g.rpi_log2) - 1);
                const float* xr = lds_x + (part * g.in_rows + r * g.stride) * g.lw * CP + lane_x;
                const float* dr = lds_dy + (row << g.wout_log2) * DP + lane_dy;
#pragma unroll 2
                for (int qc = 0; qc < (w_out >> 2); ++qc) {
                    const float a = dr[qc * 4 * DP];
                    const float* xq = xr + qc * 4 * g.stride * CP;
#pragma unroll
                    for (int t = 0; t < TAPS; ++t) {
                        const float b = xq[TAPS == 9 ? ((t / 3) * g.lw + (t % 3)) * CP : 0];
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[t], 0, 0, 0);
                    }
                }
            }
        } else {
            for (int qd = wave; qd < tile_pixels / 4; qd += WG_WAVES) {
                const int q = 4 * qd + grp;
                const float a = lds_dy[q * DP + r16];
                const int xb = pixel_lds_base<16, 0>(g, q) + r16;
#pragma unroll
                for (int t = 0; t < TAPS; ++t) {
                    const float b = lds_x[xb + (TAPS == 9 ? ((t / 3) * g.lw + (t % 3)) * CP : 0)];
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[t], 0, 0, 0);
                }
            }
        }
        if (MULTI && ((tile + 1 - tile_begin) % tiles_per_group == 0 || tile + 1 == tile_end)) fold_group();   // a pixel group ends here
    }
    // order-independent accumulation across pixel groups: replicated 64-bit fixed point, integer atomic add
    fixsum_t* out = gacc + ((int64_t)(blockIdx.x % replicas) * gridDim.y + blockIdx.y) * BLOCK_FLOATS;
    if (MULTI) {
#pragma unroll
        for (int i = 0; i < FX; ++i) {
            const int e = threadIdx.x + i * WGRAD_THREADS;
            if (e < BLOCK_FLOATS) fixsum_flush(out + e, fx_sum[i], fx_poisoned);
        }
        return;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) lds[wave * BLOCK_FLOATS + (t * 4 + j) * 64 + lane] = acc[t][j];
    __syncthreads();
    for (int e = threadIdx.x; e < BLOCK_FLOATS; e += WGRAD_THREADS) {
        float v = lds[e];
#pragma unroll
        for (int wv = 1; wv < WG_WAVES; ++wv) v += lds[wv * BLOCK_FLOATS + e];
        fixsum_add(out + e, (double)v * FIX_WGRAD_SCALE);
    }
}
#pragma clang diagnostic pop

// End of a local step, one launch: for every parameter take the gradient, apply the SGD update
// (g += wd*x; buf = mu*buf + g; x -= lr*buf), and for convolution weights also write the new value into the
// packed copies that the next forward and input-gradient kernels read.  The gradient of a convolution weight
// dw[16*ob + o][t][16*ib + i] is the sum over the replicas of accumulator (ob, ib)[(t*4 + o%4)*64 + 16*(o/4) + i]
// (blocks of 16 * taps * 16 values),
// converted back to float; the accumulators are cleared for the next step.  All other gradients, and those of layers
// with replicas == 0, come from grad[].
// The kernel also clears the batch-norm accumulators of the next step.
template <typename T>
__global__ __launch_bounds__(256) void update_kernel(float* __restrict__ params, float* __restrict__ momentum,
                                                     const float* __restrict__ grad, int64_t d, float lr, float mu, float wd,
                                                     fixsum_t* __restrict__ gacc, T* __restrict__ packed, UpdateTable tab,
                                                     fixsum_t* __restrict__ sums, int64_t n_sums, int64_t rstride, int64_t begin) {
    if (rstride) {   // one replica of several: every buffer sits blockIdx.z slots further
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        params = rep_at(params, ro); momentum = rep_at(momentum, ro); grad = rep_at(grad, ro); gacc = rep_at(gacc, ro); packed = rep_at(packed, ro);
        sums = rep_at(sums, ro);
    }
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = first; i < n_sums; i += stride) sums[i] = 0ull;
    for (int64_t i = begin + first; i < d; i += stride) {   // parameters begin .. d - 1
        int l = -1;
        for (int q = 0; q < tab.n; ++q)
            if (i >= tab.e[q].w_off && i < tab.e[q].w_off + tab.e[q].n) l = q;
        float g;
        int co = 0, t = 0, ci = 0;
        if (l >= 0) {
            const UpdateEntry& e = tab.e[l];
            const int r = (int)(i - e.w_off);
            const int ot = r / e.c_in_real;
            ci = r - ot * e.c_in_real;
            co = ot / e.taps;
            t = ot - co * e.taps;
            const int NI = e.c_in, o = co & 15;
            const int blocks = (e.c_out >> 4) * (NI >> 4);
            const int block_floats = 16 * e.taps * 16;
            const int64_t src = (int64_t)((co >> 4) * (NI >> 4) + (ci >> 4)) * block_floats + (t * 4 + (o & 3)) * 64 + 16 * (o >> 2) + (ci & 15);
            const int64_t pitch = (int64_t)blocks * block_floats;
            if (e.replicas > 0) {
                fixsum_t* acc_l = gacc + e.acc_off;
                long long acc = 0, w[WGRAD_REPLICAS];
                bool poisoned = false;
                // all replicas requested at once (a loop over e.replicas waits for one load after the other)
#pragma unroll
                for (int rep = 0; rep < WGRAD_REPLICAS; ++rep) w[rep] = rep < e.replicas ? (long long)acc_l[rep * pitch + src] : 0ll;
#pragma unroll
                for (int rep = 0; rep < WGRAD_REPLICAS; ++rep) {
                    poisoned |= w[rep] >= FIX_POISON_MIN;
                    acc += w[rep];
                    if (rep < e.replicas) acc_l[rep * pitch + src] = 0ull;
                }
                g = poisoned ? FIX_NAN : (float)((double)acc * (1.0 / FIX_WGRAD_SCALE));   // out of range: NaN, as a float sum would end
            } else {
                g = grad[i];   // this layer's weight gradient was written as floats (replicas == 0)
            }
        } else {
            g = grad[i];
        }
        const float x = params[i];
        g = __fmaf_rn(wd, x, g);
        const float buf = __fmaf_rn(mu, momentum[i], g);
        momentum[i] = buf;
        const float xn = __fmaf_rn(-lr, buf, x);
        params[i] = xn;
        if (l >= 0) {
            const UpdateEntry& e = tab.e[l];
            T xs;
            if constexpr (sizeof(T) == 4) xs = xn;
            else xs = f32_to_bf16(xn);
            {   // forward form: quad ((ob*9 + t)*S + s)*64 + lane holds w[16*ob + lane%16][t][16*s + 4*(lane/16) + 0..3]
                const int S = e.c_in >> 4;
                const int64_t quad = e.fwd_quad + ((int64_t)((co >> 4) * e.taps + t) * S + (ci >> 4)) * 64 + (co & 15) + 16 * ((ci & 15) >> 2);
                packed[quad * 4 + (ci & 3)] = xs;
            }
            if (e.dgrad_quad >= 0) {
                // transposed, flipped form: roles of input and output channels swap
                const int S = e.c_out >> 4;
                const int64_t quad = e.dgrad_quad + ((int64_t)((ci >> 4) * e.taps + (e.taps - 1 - t)) * S + (co >> 4)) * 64 + (ci & 15) + 16 * ((co & 15) >> 2);
                packed[quad * 4 + (co & 3)] = xs;
            }
        }
    }
}

void launch_update(hipStream_t s, int act, float* params, float* momentum, const float* grad, int64_t d, float lr, float mu,
                   float wd, fixsum_t* gacc, void* packed, const UpdateTable& tab, fixsum_t* sums, int64_t n_sums, Reps reps, int64_t begin,
                   int64_t end) {
    if (end < 0) end = d;
    int64_t blocks = (end - begin + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    ACT_DISPATCH(act, hipLaunchKernelGGL(update_kernel<T>, dim3((unsigned)blocks, 1, reps.n), dim3(256), 0, s, params, momentum, grad, end, lr, mu,
                                         wd, gacc, (T*)packed, tab, sums, n_sums, reps.stride, begin));
}

// Tiles of the weight-gradient kernel: up to 256 pixels (a power-of-two number of output rows), smaller
// when the staged 16-channel input slice would exceed 40 KB of LDS.
static int wgrad_slots(const ConvShape& cs) { return cs.stride == 2 ? WG_XK_STRIDE2 : WG_XK; }
static bool wgrad_fits_pipe(const ConvGeom& g, int xk) {
    return g.imgs * g.in_rows * g.lw * 4 <= xk * WGRAD_THREADS && (g.rows_tile << g.wout_log2) * 4 <= WG_DK * WGRAD_THREADS;
}

static ConvGeom wgrad_geom(const ConvShape& cs) {
    int h_out = (cs.h_in - 1) / cs.stride + 1;
    {
        // preferred: tiles of WG_PIPE_PIXELS pixels whose slots fit the prefetch registers, two or more per workgroup
        int rows = WG_PIPE_PIXELS / h_out;
        if (rows >= 1 && h_out >= 4) {
            ConvGeom g = make_geom(cs.B, cs.h_in, h_out, cs.c_out, cs.stride, 0, cs.c_in_real, rows, cs.taps == 9 ? 1 : 0);
            if (wgrad_fits_pipe(g, wgrad_slots(cs))) return g;
        }
    }
    int rows = 256 / h_out;
    if (rows < 4) rows = 4;
    for (;;) {
        ConvGeom g = make_geom(cs.B, cs.h_in, h_out, cs.c_out, cs.stride, 0, cs.c_in_real, rows, cs.taps == 9 ? 1 : 0);
        if ((size_t)g.imgs * g.in_rows * g.lw * 16 * sizeof(float) <= 40960 || rows * h_out <= 32) return g;
        rows >>= 1;
    }
}

static int wgrad_groups(const ConvShape& cs, int n_tiles) {
    int blocks = (cs.c_in / 16) * (cs.c_out / 16);
    int cap = WGRAD_GROUP_CAP / blocks / (WG_WAVES / 4);
    if (cap < 1) cap = 1;
    return n_tiles < cap ? n_tiles : cap;
}

// wgrad16.hip: the bf16 matrix-instruction kernel for wide stride-1 layers
bool wgrad16_covers(int act, const ConvShape& cs);
int wgrad16_groups(const ConvShape& cs);
void launch_wgrad16(hipStream_t s, const ConvShape& cs, const void* x, const void* dy, fixsum_t* gacc, int replicas, const KernelTiming* kt,
                    Reps reps);
int64_t wgrad16_partial_words(const ConvShape& cs);

// Accumulator replicas of a layer: as many as there are pixel groups, at most WGRAD_REPLICAS; one where the pixel groups
// leave partial sums that a second launch adds.
int conv_wgrad_replicas(int act, const ConvShape& cs) {
    if (wgrad16_covers(act, cs) && wgrad16_partial_words(cs) > 0) return 1;
    int groups = wgrad16_covers(act, cs) ? wgrad16_groups(cs) : wgrad_groups(cs, wgrad_geom(cs).n_tiles);
    return groups < WGRAD_REPLICAS ? groups : WGRAD_REPLICAS;
}

int64_t conv_wgrad_accumulators(int act, const ConvShape& cs) {
    const int64_t words = (int64_t)conv_wgrad_replicas(act, cs) * cs.c_out * cs.taps * cs.c_in;
    return words + (wgrad16_covers(act, cs) ? wgrad16_partial_words(cs) : 0);
}

template <typename T, int TAPS>
static void launch_conv_wgrad_t(hipStream_t s, const ConvShape& cs, const T* x, const T* dy, fixsum_t* gacc, const KernelTiming* kt, Reps reps) {
    ConvGeom g = wgrad_geom(cs);
    int groups = wgrad_groups(cs, g.n_tiles);
    int tiles_per_group = (g.n_tiles + groups - 1) / groups;  // trailing groups may be empty and then write zeros
    size_t lds = ((size_t)g.imgs * g.in_rows * g.lw * 16 + (size_t)(g.rows_tile << g.wout_log2) * 16) * sizeof(float);
    // several replicas in one launch: a workgroup takes as many consecutive pixel groups as there are replicas
    int groups_per_wg = reps.n > 1 ? (reps.n < groups ? reps.n : groups) : 1;
    const bool multi = groups_per_wg > 1;
    // stride-2 layers take the slot-based staging for a single tile as well: the row-wise one would leave three quarters
    // of the threads without a column
    const bool wide = cs.stride == 2 && wgrad_fits_pipe(g, WG_XK_STRIDE2);
    const bool pipe = wide || (wgrad_fits_pipe(g, WG_XK) && tiles_per_group * groups_per_wg > 1);
    auto kern = multi ? (pipe ? wgrad_kernel<T, TAPS, true, true> : wgrad_kernel<T, TAPS, false, true>)
                      : (pipe ? wgrad_kernel<T, TAPS, true, false> : wgrad_kernel<T, TAPS, false, false>);
    if (wide) kern = multi ? wgrad_kernel<T, TAPS, true, true, WG_XK_STRIDE2> : wgrad_kernel<T, TAPS, true, false, WG_XK_STRIDE2>;
    if (lds < WG_WAVES * 16 * TAPS * 16 * sizeof(float)) lds = WG_WAVES * 16 * TAPS * 16 * sizeof(float);
    if (lds > 65536) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    int blocks = (cs.c_in / 16) * (cs.c_out / 16);
    hipExtLaunchKernelGGL(kern, dim3((groups + groups_per_wg - 1) / groups_per_wg, blocks, reps.n), dim3(WGRAD_THREADS), lds, s,
                          kt ? kt->start : nullptr, kt ? kt->stop : nullptr, 0, x, dy, gacc, g, tiles_per_group, cs.c_in, cs.c_out,
                          groups < WGRAD_REPLICAS ? groups : WGRAD_REPLICAS, reps.stride, groups_per_wg);
}

void launch_conv_wgrad(hipStream_t s, int act, const ConvShape& cs, const void* x, const void* dy, fixsum_t* gacc,
                       const KernelTiming* kt, Reps reps) {
    if (wgrad16_covers(act, cs)) {
        launch_wgrad16(s, cs, x, dy, gacc, conv_wgrad_replicas(act, cs), kt, reps);
        return;
    }
    ACT_DISPATCH(act, {
        if (cs.taps == 9) launch_conv_wgrad_t<T, 9>(s, cs, (const T*)x, (const T*)dy, gacc, kt, reps);
        else launch_conv_wgrad_t<T, 1>(s, cs, (const T*)x, (const T*)dy, gacc, kt, reps);
    });
}

