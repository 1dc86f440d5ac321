// Convolutions of wide layers (up to 512 channels): 3x3 (padding 1) and 1x1, stride 1 or 2, forward and input
// gradient, as implicit GEMMs on the matrix cores.
//
// A workgroup owns a tile of 128 or 256 output pixels (whole rows, several images when maps are small) and a
// group of 64 output channels, one block of 16 per wavefront.  The input channels are consumed in chunks of
// CK = 16 or 32: the chunk of the input tile is staged with its zero halo into LDS as [row][col][CK + 4], the
// wave loads the weights of its 16 output channels for this chunk and all taps into registers from the
// lane-major packed copy, and the accumulators of all 8 or 16 pixel blocks of the tile stay in registers across
// the chunks (A = weights, B = pixels, as in the narrow kernel: lane group g supplies channels 16s + 4g .. +3).
// So a weight register feeds 8-16 MFMAs and a staged pixel is reused by 4 waves and all taps.  The epilogue
// optionally adds a tensor of the output's shape (residual branch / second gradient branch) and reduces the
// batch-norm sums of what it stores.
#include "conv_tile.h"

#include <type_traits>

struct WEpi {
    const void* add;   // tensor of the output's shape added before the store, or nullptr
    fixsum_t* sums;    // [replica][2][c_out] accumulators for (sum, sum of squares) of the stored values, or nullptr
    double scale;
    double limit;      // bound of one workgroup's partial in scaled units (the grid is not capped here: 2^61 / contributions per word)
};

// bf16 chunks of 32 channels run on v_mfma_f32_16x16x32_bf16: lane group g supplies channels 8g .. 8g+7 of both
// operands, the pixel pitch in LDS is 96 bytes (16-byte reads of 16 pixels x 4 channel groups run at the full LDS rate
// when the pitch is 32 bytes more than a multiple of 64; measured at half of it with 80 bytes), and
// the weights of a lane are two neighbouring quads of the packed copy.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
#define WC_NV 7   // 16-byte vectors of a chunk tile per thread in the prefetching path

template <typename T, int TAPS, int CK>
struct WcTraits {
    static constexpr bool K32 = sizeof(T) == 2 && CK == 32;
    static constexpr int PADE = K32 ? 16 : sizeof(T) == 4 ? 8 : 4;   // padding elements per pixel
    static constexpr int CPQ = (CK + PADE) / 4;       // pixel pitch in quads
    static constexpr int S = CK / 16;
    static constexpr int CV = CK / 4 / Tile<T>::VQ;   // 16-byte vectors per pixel and chunk
    static constexpr int WREGS = K32 ? TAPS : TAPS * S;
};

template <typename T, int TAPS, int CK>
static size_t wconv_lds_bytes(const ConvGeom& g) {
    return (size_t)g.imgs * g.in_rows * g.lw * WcTraits<T, TAPS, CK>::CPQ * sizeof(typename Tile<T>::quad);
}

template <typename T, int TAPS, int CK, int NPT>
__global__ __launch_bounds__(256) void wconv_kernel(const T* __restrict__ x, const void* __restrict__ wpk, T* __restrict__ y, WEpi e,
                                                    ConvGeom g, int c_in, int pipelined) {
    __builtin_amdgcn_s_setprio(2);   // ahead of the weight-gradient kernels of the side stream, which only the update waits for
    typedef typename Tile<T>::quad quad;
    typedef typename Tile<T>::vec16 vec16;
    typedef WcTraits<T, TAPS, CK> TR;
    // one weight register set: K32: per tap the 8 channels of this lane group; otherwise per tap and 16-channel block a quad
    typedef typename std::conditional<TR::K32, uint4, quad>::type wreg;
    extern __shared__ f32x4 lds_raw[];
    quad* lds4 = reinterpret_cast<quad*>(lds_raw);
    float* lds = reinterpret_cast<float*>(lds_raw);
    constexpr int S = TR::S, CPQ = TR::CPQ;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, grp = lane >> 4;
    const int NO = g.c_out, NOB = NO >> 4;
    const int ob = blockIdx.y * 4 + wave;
    const bool active = ob < NOB;  // the last channel group may be partly empty; idle waves still stage and synchronise
    const int tile = blockIdx.x;
    const int s_total = c_in >> 4;
    const int n_chunks = c_in / CK;

    int base[NPT];
    f32x4 acc[NPT];
#pragma unroll
    for (int pt = 0; pt < NPT; ++pt) {
        base[pt] = pixel_lds_base<CK, TR::PADE>(g, pt * 16 + r16) / 4 + (TR::K32 ? 2 * grp : grp);  // quad units
        acc[pt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const quad* wp = reinterpret_cast<const quad*>(wpk) + (int64_t)(active ? ob : 0) * TAPS * s_total * 64;

    auto load_weights = [&](wreg (&w)[TR::WREGS], int ch) {
        if constexpr (TR::K32) {
            // channels 32*ch + 8*grp .. +7: 16-channel block 2*ch + grp/2, lane groups 2*(grp%2) and 2*(grp%2) + 1
            const quad* p0 = wp + (int64_t)(2 * ch + (grp >> 1)) * 64 + r16 + 32 * (grp & 1);
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                const quad lo = p0[(int64_t)t * s_total * 64], hi = p0[(int64_t)t * s_total * 64 + 16];
                w[t] = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
        } else {
#pragma unroll
            for (int t = 0; t < TAPS; ++t)
#pragma unroll
                for (int s = 0; s < S; ++s) w[t * S + s] = wp[(int64_t)(t * s_total + ch * S + s) * 64 + lane];
        }
    };
    auto mfma_chunk = [&](const quad* tilep, const wreg (&w)[TR::WREGS]) {
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            const int tap_off = TAPS == 9 ? ((t / 3) * g.lw + (t % 3)) * CPQ : 0;
            if constexpr (TR::K32) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, w[t]);
#pragma unroll
                for (int pt = 0; pt < NPT; ++pt) {
                    const uint4 b = *reinterpret_cast<const uint4*>(tilep + base[pt] + tap_off);
                    acc[pt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b), acc[pt], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int s = 0; s < S; ++s) {
#pragma unroll
                    for (int pt = 0; pt < NPT; ++pt) {
                        const quad b = tilep[base[pt] + tap_off + 4 * s];
                        if constexpr (sizeof(T) == 4) {
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                acc[pt] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[t * S + s][j], b[j], acc[pt], 0, 0, 0);
                        } else {
                            acc[pt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, w[t * S + s]),
                                                                                __builtin_bit_cast(s16x4, b), acc[pt], 0, 0, 0);
                        }
                    }
                }
            }
        }
    };

    wreg wr[TR::WREGS];
    if (pipelined) {
        // Every thread owns up to WC_NV 16-byte vectors of the chunk tile; their global and LDS positions do not depend on
        // the chunk and are worked out once.  While the MFMAs of a chunk run from one LDS buffer, the next chunk's tile
        // and weights are in flight into registers and are then written to the other buffer (one barrier per chunk).
        const int nvec = g.imgs * g.in_rows * g.lw * TR::CV;
        const int buf_quads = g.imgs * g.in_rows * g.lw * CPQ;
        const int rpi = 1 << g.rpi_log2;
        const int row0 = tile * g.rows_tile;
        const int src_h = g.ups ? (g.h_in >> 1) : g.h_in;
        int goff[WC_NV], loff[WC_NV];
#pragma unroll
        for (int i = 0; i < WC_NV; ++i) {
            const int v = threadIdx.x + 256 * i;
            const int cv = v % TR::CV, px = v / TR::CV;
            const int lc = px % g.lw, lr = px / g.lw;
            const int part = lr / g.in_rows, li = lr - part * g.in_rows;
            const int grow = row0 + part * rpi;
            const int n = grow >> g.wout_log2;
            const int hi = (grow & (g.h_out - 1)) * g.stride - g.pad + li;
            const int wi = lc - g.pad;
            bool ok = v < nvec && n < g.B && (unsigned)hi < (unsigned)g.h_in && (unsigned)wi < (unsigned)g.h_in;
            int hs = hi, ws = wi;
            if (g.ups) {
                ok = ok && ((hi | wi) & 1) == 0;
                hs = hi >> 1;
                ws = wi >> 1;
            }
            goff[i] = ok ? ((n * src_h + hs) * src_h + ws) * c_in + cv * (4 * Tile<T>::VQ) : -1;
            loff[i] = v < nvec ? px * CPQ + cv * Tile<T>::VQ : -1;
        }
        vec16 pre[WC_NV];
        auto tile_fetch = [&](int ch) {
#pragma unroll
            for (int i = 0; i < WC_NV; ++i) {
                pre[i] = Tile<T>::zero16();
                if (goff[i] >= 0) pre[i] = *reinterpret_cast<const vec16*>(x + goff[i] + ch * CK);
            }
        };
        auto tile_put = [&](quad* buf) {
#pragma unroll
            for (int i = 0; i < WC_NV; ++i)
                if (loff[i] >= 0) {
                    if constexpr (TR::K32) *reinterpret_cast<vec16*>(buf + loff[i]) = pre[i];
                    else Tile<T>::store16(buf + loff[i], pre[i]);
                }
        };
        tile_fetch(0);
        load_weights(wr, 0);
        tile_put(lds4);
        __syncthreads();
        for (int ch = 0; ch < n_chunks; ++ch) {
            wreg wn[TR::WREGS];
            const bool more = ch + 1 < n_chunks;
            if (more) {
                tile_fetch(ch + 1);
                load_weights(wn, ch + 1);
            }
            if (active) mfma_chunk(lds4 + (ch & 1) * buf_quads, wr);
            if (more) {
                tile_put(lds4 + ((ch + 1) & 1) * buf_quads);
#pragma unroll
                for (int i = 0; i < TR::WREGS; ++i) wr[i] = wn[i];
            }
            __syncthreads();
        }
    } else {
        for (int ch = 0; ch < n_chunks; ++ch) {
            __syncthreads();  // the previous chunk has been consumed
            stage_input<T, quad, CK, 256, TR::PADE>(lds4, x, g, tile, c_in, ch * CK);
            load_weights(wr, ch);
            __syncthreads();
            if (active) mfma_chunk(lds4, wr);
        }
        __syncthreads();
    }

    // epilogue: lane holds channels c0 .. c0+3 of pixel (pt*16 + r16)
    const int64_t pix0 = (int64_t)tile * (NPT * 16);
    const int64_t total_pixels = (int64_t)g.total_rows << g.wout_log2;
    const int c0 = ob * 16 + 4 * grp;
    const T* add = static_cast<const T*>(e.add);
    f32x4 ssum = {0.f, 0.f, 0.f, 0.f}, ssq = {0.f, 0.f, 0.f, 0.f};
    if (active) {
#pragma unroll
        for (int pt = 0; pt < NPT; ++pt) {
            const int64_t p = pix0 + pt * 16 + r16;
            if (p < total_pixels) {
                f32x4 v = acc[pt];
                if (add) v += Act<T>::load4(add + p * NO + c0);
                v = Act<T>::rounded(v);  // the sums see what later kernels read back
                Act<T>::store4(y + p * NO + c0, v);
                ssum += v;
                ssq += v * v;
            }
        }
    }
    if (e.sums) {
#pragma unroll
        for (int o = 1; o < 16; o <<= 1)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ssum[j] += __shfl_xor(ssum[j], o, 64);
                ssq[j] += __shfl_xor(ssq[j], o, 64);
            }
        float* red = lds;  // every wave is past its last tile read (barrier after the last chunk)  // [wave][2][16]
        if (r16 == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                red[(wave * 2 + 0) * 16 + 4 * grp + j] = ssum[j];
                red[(wave * 2 + 1) * 16 + 4 * grp + j] = ssq[j];
            }
        }
        __syncthreads();
        if (threadIdx.x < 128) {
            const int which = threadIdx.x >> 6, c = threadIdx.x & 63;  // channel c of this group: wave c/16 holds it
            const int ch = blockIdx.y * 64 + c;
            if (ch < NO)
                fixsum_add(e.sums + ((blockIdx.x % FIX_REPLICAS) * 2 + which) * NO + ch, (double)red[((c >> 4) * 2 + which) * 16 + (c & 15)] * e.scale, e.limit);
        }
    }
}

// Tile: 256 pixels when the staged chunk fits 64 KB (two workgroups per compute unit), else 128.  The prefetching
// path needs the chunk tile to fit WC_NV vectors per thread and two buffers to fit 80 KB.
template <typename T, int TAPS, int CK>
static int launch_wconv_t(hipStream_t s, int B, int h_in, int h_out, int c_in, int c_out, int stride, int ups, const T* x, const void* w,
                          T* y, const WEpi& e_in) {
    typedef WcTraits<T, TAPS, CK> TR;
    const int pad = TAPS == 9 ? 1 : 0;
    auto geom = [&](int npt) { return make_geom(B, h_in, h_out, c_out, stride, ups, c_in, (npt * 16) / h_out, pad); };
    if (h_out > 128) return -1;
    ConvGeom g = geom(16);
    int npt = 16;
    size_t lds = wconv_lds_bytes<T, TAPS, CK>(g);
    if (lds > 65536 || 256 / h_out < 1) {
        g = geom(8);
        npt = 8;
        lds = wconv_lds_bytes<T, TAPS, CK>(g);
    }
    if (lds > 160 * 1024 - 2048 || (npt * 16) / h_out < 1) return -1;
    const int nvec = g.imgs * g.in_rows * g.lw * TR::CV;
    const int pipelined = (nvec <= 256 * WC_NV && 2 * lds <= 80 * 1024 && c_in / CK > 1) ? 1 : 0;
    if (pipelined) lds *= 2;
    if (lds < 1024) lds = 1024;
    dim3 grid(g.n_tiles, (c_out / 16 + 3) / 4);
    WEpi e = e_in;
    e.limit = 576460752303423488.0 / (double)((g.n_tiles + FIX_REPLICAS - 1) / FIX_REPLICAS);   // 2^59 over the partials one word takes
    if (npt == 16) {
        auto kern = wconv_kernel<T, TAPS, CK, 16>;
        if (lds > 65536) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, x, w, y, e, g, c_in, pipelined);
    } else {
        auto kern = wconv_kernel<T, TAPS, CK, 8>;
        if (lds > 65536) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, x, w, y, e, g, c_in, pipelined);
    }
    return 0;
}

// c_in is 16 or a multiple of 32, c_out a multiple of 16, maps are squares with power-of-two sides.
// Returns 0, or -1 when the shape is outside what the kernel is built for (nothing is launched then).
int launch_wconv(hipStream_t s, int act, int taps, int B, int h_in, int h_out, int c_in, int c_out, int stride, int ups, const void* x,
                 const void* w, void* y, const void* add, fixsum_t* sums, double scale) {
    if (!(c_in == 16 || c_in % 32 == 0) || c_out % 16 != 0 || (taps != 9 && taps != 1)) return -1;
    WEpi e{add, sums, scale, 0.0};
    int rc = -1;
    ACT_DISPATCH(act, {
        if (taps == 9) rc = c_in == 16 ? launch_wconv_t<T, 9, 16>(s, B, h_in, h_out, c_in, c_out, stride, ups, (const T*)x, w, (T*)y, e)
                                       : launch_wconv_t<T, 9, 32>(s, B, h_in, h_out, c_in, c_out, stride, ups, (const T*)x, w, (T*)y, e);
        else rc = c_in == 16 ? launch_wconv_t<T, 1, 16>(s, B, h_in, h_out, c_in, c_out, stride, ups, (const T*)x, w, (T*)y, e)
                             : launch_wconv_t<T, 1, 32>(s, B, h_in, h_out, c_in, c_out, stride, ups, (const T*)x, w, (T*)y, e);
    });
    return rc;
}
