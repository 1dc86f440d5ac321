// Pieces shared by the convolution kernels: the storage-type traits of a tile, the tile geometry, and the
// staging of an input tile (with its zero halo) into LDS.
#pragma once
#include "act.h"

// A "quad" is 4 consecutive channels as they sit in LDS and in the packed weights; vec16 is one 16-byte
// global load (VQ quads).
template <typename T>
struct Tile;
template <>
struct Tile<float> {
    typedef f32x4 quad;
    typedef f32x4 vec16;
    static constexpr int VQ = 1;
    static __device__ __forceinline__ vec16 zero16() { return f32x4{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ void store16(quad* dst, const vec16& v) { dst[0] = v; }
};
template <>
struct Tile<bf16_t> {
    typedef uint2 quad;
    typedef uint4 vec16;
    static constexpr int VQ = 2;
    static __device__ __forceinline__ vec16 zero16() { return make_uint4(0u, 0u, 0u, 0u); }
    static __device__ __forceinline__ void store16(quad* dst, const vec16& v) {
        dst[0] = make_uint2(v.x, v.y);
        dst[1] = make_uint2(v.z, v.w);
    }
};

constexpr int clog2(int v) { return v <= 1 ? 0 : 1 + clog2(v >> 1); }

#define CONV_THREADS 256
#define CONV_MT 2   // 16-pixel tiles a wave accumulates at once
#define CONV_NW 4   // waves per workgroup of the forward / input-gradient kernel

struct ConvGeom {
    int B, h_in, h_out, c_out, stride, ups;  // ups: input is read with zeros inserted (h_in is the virtual size)
    int rpi_log2, imgs, in_rows, lw;          // rows per image part (log2), image parts per tile, LDS rows per part, LDS row width
    int wout_log2;
    int total_rows;                           // B * h_out
    int w_ci;                                 // input channels actually present in the weight tensor
    int n_tiles;
    int rows_tile;                            // output rows per tile: 4, or more so that a tile has >= 32 pixels
    int pad;                                  // zero border of the filter: 1 for 3x3, 0 for 1x1
};

static inline int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

static ConvGeom make_geom(int B, int h_in, int h_out, int c_out, int stride, int ups, int w_ci, int rows_tile = 0, int pad = 1) {
    ConvGeom g;
    g.B = B; g.h_in = h_in; g.h_out = h_out; g.c_out = c_out; g.stride = stride; g.ups = ups;
    g.rows_tile = rows_tile ? rows_tile : (h_out >= 8 ? 4 : 32 / h_out);
    int rpi = h_out < g.rows_tile ? h_out : g.rows_tile;
    g.rpi_log2 = ilog2(rpi);
    g.imgs = g.rows_tile / rpi;
    g.pad = pad;
    g.in_rows = (rpi - 1) * stride + 1 + 2 * pad;
    g.lw = h_in + 2 * pad;
    g.wout_log2 = ilog2(h_out);
    g.total_rows = B * h_out;
    g.w_ci = w_ci;
    g.n_tiles = (g.total_rows + g.rows_tile - 1) / g.rows_tile;
    return g;
}

// LDS bytes of one staged tile: pixel pitch CIN/4 + 1 quads
template <typename T, int CIN>
static size_t input_lds_bytes(const ConvGeom& g) {
    return (size_t)g.imgs * g.in_rows * g.lw * (CIN / 4 + 1) * sizeof(typename Tile<T>::quad);
}

// Stages the input rows of tile `tile` into lds[(part*in_rows + li)*lw + lc][CIN + PAD], zero outside the image.
// `pitch` is the channel count of the tensor in memory and `c_off` the first channel of the CIN-wide slice.
// A thread owns one quad column (lc, 4 channels) and walks the rows, so the row arithmetic is
// wave-uniform (scalar unit) and no per-element division is needed; loads are issued six rows at a time.
// D is the LDS element: the quad as stored, or f32x4 to widen bf16 to fp32 on the way in.
template <typename T, typename D, int CIN, int THREADS = CONV_THREADS, int PAD = 4>
__device__ __forceinline__ void stage_input(D* __restrict__ lds4, const T* __restrict__ x, const ConvGeom& g,
                                            int tile, int pitch = CIN, int c_off = 0) {
    typedef typename Act<T>::raw4 raw4;
    constexpr int CP4 = (CIN + PAD) / 4, CQ = CIN / 4;
    constexpr int CQ_LOG2 = CQ == 4 ? 2 : (CQ == 8 ? 3 : 4);
    constexpr int R = 6;
    const int rpi = 1 << g.rpi_log2;
    const int row0 = tile * g.rows_tile;
    const int n_cols = g.lw * CQ;
    const int rows_total = g.imgs * g.in_rows;
    const int src_h = g.ups ? (g.h_in >> 1) : g.h_in;
    for (int col = threadIdx.x; col < n_cols; col += THREADS) {
        const int cq = col & (CQ - 1), lc = col >> CQ_LOG2;
        const int wi = lc - g.pad;
        bool wok = (unsigned)wi < (unsigned)g.h_in;
        int wsrc = wi;
        if (g.ups) {
            wok = wok && ((wi & 1) == 0);
            wsrc = wi >> 1;
        }
        const T* colp = x + (int64_t)(wok ? wsrc : 0) * pitch + c_off + cq * 4;
        D* dst = lds4 + lc * CP4 + cq;
        for (int r0 = 0; r0 < rows_total; r0 += R) {
            raw4 v[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int lr = r0 + r;                               // wave-uniform
                const int part = lr / g.in_rows, li = lr - part * g.in_rows;
                const int grow = row0 + part * rpi;
                const int n = grow >> g.wout_log2;                   // h_out == w_out
                const int hi = (grow & (g.h_out - 1)) * g.stride - g.pad + li;
                bool ok = lr < rows_total && n < g.B && (unsigned)hi < (unsigned)g.h_in && wok;
                int hsrc = hi;
                if (g.ups) {
                    ok = ok && ((hi & 1) == 0);
                    hsrc = hi >> 1;
                }
                v[r] = Act<T>::zero();
                if (ok) v[r] = Act<T>::load_raw(colp + ((int64_t)n * src_h + hsrc) * src_h * pitch);
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (r0 + r < rows_total) {
                    if constexpr (sizeof(D) == sizeof(raw4)) dst[(r0 + r) * g.lw * CP4] = v[r];
                    else dst[(r0 + r) * g.lw * CP4] = Act<T>::widen(v[r]);
                }
        }
    }
}

// LDS float offset of the top-left tap of output pixel q (index inside the tile).
template <int CIN, int PAD = 4>
__device__ __forceinline__ int pixel_lds_base(const ConvGeom& g, int q) {
    int rowq = q >> g.wout_log2, col = q & (g.h_out - 1);
    int part = rowq >> g.rpi_log2, r = rowq & ((1 << g.rpi_log2) - 1);
    return ((part * g.in_rows + r * g.stride) * g.lw + col * g.stride) * (CIN + PAD);
}

