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
#include <utility>

struct WEpi {
    const void* add;   // tensor of the output's shape added before the store, or nullptr
    fixsum_t* sums;    // [replica][2][c_out] accumulators for (sum, sum of squares) of the stored values, or nullptr
    double scale;
    double limit;      // bound of one workgroup's partial in scaled units (the grid is not capped here: 2^61 / contributions per word)
    WconvBn bn;        // bn.mean != nullptr: batch norm and ReLU of the reading layer before the store (inference)
};

// relu(bn(v)) for the four channels of a lane, exactly as bn_apply_kernel computes it (its residual term is zero here)
__device__ __forceinline__ f32x4 wconv_bn_relu(f32x4 v, const f32x4& mu, const f32x4& is, const f32x4& ga, const f32x4& be) {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = relu_keep_nan(__fmaf_rn((v[j] - mu[j]) * is[j], ga[j], be[j]) + 0.f);
    return v;
}

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

// (two workgroups per compute unit for the 16-channel inputs of bf16 layers: they have a single chunk, so nothing inside a
// workgroup overlaps its loads, its few matrix instructions and its stores)
template <typename T, int TAPS, int CK, int NPT>
__global__ __launch_bounds__(256, (sizeof(T) == 2 && CK == 16) ? 2 : 1) void wconv_kernel(const T* __restrict__ x, const void* __restrict__ wpk, T* __restrict__ y, WEpi e,
                                                    ConvGeom g, int c_in, int pipelined, int sub) {
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
        // sub: the geometry describes a stride-1 layer over every second row and column of a map twice the size (a 1x1
        // stride-2 filter reads nothing else)
        const int src_h = sub ? 2 * g.h_in : g.ups ? (g.h_in >> 1) : g.h_in;
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
            if (sub) {
                hs = 2 * hi;
                ws = 2 * wi;
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
        // the added tensor is requested for the whole tile before the first store: behind a store the compiler would have to
        // keep every later load (the two tensors may be the same memory for all it knows), one memory round trip per pixel block
        typename Act<T>::raw4 addv[NPT];
        if (add) {
#pragma unroll
            for (int pt = 0; pt < NPT; ++pt) {
                const int64_t p = pix0 + pt * 16 + r16;
                addv[pt] = Act<T>::zero();
                if (p < total_pixels) addv[pt] = Act<T>::load_raw(add + p * NO + c0);
            }
        }
        f32x4 bn_mu = {0.f, 0.f, 0.f, 0.f}, bn_is = bn_mu, bn_ga = bn_mu, bn_be = bn_mu;
        T* raw = static_cast<T*>(e.bn.raw);
        if (e.bn.mean) {
            bn_mu = *reinterpret_cast<const f32x4*>(e.bn.mean + c0);
            bn_is = *reinterpret_cast<const f32x4*>(e.bn.invstd + c0);
            bn_ga = *reinterpret_cast<const f32x4*>(e.bn.gamma + c0);
            bn_be = *reinterpret_cast<const f32x4*>(e.bn.beta + c0);
        }
#pragma unroll
        for (int pt = 0; pt < NPT; ++pt) {
            const int64_t p = pix0 + pt * 16 + r16;
            if (p < total_pixels) {
                f32x4 v = acc[pt];
                if (add) v += Act<T>::widen(addv[pt]);
                v = Act<T>::rounded(v);  // the sums see what later kernels read back
                if (e.bn.mean) {
                    if (raw) Act<T>::store4(raw + p * NO + c0, v);
                    v = wconv_bn_relu(v, bn_mu, bn_is, bn_ga, bn_be);
                }
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

// calls f(std::integral_constant<int, 0>) .. f(std::integral_constant<int, N - 1>) in order: a loop whose index is a constant
// expression in the body, unrolled whatever its size
template <class F, int... I>
__device__ __forceinline__ void static_for_seq(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_seq(f, std::make_integer_sequence<int, N>{});
}

// bf16 3x3 stride-1 layers whose output channels come in multiples of 128, in launches large enough to fill the chip
// with workgroups of 256 pixels x 128 output channels.
//
// In wconv_kernel every matrix instruction has an LDS read of its own (a wave holds one block of 16 output channels), and
// four waves reading 1 KB per instruction keep the LDS pipe (128 bytes per clock) busier than the matrix pipe can be.
// Here a wave holds WB_OB x WB_PB accumulator blocks (output channels x pixels): one pixel operand read from LDS feeds
// WB_OB instructions, one weight operand (registers, from the lane-major packed copy) feeds WB_PB.  The waves of a
// workgroup are a 2 x 2 arrangement of (64 output channels, 128 pixels).
//
// The chunk tile goes from global memory straight into LDS (global_load_lds, 16 bytes per lane: the 64 lanes of an
// instruction fill 1 KB of consecutive LDS), so it passes through no registers and a wave stays within 128 vector + 128
// accumulation registers: two workgroups per compute unit, one computing while the other waits for memory, stores its
// tile or sits at a barrier.  Consecutive LDS per instruction means no padding between pixels: a pixel's 32 channels
// are 64 bytes, positions follow each other ([row][column] of the halo'd tile), and the 16-byte reads of the matrix
// operands run at 93 % of the padded layout's rate (measured).  Positions outside the image are never written by a
// load; they are zeroed once, in both buffers, before the first chunk.
//
// Chunks, taps and the K = 32 grouping of the channels are consumed in wconv_kernel's order, and the batch-norm sums of a
// 256-pixel tile are taken in its order too (the waves of the second pixel half continue the lane sums of the first),
// so both kernels give the same bits.
#define WB_OB 4
#define WB_PB 8
#define WB_NV 7            // 16-byte slots of a chunk tile per thread, at most
#define WB_NV_STRIDE2 10   // the same for a stride-2 layer (17 input rows of 34 positions)
#define WB_AHEAD 3     // pixel operands requested from LDS ahead of their matrix instructions
// Weight register sets (one tap each): the tap in use and the ones requested behind it.  Three sets leave a wave within
// 128 + 128 registers: two workgroups per compute unit, which is what large launches want.  A launch with at most one
// workgroup per compute unit has nobody to hide a wave's waits: it takes nine sets (a weight is requested eight taps, ~2 us,
// before its use) and the registers of the absent second workgroup.
#define WB_WSETS_SHARED 3
#define WB_WSETS_ALONE 9
// The matrix instruction as an assembly statement: accumulator in place in the accumulation registers, operands in
// vector registers.  (Written as the builtin, the compiler keeps moving the 128 accumulator registers between the two
// register files: two moves per matrix instruction.)  The compiler does not see the instruction's latency: a wait stands
// between the last matrix instruction and the first other reader of an accumulator.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
#define WB_MFMA(acc, a, b) \
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(__builtin_bit_cast(u32x4, a)), "v"(__builtin_bit_cast(u32x4, b)))
typedef __attribute__((address_space(1))) const void wb_global_ptr;
typedef __attribute__((address_space(3))) void wb_lds_ptr;

template <int LW, int STRIDE, bool BN, int WSETS>
__global__ __launch_bounds__(256, WSETS == WB_WSETS_SHARED ? 2 : 1) void wconv_block_kernel(const bf16_t* __restrict__ x, const void* __restrict__ wpk, bf16_t* __restrict__ y,
                                                             WEpi e, ConvGeom g, int c_in) {
    __builtin_amdgcn_s_setprio(2);
    typedef bf16_t T;
    typedef Tile<T>::quad quad;
    constexpr int TAPS = 9, STEPS = TAPS * WB_PB;
    // Stride 1: 2 x 2 waves of (64 channels, 128 pixels).  Stride 2: the input rows of 256 output pixels do not fit two
    // buffers, so the tile has 128 pixels and the four waves hold 64 channels each (WIDE).
    constexpr bool WIDE = STRIDE == 2;
    constexpr int OCW = WIDE ? 4 : 2;                                     // 64-channel groups of a workgroup
    constexpr int IN_ROWS = WIDE ? 17 : (LW == 18 ? 18 : 10);             // rows of an image part with halo (8 output rows, or a whole 16-row image)
    constexpr int NV = WIDE ? WB_NV_STRIDE2 : WB_NV;
    extern __shared__ f32x4 lds_raw[];
    char* lds_bytes = reinterpret_cast<char*>(lds_raw);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform by construction; says so to the compiler
    const int r16 = lane & 15, grp = lane >> 4;
    const int wo = WIDE ? wave : wave & 1, wpx = WIDE ? 0 : wave >> 1;   // 64-channel group and pixel half of this wave
    const int NO = g.c_out;
    const int ob0 = blockIdx.y * (OCW * WB_OB) + wo * WB_OB;
    const int tile = blockIdx.x;
    const int s_total = c_in >> 4;
    const int n_chunks = c_in >> 5;
    const int n_slots = g.imgs * IN_ROWS * LW * 4;             // 16-byte slots of one buffer: [position][4]
    const int buf_bytes = ((n_slots + 255) & ~255) * 16;       // whole 1 KB blocks of a load instruction

    int base[WB_PB];   // byte offset of the lane's 8 channels of the pixel block's tap (0, 0)
    f32x4 acc[WB_OB][WB_PB];
#pragma unroll
    for (int pt = 0; pt < WB_PB; ++pt) {
        base[pt] = pixel_lds_base<32, 0>(g, (wpx * WB_PB + pt) * 16 + r16) * (int)sizeof(T) + 16 * grp;
#pragma unroll
        for (int o = 0; o < WB_OB; ++o) acc[o][pt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // channels 32*ch + 8*grp .. +7 of a tap: 16-channel block 2*ch + grp/2 of the packed copy, lane groups 2*(grp%2) and
    // 2*(grp%2) + 1, i.e. two 8-byte pieces 16 lanes apart.  Uniform base plus a per-lane byte offset: one address
    // register per lane for all weight loads.
    const char* wbase = static_cast<const char*>(wpk) + (int64_t)ob0 * TAPS * s_total * 512;
    const unsigned lane_off = (unsigned)(((grp >> 1) * 64 + r16 + 32 * (grp & 1)) * 8);
    // the weights of block o, tap t, chunk ch
    auto weights_of = [&](int o, int t, int ch) {
        const char* p = wbase + (int64_t)((o * TAPS + t) * s_total + 2 * ch) * 512;
        const quad lo = *reinterpret_cast<const quad*>(p + lane_off), hi = *reinterpret_cast<const quad*>(p + lane_off + 128);
        return make_uint4(lo.x, lo.y, hi.x, hi.y);
    };

    // staging: slot v = 256*i + thread of a buffer holds channels 8*(v%4) .. +7 of position v/4; its place in the
    // tensor does not depend on the chunk
    const int rpi = 1 << g.rpi_log2;
    const int row0 = tile * g.rows_tile;
    const int src_h = g.ups ? (g.h_in >> 1) : g.h_in;
    int goff[NV];   // element offset of the slot's channels in chunk 0, or -1 for a slot that stays zero
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = threadIdx.x + 256 * i;
        const int cq = v & 3, pos = v >> 2;
        const int lc = pos % LW, lr = pos / LW;
        const int part = lr / IN_ROWS, li = lr - part * IN_ROWS;
        const int grow = row0 + part * rpi;
        const int n = grow >> g.wout_log2;
        const int hi = (grow & (g.h_out - 1)) * STRIDE - g.pad + li;
        const int wi = lc - g.pad;
        bool ok = v < n_slots && n < g.B && (unsigned)hi < (unsigned)g.h_in && (unsigned)wi < (unsigned)g.h_in;
        int hs = hi, ws = wi;
        if (g.ups) {
            ok = ok && ((hi | wi) & 1) == 0;
            hs = hi >> 1;
            ws = wi >> 1;
        }
        goff[i] = ok ? ((n * src_h + hs) * src_h + ws) * c_in + cq * 8 : -1;
        if (!ok && v < n_slots) {
            *reinterpret_cast<uint4*>(lds_bytes + v * 16) = make_uint4(0u, 0u, 0u, 0u);
            *reinterpret_cast<uint4*>(lds_bytes + buf_bytes + v * 16) = make_uint4(0u, 0u, 0u, 0u);
        }
    }
    auto tile_request = [&](int ch, int buf) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
            if (goff[i] >= 0)
                __builtin_amdgcn_global_load_lds((wb_global_ptr*)(x + (unsigned)(goff[i] + ch * 32)),
                                                 (wb_lds_ptr*)(lds_bytes + buf * buf_bytes + (i * 256 + wave * 64) * 16), 16, 0, 0);
    };

    // The chunk loop is scheduled by hand; every step ends in a scheduling barrier, so the compiler keeps the order.  A
    // step is one pixel block of one tap: WB_OB matrix instructions.  Before them the pixel operand of step i + WB_AHEAD
    // is requested from LDS, and in the first WB_OB steps of a tap the weights of one block for the tap after next (the
    // sets rotate: nine taps, three sets, no copies).  The next chunk's tile is requested at the top of a chunk into the
    // buffer that every wave left at the barrier.  Loads return in order: the weights requested behind the tile wait for
    // it (this is where the second workgroup of the compute unit takes over), and by the time the last taps of a chunk
    // have their weights the tile has landed, so the barrier at the end of the chunk is all that the next chunk needs.
    // constants of a batch norm applied in the epilogue (read from global memory there, every one of them would wait behind
    // the stores before it).  Stride 1: mean and invstd in the unused tail of the first buffer's last 1 KB block, gamma and
    // beta in the second buffer's, written now.  Stride 2 (the tails are too short for 256 channels): at the start of the
    // first buffer, written after the last chunk.
    constexpr int CH = OCW * 64;   // channels of this workgroup
    auto bn_lds = [&](int k) {
        return WIDE ? reinterpret_cast<float*>(lds_bytes) + k * CH : reinterpret_cast<float*>(lds_bytes + (k >> 1) * buf_bytes + n_slots * 16) + (k & 1) * CH;
    };
    auto bn_constants_to_lds = [&]() {
        if (BN && threadIdx.x < CH) {
            const int c = blockIdx.y * CH + threadIdx.x;
            bn_lds(0)[threadIdx.x] = e.bn.mean[c];
            bn_lds(1)[threadIdx.x] = e.bn.invstd[c];
            bn_lds(2)[threadIdx.x] = e.bn.gamma[c];
            bn_lds(3)[threadIdx.x] = e.bn.beta[c];
        }
    };
    if constexpr (!WIDE) bn_constants_to_lds();
    uint4 ws[WSETS][WB_OB];
    tile_request(0, 0);
#pragma unroll
    for (int k = 0; k < WSETS - 1; ++k)
#pragma unroll
        for (int o = 0; o < WB_OB; ++o) ws[k][o] = weights_of(o, k, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int ch = 0; ch < n_chunks; ++ch) {
        const bool more = ch + 1 < n_chunks;
        if (more) tile_request(ch + 1, (ch + 1) & 1);
        // byte addresses of the pixel blocks in this chunk's buffer, as opaque values: the reads below are base register
        // plus immediate offset of the tap (left to itself the compiler re-adds the terms of base[] before every read)
        int cur[WB_PB];
#pragma unroll
        for (int pt = 0; pt < WB_PB; ++pt) {
            cur[pt] = base[pt] + (ch & 1) * buf_bytes;
            asm volatile("" : "+v"(cur[pt]));
        }
        auto pixel_operand = [&](int step) {
            const int t = step / WB_PB, pt = step % WB_PB;
            const int tap_off = ((t / 3) * LW + (t % 3)) * 64;
            return *reinterpret_cast<const uint4*>(lds_bytes + cur[pt] + tap_off);
        };
        uint4 ring[WB_AHEAD + 1];
#pragma unroll
        for (int i = 0; i < WB_AHEAD; ++i) ring[i] = pixel_operand(i);
        static_for<STEPS>([&](auto step_c) {
            constexpr int step = decltype(step_c)::value;
            constexpr int t = step / WB_PB, pt = step % WB_PB;
            if constexpr (step + WB_AHEAD < STEPS) ring[(step + WB_AHEAD) % (WB_AHEAD + 1)] = pixel_operand(step + WB_AHEAD);
            if constexpr (pt < WB_OB) {
                // tap t + 2, possibly of the next chunk (the last chunk reads its own first taps again: unused)
                constexpr int tn = (t + WSETS - 1) % TAPS;
                const int nch = (t + WSETS - 1 >= TAPS && more) ? ch + 1 : ch;
                ws[(t + WSETS - 1) % WSETS][pt] = weights_of(pt, tn, nch);
            }
            const uint4 b = ring[step % (WB_AHEAD + 1)];
#pragma unroll
            for (int o = 0; o < WB_OB; ++o) WB_MFMA(acc[o][pt], ws[t % WSETS][o], b);
            __builtin_amdgcn_sched_barrier(0);
        });
        // The tile was requested before this chunk's weight loads, of which 2 * WB_OB * (WSETS - 1) are still wanted in flight
        // (the taps requested ahead).  With three sets that is what the wait allows; with nine it is more than the counter
        // holds, and the wait (all but the 56 youngest have returned) is the one the next chunk's first tap would make anyway.
        if constexpr (WSETS == WB_WSETS_SHARED) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(56)" ::: "memory");
        static_assert(2 * WB_OB * (WB_WSETS_SHARED - 1) == 16 && 2 * WB_OB * (WB_WSETS_ALONE - 1) - 2 * WB_OB == 56 && TAPS % WSETS == 0,
                      "the waits above count the weight loads of the taps requested ahead; the sets rotate once per chunk");
        __syncthreads();
    }

    if constexpr (WIDE && BN) {
        bn_constants_to_lds();
        __syncthreads();
    }
    // the results of the last matrix instructions are not interlocked against vector-unit readers: wait them out, in
    // statements the accumulators pass through, so that no reader moves ahead of the wait
#pragma unroll
    for (int o = 0; o < WB_OB; ++o)
        asm volatile("s_nop 15\n\ts_nop 15"
                     : "+a"(acc[o][0]), "+a"(acc[o][1]), "+a"(acc[o][2]), "+a"(acc[o][3]), "+a"(acc[o][4]), "+a"(acc[o][5]), "+a"(acc[o][6]), "+a"(acc[o][7]));
    // epilogue: the lane holds channels (ob0 + o)*16 + 4*grp .. +3 of pixel ((wpx*WB_PB + pt)*16 + r16) of the tile
    const int64_t pix0 = (int64_t)tile * ((WIDE ? 1 : 2) * WB_PB * 16);
    const int64_t total_pixels = (int64_t)g.total_rows << g.wout_log2;
    const T* add = static_cast<const T*>(e.add);
    T* raw = static_cast<T*>(e.bn.raw);
    // the added tensor is requested for half of the wave's pixel blocks before their first store (see wconv_kernel); what was
    // stored goes back into the accumulation registers for the batch-norm sums, so that the vector registers stay free
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        constexpr int HP = WB_PB / 2;
        typename Act<T>::raw4 addv[HP][WB_OB];
        if (add) {
#pragma unroll
            for (int k = 0; k < HP; ++k) {
                const int64_t p = pix0 + (wpx * WB_PB + half * HP + k) * 16 + r16;
#pragma unroll
                for (int o = 0; o < WB_OB; ++o) {
                    addv[k][o] = Act<T>::zero();
                    if (p < total_pixels) addv[k][o] = Act<T>::load_raw(add + p * NO + (ob0 + o) * 16 + 4 * grp);
                }
            }
        }
#pragma unroll
        for (int o = 0; o < WB_OB; ++o) {
            const int c0 = (ob0 + o) * 16 + 4 * grp;
            f32x4 bn_mu = {0.f, 0.f, 0.f, 0.f}, bn_is = bn_mu, bn_ga = bn_mu, bn_be = bn_mu;
            if constexpr (BN) {
                const int cl = (wo * WB_OB + o) * 16 + 4 * grp;   // channel inside the workgroup's group
                bn_mu = *reinterpret_cast<const f32x4*>(bn_lds(0) + cl);
                bn_is = *reinterpret_cast<const f32x4*>(bn_lds(1) + cl);
                bn_ga = *reinterpret_cast<const f32x4*>(bn_lds(2) + cl);
                bn_be = *reinterpret_cast<const f32x4*>(bn_lds(3) + cl);
            }
#pragma unroll
            for (int k = 0; k < HP; ++k) {
                const int pt = half * HP + k;
                const int64_t p = pix0 + (wpx * WB_PB + pt) * 16 + r16;
                f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
                if (p < total_pixels) {
                    v = acc[o][pt];
                    if (add) v += Act<T>::widen(addv[k][o]);
                    v = Act<T>::rounded(v);  // the sums see what later kernels read back
                    if constexpr (BN) {
                        if (raw) Act<T>::store4(raw + p * NO + c0, v);
                        v = wconv_bn_relu(v, bn_mu, bn_is, bn_ga, bn_be);
                    }
                    Act<T>::store4(y + p * NO + c0, v);
                }
                if (!BN && e.sums) {
                    acc[o][pt] = v;
                    asm volatile("" : "+a"(acc[o][pt]));
                }
            }
        }
    }
    if (!BN && e.sums) {
        // every wave is past its last tile read (barrier after the last chunk): the tile's space carries the lane sums of the
        // first pixel half ([wo][o][sum, sum of squares][lane] vectors) and the per-wave partials ([block][2][16])
        f32x4* hand = lds_raw;
        float* red = reinterpret_cast<float*>(lds_raw + 2 * WB_OB * 2 * 64);
        f32x4 ssum[WB_OB], ssq[WB_OB];
#pragma unroll
        for (int o = 0; o < WB_OB; ++o) ssum[o] = ssq[o] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto lane_sums = [&]() {
#pragma unroll
            for (int o = 0; o < WB_OB; ++o)
#pragma unroll
                for (int pt = 0; pt < WB_PB; ++pt) {
                    const f32x4 v = acc[o][pt];
                    ssum[o] += v;
                    ssq[o] += v * v;
                }
        };
        auto fold_lanes = [&]() {   // the 16 pixels of a lane group, then one lane per group writes its four channels
#pragma unroll
            for (int o = 0; o < WB_OB; ++o) {
#pragma unroll
                for (int s = 1; s < 16; s <<= 1)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        ssum[o][j] += __shfl_xor(ssum[o][j], s, 64);
                        ssq[o][j] += __shfl_xor(ssq[o][j], s, 64);
                    }
                if (r16 == 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        red[((wo * WB_OB + o) * 2 + 0) * 16 + 4 * grp + j] = ssum[o][j];
                        red[((wo * WB_OB + o) * 2 + 1) * 16 + 4 * grp + j] = ssq[o][j];
                    }
                }
            }
        };
        if constexpr (WIDE) {   // a wave has all pixel blocks of its channels
            lane_sums();
            fold_lanes();
        } else {
            if (wpx == 0) {
                lane_sums();
#pragma unroll
                for (int o = 0; o < WB_OB; ++o) {
                    hand[((wo * WB_OB + o) * 2 + 0) * 64 + lane] = ssum[o];
                    hand[((wo * WB_OB + o) * 2 + 1) * 64 + lane] = ssq[o];
                }
            }
            __syncthreads();
            if (wpx == 1) {
#pragma unroll
                for (int o = 0; o < WB_OB; ++o) {
                    ssum[o] = hand[((wo * WB_OB + o) * 2 + 0) * 64 + lane];
                    ssq[o] = hand[((wo * WB_OB + o) * 2 + 1) * 64 + lane];
                }
                lane_sums();
                fold_lanes();
            }
        }
        __syncthreads();
        for (int k = threadIdx.x; k < 2 * CH; k += 256) {
            const int which = k / CH, c = k % CH;
            fixsum_add(e.sums + ((blockIdx.x % FIX_REPLICAS) * 2 + which) * NO + blockIdx.y * CH + c,
                       (double)red[((c >> 4) * 2 + which) * 16 + (c & 15)] * e.scale, e.limit);
        }
    }
}

// the instantiation for a row width and stride: batch norm in the epilogue or not, alone on its compute unit or not
#define WB_ALONE_MAX 256
#define WB_PICK(LW, STRIDE)                                                                                                                 \
    (bn ? (alone ? wconv_block_kernel<LW, STRIDE, true, WB_WSETS_ALONE> : wconv_block_kernel<LW, STRIDE, true, WB_WSETS_SHARED>)            \
        : (alone ? wconv_block_kernel<LW, STRIDE, false, WB_WSETS_ALONE> : wconv_block_kernel<LW, STRIDE, false, WB_WSETS_SHARED>))

// Tile: 256 pixels when the staged chunk fits 64 KB (two workgroups per compute unit), else 128.  The prefetching
// path needs the chunk tile to fit WC_NV vectors per thread and two buffers to fit 80 KB.
template <typename T, int TAPS, int CK>
static int launch_wconv_t(hipStream_t s, int B, int h_in, int h_out, int c_in, int c_out, int stride, int ups, const T* x, const void* w,
                          T* y, const WEpi& e_in) {
    typedef WcTraits<T, TAPS, CK> TR;
    const int pad = TAPS == 9 ? 1 : 0;
    auto geom = [&](int npt) { return make_geom(B, h_in, h_out, c_out, stride, ups, c_in, (npt * 16) / h_out, pad); };
    if (h_out > 128) return -1;
    if constexpr (sizeof(T) == 2 && TAPS == 9 && CK == 32) {
        // launches of at least 128 workgroups of the register-blocked kernel: stride 1 with output channels in multiples of 128,
        // stride 2 in multiples of 256
        const bool small_offsets = (int64_t)B * (ups ? h_in / 2 : h_in) * (ups ? h_in / 2 : h_in) * c_in < (int64_t(1) << 31);
        const size_t fold = (2 * WB_OB * 2 * 64) * sizeof(f32x4) + 4 * WB_OB * 2 * 16 * sizeof(float);   // lane sums + per-wave partials
        // unused 16-byte slots behind a buffer's tile: the epilogue's batch-norm constants need half a slot per channel of the workgroup
        auto tail_slots = [](const ConvGeom& gb) {
            const int n_slots = gb.imgs * gb.in_rows * gb.lw * 4;
            return ((n_slots + 255) & ~255) - n_slots;
        };
        auto launch_block = [&](auto kern, const ConvGeom& gb, int oc_wg) {
            const int n_slots = gb.imgs * gb.in_rows * gb.lw * 4;
            size_t lds_b = 2 * (size_t)((n_slots + 255) & ~255) * 16;
            if (lds_b < fold) lds_b = fold;
            WEpi eb = e_in;
            eb.limit = 576460752303423488.0 / (double)((gb.n_tiles + FIX_REPLICAS - 1) / FIX_REPLICAS);   // 2^59 over the partials one word takes
            if (lds_b > 65536) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_b);
            hipLaunchKernelGGL(kern, dim3(gb.n_tiles, c_out / oc_wg), dim3(256), lds_b, s, x, w, y, eb, gb, c_in);
        };
        if (stride == 1 && c_out % 128 == 0 && c_in % 32 == 0 && small_offsets) {
            const ConvGeom gb = geom(2 * WB_PB);
            const bool shape = (gb.lw == 34 && gb.in_rows == 10) || (gb.lw == 18 && gb.in_rows == 18) || (gb.lw == 10 && gb.in_rows == 10);
            if (shape && gb.imgs * gb.in_rows * gb.lw * 4 <= 256 * WB_NV && tail_slots(gb) >= 128 / 2 && (int64_t)gb.n_tiles * (c_out / 128) >= 128) {
                const bool bn = e_in.bn.mean != nullptr;
                const bool alone = (int64_t)gb.n_tiles * (c_out / 128) <= WB_ALONE_MAX;
                if (gb.lw == 34) launch_block(WB_PICK(34, 1), gb, 128);
                else if (gb.lw == 18) launch_block(WB_PICK(18, 1), gb, 128);
                else launch_block(WB_PICK(10, 1), gb, 128);
                return 0;
            }
        }
        if (stride == 2 && !ups && c_out % 256 == 0 && c_in % 32 == 0 && small_offsets) {
            const ConvGeom gb = geom(WB_PB);
            const bool shape = (gb.lw == 34 || gb.lw == 18) && gb.in_rows == 17;
            if (shape && gb.imgs * gb.in_rows * gb.lw * 4 <= 256 * WB_NV_STRIDE2 && (int64_t)gb.n_tiles * (c_out / 256) >= 128) {
                const bool bn = e_in.bn.mean != nullptr;
                const bool alone = (int64_t)gb.n_tiles * (c_out / 256) <= WB_ALONE_MAX;
                if (gb.lw == 34) launch_block(WB_PICK(34, 2), gb, 256);
                else launch_block(WB_PICK(18, 2), gb, 256);
                return 0;
            }
        }
    }
    int sub = 0;
    if (TAPS == 1 && stride == 2 && !ups && h_in == 2 * h_out) {
        // a 1x1 stride-2 filter as a stride-1 layer over the pixels it reads; only the prefetching path knows how to fetch them
        const ConvGeom gs = make_geom(B, h_out, h_out, c_out, 1, 0, c_in, 256 / h_out, 0);
        const size_t ls = wconv_lds_bytes<T, TAPS, CK>(gs);
        if (256 / h_out >= 1 && ls <= 65536 && gs.imgs * gs.in_rows * gs.lw * TR::CV <= 256 * WC_NV && 2 * ls <= 80 * 1024 && c_in / CK > 1) {
            sub = 1;
            h_in = h_out;
            stride = 1;
        }
    }
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
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, x, w, y, e, g, c_in, pipelined, sub);
    } else {
        auto kern = wconv_kernel<T, TAPS, CK, 8>;
        if (lds > 65536) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, x, w, y, e, g, c_in, pipelined, sub);
    }
    return 0;
}

// c_in is 16 or a multiple of 32, c_out a multiple of 16, maps are squares with power-of-two sides.
// Returns 0, or -1 when the shape is outside what the kernel is built for (nothing is launched then).
int launch_wconv(hipStream_t s, int act, int taps, int B, int h_in, int h_out, int c_in, int c_out, int stride, int ups, const void* x,
                 const void* w, void* y, const void* add, fixsum_t* sums, double scale, const WconvBn* bn) {
    if (!(c_in == 16 || c_in % 32 == 0) || c_out % 16 != 0 || (taps != 9 && taps != 1) || (bn && sums)) return -1;
    WEpi e{add, sums, scale, 0.0, bn ? *bn : WconvBn{nullptr, nullptr, nullptr, nullptr, nullptr}};
    int rc = -1;
    ACT_DISPATCH(act, {
        if (taps == 9) rc = c_in == 16 ? launch_wconv_t<T, 9, 16>(s, B, h_in, h_out, c_in, c_out, stride, ups, (const T*)x, w, (T*)y, e)
                                       : launch_wconv_t<T, 9, 32>(s, B, h_in, h_out, c_in, c_out, stride, ups, (const T*)x, w, (T*)y, e);
        else rc = c_in == 16 ? launch_wconv_t<T, 1, 16>(s, B, h_in, h_out, c_in, c_out, stride, ups, (const T*)x, w, (T*)y, e)
                             : launch_wconv_t<T, 1, 32>(s, B, h_in, h_out, c_in, c_out, stride, ups, (const T*)x, w, (T*)y, e);
    });
    return rc;
}
