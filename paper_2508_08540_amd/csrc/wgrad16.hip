// Weight gradient of wide bf16 layers on the bf16 matrix instruction: the convolution part of the stochastic gradient in the
// local SGD update of a fast worker (Section 2, the local update rule; fast-worker branch of Algorithm 1).
//
// dW[o][tap][i] = sum over pixels p of dy[p][o] * x[p + tap][i] contracts over pixels, so both operands of
// v_mfma_f32_16x16x16_bf16 must supply four *consecutive pixels* of one channel per lane.  Activations are
// stored pixel-major with channels innermost, therefore the staging transposes 4x4 (pixel x channel) blocks in
// registers and keeps channel-major planes in LDS: dyT[64 output channels][128 pixels] and
// xT[64 input channels][rows with halo][row width + 4].  A k-step takes 16 consecutive output pixels; lane
// group g reads the aligned pixel quad 4g of its channel (A: output channel lane%16 of the wave's block,
// B: input channel lane%16 of one of four 16-channel blocks).  For a 3x3 filter the horizontal tap shifts the
// x quad by 0, 1 or 2 pixels: the two aligned quads around it are read once and the shifted operands are cut
// out with alignbit, so no shifted copies of the tile are needed.
// Workgroup = (pixel group, 64 output channels, 64 input channels); wave w owns output-channel block w with
// all four input-channel blocks and all taps (36 accumulators for 3x3).  Waves own distinct 16x16 blocks, so
// the sums go from registers straight into the replicated 64-bit fixed-point accumulators (same layout and
// scale as wgrad_kernel: block (ob, ib), element (t*4 + j)*64 + lane).
// Covers stride 1, channel counts that are multiples of 64.
//
// Layers of at most 64 channels (multiples of 16; the narrow residual network) have few pixels per channel pair, and a
// workgroup that owned 64 x 64 channels would leave most of the machine idle or dump its 36 864 sums from too many pixel
// groups.  wgrad16_pair_kernel keeps wgrad_kernel's decomposition instead: workgroup = (pixel group, 16 x 16 channel
// block), the four waves take the k-steps of a 512-pixel tile in turn, fold their nine accumulators through LDS in wave
// order and add 2304 sums; staging and operands are those described above, for one 16-channel slice of x and of dy.
// Other layers use wgrad_kernel.
#include "conv_tile.h"


#define FIX_WGRAD_SCALE 1099511627776.0  // 2^40, as in wgrad_kernel
#define W16_TILE_PX 128
#define W16_XT 4   // staging tasks of x and of dy that a thread prefetches for the next tile
#define W16_DT 2

struct W16Geom {
    int lwp;   // LDS row width of an xT plane: w_out + 4 (3x3) or w_out (1x1)
    int xp;    // elements per xT plane (xp / 4 odd: channel rows fall into different banks)
    int dp;    // elements per dyT row
};

template <int TAPS>
__global__ __launch_bounds__(256) void wgrad16_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy, fixsum_t* __restrict__ gacc,
                                                      ConvGeom g, W16Geom wg, int tiles_per_group, int NI, int NO, int replicas, int64_t rstride) {
    if (rstride) {   // one replica of several: every buffer sits blockIdx.z slots further
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        x = rep_at(x, ro); dy = rep_at(dy, ro); gacc = rep_at(gacc, ro);
    }
    extern __shared__ uint2 lds2[];
    uint2* xT = lds2;                       // [64][xp / 4] quads
    uint2* dyT = lds2 + 64 * (wg.xp / 4);   // [64][dp / 4] quads
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, grp = lane >> 4;
    const int nib = NI >> 6;
    const int cob = blockIdx.y / nib, cib = blockIdx.y - cob * nib;
    const int W = g.h_out, pad = g.pad;
    const int rpi = 1 << g.rpi_log2;
    const int64_t total_pixels = (int64_t)g.total_rows << g.wout_log2;
    const int xq = wg.xp >> 2, dq = wg.dp >> 2, lwq = wg.lwp >> 2;

    f32x4 acc[TAPS][4];
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[t][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int tile_begin = blockIdx.x * tiles_per_group;
    const int tile_end = min(g.n_tiles, tile_begin + tiles_per_group);
    // Staging.  A task is (4 channels, 4 consecutive pixels): four 8-byte loads, a 4x4 transpose in registers, four 8-byte
    // LDS writes; for x the pixels are padded columns of one staged row.  The loads of a thread's first W16_XT + W16_DT
    // tasks of the next tile are requested before the matrix instructions of the current one (a tile has 800 .. 1100 tasks of
    // x and 512 of dy for 256 threads; taken one after the other they cost five to six memory round trips per tile, ten
    // times the tile's matrix work); tasks beyond those are loaded when the tile is written.
    const int rows_total = g.imgs * g.in_rows;
    const int x_tasks = 16 * rows_total * lwq, d_tasks = 16 * (W16_TILE_PX / 4);
    uint2 rx[W16_XT][4], rd[W16_DT][4];
    auto x_task = [&](int tile, int id, uint2 (&r)[4]) {   // requests the four pixels of task id; returns its LDS quad or -1
        if (id >= x_tasks) return -1;
        const int cq = id & 15, rest = id >> 4;
        const int lr = rest / lwq, pq = rest - lr * lwq;
        const int part = lr / g.in_rows, li = lr - part * g.in_rows;
        const int grow = tile * g.rows_tile + part * rpi;
        const int n = grow >> g.wout_log2;
        const int hi = (grow & (g.h_out - 1)) - pad + li;
        const bool rok = n < g.B && (unsigned)hi < (unsigned)g.h_in;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int wi = pq * 4 + j - pad;
            r[j] = make_uint2(0u, 0u);
            if (rok && (unsigned)wi < (unsigned)W)
                r[j] = *reinterpret_cast<const uint2*>(x + (((int64_t)n * g.h_in + hi) * g.h_in + wi) * NI + cib * 64 + cq * 4);
        }
        return (cq * 4) * xq + lr * lwq + pq;
    };
    auto d_task = [&](int tile, int id, uint2 (&r)[4]) {
        if (id >= d_tasks) return -1;
        const int cq = id & 15, pq = id >> 4;
        const int64_t pix0 = (int64_t)tile * W16_TILE_PX;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t p = pix0 + pq * 4 + j;
            r[j] = make_uint2(0u, 0u);
            if (p < total_pixels) r[j] = *reinterpret_cast<const uint2*>(dy + p * NO + cob * 64 + cq * 4);
        }
        return (cq * 4) * dq + pq;
    };
    auto transpose_store = [](uint2* dst, int pitch, const uint2 (&r)[4]) {
        dst[0 * pitch] = make_uint2((r[0].x & 0xffffu) | (r[1].x << 16), (r[2].x & 0xffffu) | (r[3].x << 16));
        dst[1 * pitch] = make_uint2((r[0].x >> 16) | (r[1].x & 0xffff0000u), (r[2].x >> 16) | (r[3].x & 0xffff0000u));
        dst[2 * pitch] = make_uint2((r[0].y & 0xffffu) | (r[1].y << 16), (r[2].y & 0xffffu) | (r[3].y << 16));
        dst[3 * pitch] = make_uint2((r[0].y >> 16) | (r[1].y & 0xffff0000u), (r[2].y >> 16) | (r[3].y & 0xffff0000u));
    };
    int x_at[W16_XT], d_at[W16_DT];
    auto request = [&](int tile) {
#pragma unroll
        for (int k = 0; k < W16_XT; ++k) x_at[k] = x_task(tile, k * 256 + (int)threadIdx.x, rx[k]);
#pragma unroll
        for (int k = 0; k < W16_DT; ++k) d_at[k] = d_task(tile, k * 256 + (int)threadIdx.x, rd[k]);
    };
    if (tile_begin < tile_end) request(tile_begin);
    for (int tile = tile_begin; tile < tile_end; ++tile) {
        __syncthreads();  // previous tile consumed
#pragma unroll
        for (int k = 0; k < W16_XT; ++k)
            if (x_at[k] >= 0) transpose_store(xT + x_at[k], xq, rx[k]);
#pragma unroll
        for (int k = 0; k < W16_DT; ++k)
            if (d_at[k] >= 0) transpose_store(dyT + d_at[k], dq, rd[k]);
        for (int id = W16_XT * 256 + threadIdx.x; id < x_tasks; id += 256) {   // what the prefetch registers do not cover
            uint2 r[4];
            const int at = x_task(tile, id, r);
            transpose_store(xT + at, xq, r);
        }
        for (int id = W16_DT * 256 + threadIdx.x; id < d_tasks; id += 256) {
            uint2 r[4];
            const int at = d_task(tile, id, r);
            transpose_store(dyT + at, dq, r);
        }
        __syncthreads();
        if (tile + 1 < tile_end) request(tile + 1);
        // ---- 8 k-steps of 16 pixels -------------------------------------------------------------------------
        const uint2* arow = dyT + (wave * 16 + r16) * dq + grp;
        const uint2* brow = xT + r16 * xq;
#pragma unroll 1
        for (int ks = 0; ks < W16_TILE_PX / 16; ++ks) {
            const s16x4 a = __builtin_bit_cast(s16x4, arow[ks * 4]);
            const int q = ks * 16 + 4 * grp;                      // first pixel of this lane group's quad inside the tile
            const int orow = q >> g.wout_log2, ocol = q & (W - 1);
            const int part = orow >> g.rpi_log2, rr = orow & (rpi - 1);
            const int xoff = (part * g.in_rows + rr) * lwq + (ocol >> 2);  // quad index of tap (0, 0)
            if (TAPS == 9) {
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) {
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const uint2 q0 = brow[b * 16 * xq + xoff + kh * lwq];
                        const uint2 q1 = brow[b * 16 * xq + xoff + kh * lwq + 1];
                        // pixels shifted by one and by two columns
                        const uint2 s1 = make_uint2(__builtin_amdgcn_alignbit(q0.y, q0.x, 16), __builtin_amdgcn_alignbit(q1.x, q0.y, 16));
                        const uint2 s2 = make_uint2(q0.y, q1.x);
                        acc[kh * 3 + 0][b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(s16x4, q0), acc[kh * 3 + 0][b], 0, 0, 0);
                        acc[kh * 3 + 1][b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(s16x4, s1), acc[kh * 3 + 1][b], 0, 0, 0);
                        acc[kh * 3 + 2][b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(s16x4, s2), acc[kh * 3 + 2][b], 0, 0, 0);
                    }
                }
            } else {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint2 q0 = brow[b * 16 * xq + xoff];
                    acc[0][b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(s16x4, q0), acc[0][b], 0, 0, 0);
                }
            }
        }
    }
    // accumulators: block (ob, ib) of 16 * TAPS * 16 values, element (t*4 + j)*64 + lane
    constexpr int BLOCK_FLOATS = 16 * TAPS * 16;
    const int nblocks = (NO >> 4) * (NI >> 4);
    fixsum_t* rep = gacc + (int64_t)(blockIdx.x % replicas) * nblocks * BLOCK_FLOATS;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        fixsum_t* out = rep + (int64_t)((cob * 4 + wave) * (NI >> 4) + cib * 4 + b) * BLOCK_FLOATS + lane;
#pragma unroll
        for (int t = 0; t < TAPS; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) fixsum_add(out + (t * 4 + j) * 64, (double)acc[t][b][j] * FIX_WGRAD_SCALE);
    }
}

#define W16P_TILE_PX 512
#define W16P_XT 4   // staging tasks of x and of dy whose loads a thread keeps in flight together
#define W16P_DT 2

template <int TAPS>
__global__ __launch_bounds__(256) void wgrad16_pair_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy, fixsum_t* __restrict__ gacc,
                                                           ConvGeom g, W16Geom wg, int tiles_per_group, int NI, int NO, int replicas, int64_t rstride) {
    if (rstride) {   // one replica of several: every buffer sits blockIdx.z slots further
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        x = rep_at(x, ro); dy = rep_at(dy, ro); gacc = rep_at(gacc, ro);
    }
    extern __shared__ uint2 lds2[];
    uint2* xT = lds2;                       // [16][xp / 4] quads
    uint2* dyT = lds2 + 16 * (wg.xp / 4);   // [16][dp / 4] quads
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, grp = lane >> 4;
    const int nib = NI >> 4;
    const int ob = blockIdx.y / nib, ib = blockIdx.y - ob * nib;
    const int W = g.h_out, pad = g.pad;
    const int rpi = 1 << g.rpi_log2;
    const int tile_pixels = g.rows_tile << g.wout_log2;
    const int64_t total_pixels = (int64_t)g.total_rows << g.wout_log2;
    const int xq = wg.xp >> 2, dq = wg.dp >> 2, lwq = wg.lwp >> 2;

    f32x4 acc[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int tile_begin = blockIdx.x * tiles_per_group;
    const int tile_end = min(g.n_tiles, tile_begin + tiles_per_group);
    for (int tile = tile_begin; tile < tile_end; ++tile) {
        __syncthreads();  // previous tile consumed
        const int row0 = tile * g.rows_tile;
        // ---- stage x and dy.  A task is (4 channels, 4 consecutive pixels): four 8-byte loads, a 4x4 transpose in
        // registers, four 8-byte LDS writes.  For x the pixels are padded columns of one staged row.  The loads of up
        // to W16P_XT + W16P_DT tasks per thread are all requested before the first transpose waits for any of them.
        const int rows_total = g.imgs * g.in_rows;
        const int x_tasks = 4 * rows_total * lwq, d_tasks = tile_pixels;   // 4 channel quads x (positions / 4)
        const int64_t pix0 = (int64_t)tile * tile_pixels;
        auto transpose_store = [](uint2* dst, int pitch, const uint2 (&r)[4]) {
            dst[0 * pitch] = make_uint2((r[0].x & 0xffffu) | (r[1].x << 16), (r[2].x & 0xffffu) | (r[3].x << 16));
            dst[1 * pitch] = make_uint2((r[0].x >> 16) | (r[1].x & 0xffff0000u), (r[2].x >> 16) | (r[3].x & 0xffff0000u));
            dst[2 * pitch] = make_uint2((r[0].y & 0xffffu) | (r[1].y << 16), (r[2].y & 0xffffu) | (r[3].y << 16));
            dst[3 * pitch] = make_uint2((r[0].y >> 16) | (r[1].y & 0xffff0000u), (r[2].y >> 16) | (r[3].y & 0xffff0000u));
        };
        for (int xb = 0, db = 0; xb < x_tasks || db < d_tasks; xb += W16P_XT * 256, db += W16P_DT * 256) {
            uint2 rx[W16P_XT][4], rd[W16P_DT][4];
            int x_dst[W16P_XT];
#pragma unroll
            for (int k = 0; k < W16P_XT; ++k) {
                const int id = xb + k * 256 + threadIdx.x;
                const int cq = id & 3, rest = id >> 2;
                const int lr = rest / lwq, pq = rest - lr * lwq;
                const int part = lr / g.in_rows, li = lr - part * g.in_rows;
                const int grow = row0 + part * rpi;
                const int n = grow >> g.wout_log2;
                const int hi = (grow & (g.h_out - 1)) - pad + li;
                const bool rok = id < x_tasks && n < g.B && (unsigned)hi < (unsigned)g.h_in;
                x_dst[k] = id < x_tasks ? (cq * 4) * xq + lr * lwq + pq : -1;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int wi = pq * 4 + j - pad;
                    rx[k][j] = make_uint2(0u, 0u);
                    if (rok && (unsigned)wi < (unsigned)W)
                        rx[k][j] = *reinterpret_cast<const uint2*>(x + (((int64_t)n * g.h_in + hi) * g.h_in + wi) * NI + ib * 16 + cq * 4);
                }
            }
#pragma unroll
            for (int k = 0; k < W16P_DT; ++k) {
                const int id = db + k * 256 + threadIdx.x;
                const int cq = id & 3, pq = id >> 2;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t p = pix0 + pq * 4 + j;
                    rd[k][j] = make_uint2(0u, 0u);
                    if (id < d_tasks && p < total_pixels) rd[k][j] = *reinterpret_cast<const uint2*>(dy + p * NO + ob * 16 + cq * 4);
                }
            }
#pragma unroll
            for (int k = 0; k < W16P_XT; ++k)
                if (x_dst[k] >= 0) transpose_store(xT + x_dst[k], xq, rx[k]);
#pragma unroll
            for (int k = 0; k < W16P_DT; ++k) {
                const int id = db + k * 256 + threadIdx.x;
                if (id < d_tasks) transpose_store(dyT + ((id & 3) * 4) * dq + (id >> 2), dq, rd[k]);
            }
        }
        __syncthreads();
        // ---- k-steps of 16 pixels, taken by the waves in turn ------------------------------------------------
        const uint2* arow = dyT + r16 * dq + grp;
        const uint2* brow = xT + r16 * xq;
        for (int ks = wave; ks < (tile_pixels >> 4); ks += 4) {
            const s16x4 a = __builtin_bit_cast(s16x4, arow[ks * 4]);
            const int q = ks * 16 + 4 * grp;                      // first pixel of this lane group's quad inside the tile
            const int orow = q >> g.wout_log2, ocol = q & (W - 1);
            const int part = orow >> g.rpi_log2, rr = orow & (rpi - 1);
            const int xoff = (part * g.in_rows + rr) * lwq + (ocol >> 2);  // quad index of tap (0, 0)
            if (TAPS == 9) {
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) {
                    const uint2 q0 = brow[xoff + kh * lwq];
                    const uint2 q1 = brow[xoff + kh * lwq + 1];
                    // pixels shifted by one and by two columns
                    const uint2 s1 = make_uint2(__builtin_amdgcn_alignbit(q0.y, q0.x, 16), __builtin_amdgcn_alignbit(q1.x, q0.y, 16));
                    const uint2 s2 = make_uint2(q0.y, q1.x);
                    acc[kh * 3 + 0] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(s16x4, q0), acc[kh * 3 + 0], 0, 0, 0);
                    acc[kh * 3 + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(s16x4, s1), acc[kh * 3 + 1], 0, 0, 0);
                    acc[kh * 3 + 2] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(s16x4, s2), acc[kh * 3 + 2], 0, 0, 0);
                }
            } else {
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(s16x4, brow[xoff]), acc[0], 0, 0, 0);
            }
        }
    }
    // Fold the four waves in wave order; element (t*4 + j)*64 + lane holds dW[o = 4*(lane/16) + j][t][i = lane%16] of the
    // block, the layout of wgrad_kernel's accumulators.
    constexpr int BLOCK_FLOATS = 16 * TAPS * 16;
    float* fold = reinterpret_cast<float*>(lds2);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) fold[wave * BLOCK_FLOATS + (t * 4 + j) * 64 + lane] = acc[t][j];
    __syncthreads();
    fixsum_t* out = gacc + ((int64_t)(blockIdx.x % replicas) * gridDim.y + blockIdx.y) * BLOCK_FLOATS;
    for (int e = threadIdx.x; e < BLOCK_FLOATS; e += 256) {
        float v = fold[e];
#pragma unroll
        for (int wv = 1; wv < 4; ++wv) v += fold[wv * BLOCK_FLOATS + e];
        fixsum_add(out + e, (double)v * FIX_WGRAD_SCALE);
    }
}

// ---- 3x3 layers on 8 x 8, 16 x 16 and 32 x 32 maps: 32 x 32 channel blocks per wave, 32 pixels per matrix instruction --------
// Workgroup = (pixel group, 64 output channels, 64 input channels) of two teams of four waves; a team walks every other tile
// of the group with accumulators of its own (folded through LDS in team order at the end, so the workgroup adds its sums
// once).  A wave owns 32 x 32 channels: 2 x 2 blocks x 9 taps of v_mfma_f32_16x16x32_bf16.
// A tile is 128 consecutive output pixels (four rows of a 32-wide map, half a 16 x 16 map, two 8 x 8 maps) in four steps
// of 32; lane group g of a step takes 8 consecutive pixels of one row, and the assignment of pixels to (step, group) is the
// same for dy and x, which is all the contraction needs: group g keeps its columns and moves one row down per step.
// LDS holds one plane per channel (dy: the 128 pixels; x: the staged rows of the tile with their halo rows, each row
// followed by eight zero pixels that serve as the right border of this row and the left border of the next).  An operand
// is one aligned 16-byte read of 8 pixels; the operands of the left and right taps are cut out of it and the two
// neighbouring pixel pairs with alignbit.  Planes of channel group c / 8 start 16 bytes later than those of the group
// before (measured: 8-byte staging writes of eight channel groups then spread over the banks; the 16-byte reads run at
// full rate at either pitch).
// Staging: a task is 8 channels x 4 pixels: four 16-byte loads (eight lanes cover the 128 contiguous bytes of a pixel's 64
// channels), a transpose in registers, eight 8-byte LDS writes.  A thread has one task of dy and up to two of x per tile;
// their loads for the next tile are requested before the matrix instructions of the current one.
#define WT_PX 128
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

template <int WLOG>
struct WtGeom {
    static constexpr int W = 1 << WLOG;                        // map width and height
    static constexpr int BANDS = W == 8 ? 2 : 1;               // image parts per tile (two whole 8 x 8 maps)
    static constexpr int BROWS = WT_PX / W / BANDS;            // output rows per band: 4, 8, 8
    static constexpr int RB = BROWS + 2;                       // staged rows per band
    static constexpr int RP = W + 8;                           // pixels per staged row, the zeros included
    static constexpr int XPX = BANDS * RB * RP;                // pixels per x plane
    static constexpr int PPX = 16 + 2 * XPX + 112 + (W == 8 ? 16 : 0);   // bytes from plane to plane: 608, 608, 784
    static constexpr int PPD = 2 * WT_PX + 112;                // 368
    static constexpr int TEAM_BYTES = 64 * (PPX + PPD);
    static constexpr int XTASKS = 8 * BANDS * RB * (W / 4);    // 384, 320, 320
    // a plane holds its lead, the largest skew (7 channel groups) and its pixels; a thread has at most two x tasks; both teams'
    // tiles fit the 160 KB of a compute unit and are at least as large as the fold buffer of the epilogue
    static_assert(PPX >= 16 + 7 * 16 + 2 * XPX && PPD >= 7 * 16 + 2 * WT_PX && PPX % 16 == 0 && PPD % 16 == 0, "plane pitch");
    static_assert(XTASKS <= 512, "staging tasks per thread");
    static_assert(2 * TEAM_BYTES <= 160 * 1024 && 2 * TEAM_BYTES >= 4 * 18 * 4 * 64 * 4, "LDS of a workgroup");
};

template <int WLOG>
__global__ __launch_bounds__(512) void wgrad16_tile_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy, fixsum_t* __restrict__ gacc,
                                                           int B, int NI, int NO, int n_tiles, int tiles_per_group, int64_t rstride) {
    typedef WtGeom<WLOG> G;
    constexpr int W = G::W, RP = G::RP, PPX = G::PPX, PPD = G::PPD;
    if (rstride) {   // one replica of several: every buffer sits blockIdx.z slots further
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        x = rep_at(x, ro); dy = rep_at(dy, ro); gacc = rep_at(gacc, ro);
    }
    extern __shared__ uint4 lds16[];
    const int team = threadIdx.x >> 8, tid = threadIdx.x & 255;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    const int nib = NI >> 6;
    const int cob = blockIdx.y / nib, cib = blockIdx.y - cob * nib;
    char* const xT = reinterpret_cast<char*>(lds16) + team * G::TEAM_BYTES;
    char* const dT = xT + 64 * PPX;
    const int64_t total_px = (int64_t)B * W * W;

    // pads and borders are zero for the whole launch: the staging only ever writes pixels of the map
    for (int i = tid; i < G::TEAM_BYTES / 16; i += 256) reinterpret_cast<uint4*>(xT)[i] = make_uint4(0u, 0u, 0u, 0u);

    f32x4 acc[2][2][9];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int t = 0; t < 9; ++t) acc[a][b][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- staging tasks of this thread -----------------------------------------------------------------------------------
    const int cg = tid & 7;
    const int qd = tid >> 3;                                   // pixel quad of the dy task
    char* const d_dst = dT + 8 * cg * PPD + cg * 16 + 8 * qd;
    int x_row[2], x_band[2], x_col[2];
    char* x_dst[2];
    bool x_on[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int id = tid + 256 * k;
        x_on[k] = id < G::XTASKS;
        const int qx = id >> 3;
        const int row = qx >> (WLOG - 2);
        x_col[k] = 4 * (qx & (W / 4 - 1));
        x_band[k] = (G::BANDS == 2 && row >= G::RB) ? 1 : 0;
        x_row[k] = row - x_band[k] * G::RB;
        x_dst[k] = xT + 8 * cg * PPX + cg * 16 + 16 + 2 * (row * RP + x_col[k]);
    }
    u32x4_t rd[4], rx[2][4];
    auto request = [&](int tile) {
        const int64_t p0 = (int64_t)tile * WT_PX + 4 * qd;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            rd[j] = u32x4_t{0u, 0u, 0u, 0u};
            if (tile < n_tiles && p0 + j < total_px) rd[j] = *reinterpret_cast<const u32x4_t*>(dy + (p0 + j) * NO + cob * 64 + 8 * cg);
        }
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int grow = tile * (WT_PX / W) + x_band[k] * G::BROWS;   // first output row of the band, counted over all images
            const int n = grow >> WLOG;
            const int h = (grow & (W - 1)) - 1 + x_row[k];
            const bool ok = x_on[k] && tile < n_tiles && n < B && (unsigned)h < (unsigned)W;
            const bf16_t* p = x + ((((int64_t)n << WLOG) + h) * W + x_col[k]) * NI + cib * 64 + 8 * cg;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                rx[k][j] = u32x4_t{0u, 0u, 0u, 0u};
                if (ok) rx[k][j] = *reinterpret_cast<const u32x4_t*>(p + (int64_t)j * NI);
            }
        }
    };
    // v[j] = 8 channels of pixel j; plane e of the task's channel group receives pixels 0 .. 3 of channel e
    auto put = [](char* dst, int pp, const u32x4_t (&v)[4]) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint32_t lo0 = __builtin_amdgcn_perm(v[1][m], v[0][m], 0x05040100u), lo1 = __builtin_amdgcn_perm(v[3][m], v[2][m], 0x05040100u);
            const uint32_t hi0 = __builtin_amdgcn_perm(v[1][m], v[0][m], 0x07060302u), hi1 = __builtin_amdgcn_perm(v[3][m], v[2][m], 0x07060302u);
            *reinterpret_cast<u32x2_t*>(dst + (2 * m) * pp) = u32x2_t{lo0, lo1};
            *reinterpret_cast<u32x2_t*>(dst + (2 * m + 1) * pp) = u32x2_t{hi0, hi1};
        }
    };
    auto store_tile = [&]() {
        put(d_dst, PPD, rd);
#pragma unroll
        for (int k = 0; k < 2; ++k)
            if (x_on[k]) put(x_dst[k], PPX, rx[k]);
    };

    // ---- operand addresses of this lane ------------------------------------------------------------------------------------
    // pixel offsets of lane group g at step 0, tap row 0: in the dy plane and in the x plane (whose row 0 is the halo row)
    int d_off, x_off;
    if (W == 32) { d_off = 8 * g; x_off = 8 * g; }
    else if (W == 16) { d_off = 64 * (g >> 1) + 8 * (g & 1); x_off = 4 * (g >> 1) * RP + 8 * (g & 1); }
    else { d_off = 32 * g; x_off = (g >> 1) * G::RB * RP + 4 * (g & 1) * RP; }
    const int ca = 32 * wm + r, cb = 32 * wn + r;   // channels of block 0; block 1 is 16 channels = two channel groups further
    const char* const a_base = dT + ca * PPD + (ca >> 3) * 16 + 2 * d_off;
    const char* const b_base = xT + cb * PPX + (cb >> 3) * 16 + 16 + 2 * x_off;
    auto compute = [&]() {
#pragma unroll 1
        for (int step = 0; step < 4; ++step) {
            bf16x8_t a[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
                a[mb] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(a_base + mb * (16 * PPD + 32) + 2 * W * step));
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) {
                    const char* p = b_base + nb * (16 * PPX + 32) + 2 * RP * (step + kh);
                    const u32x4_t c = *reinterpret_cast<const u32x4_t*>(p);
                    // the pixel pairs on either side of the eight; on 8-wide maps they are always the zeros between two rows
                    uint32_t left = 0u, right = 0u;
                    if (W >= 16) {
                        left = *reinterpret_cast<const uint32_t*>(p - 4);
                        right = *reinterpret_cast<const uint32_t*>(p + 16);
                    }
                    const uint32_t s01 = __builtin_amdgcn_alignbit(c[1], c[0], 16), s12 = __builtin_amdgcn_alignbit(c[2], c[1], 16),
                                   s23 = __builtin_amdgcn_alignbit(c[3], c[2], 16);
                    const bf16x8_t o0 = __builtin_bit_cast(bf16x8_t, (u32x4_t{__builtin_amdgcn_alignbit(c[0], left, 16), s01, s12, s23}));
                    const bf16x8_t o1 = __builtin_bit_cast(bf16x8_t, c);
                    const bf16x8_t o2 = __builtin_bit_cast(bf16x8_t, (u32x4_t{s01, s12, s23, __builtin_amdgcn_alignbit(right, c[3], 16)}));
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb) {
                        acc[mb][nb][kh * 3 + 0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mb], o0, acc[mb][nb][kh * 3 + 0], 0, 0, 0);
                        acc[mb][nb][kh * 3 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mb], o1, acc[mb][nb][kh * 3 + 1], 0, 0, 0);
                        acc[mb][nb][kh * 3 + 2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mb], o2, acc[mb][nb][kh * 3 + 2], 0, 0, 0);
                    }
                }
        }
    };

    // ---- the team's tiles: tile_begin + team, + 2, ...; both teams make the same number of turns ----------------------------
    const int tile_begin = blockIdx.x * tiles_per_group;
    const int tile_end = min(n_tiles, tile_begin + tiles_per_group);
    const int turns = (tile_end - tile_begin + 1) >> 1;
    int tile = tile_begin + team;
    if (turns > 0) request(tile < tile_end ? tile : n_tiles);
    __syncthreads();   // zeros in place
    for (int turn = 0; turn < turns; ++turn, tile += 2) {
        store_tile();
        __syncthreads();
        if (turn + 1 < turns) request(tile + 2 < tile_end ? tile + 2 : n_tiles);
        if (tile < tile_end) compute();
        __syncthreads();   // the tile is consumed
    }

    // ---- team 1's sums go to team 0 through LDS, block row by block row; team 0 adds the sums of the workgroup ---------------
    float* const fold = reinterpret_cast<float*>(lds16);   // [4 waves][18 blocks][4][64]
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        if (team == 1) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int t = 0; t < 9; ++t)
#pragma unroll
                    for (int j = 0; j < 4; ++j) fold[((wave * 18 + nb * 9 + t) * 4 + j) * 64 + lane] = acc[mb][nb][t][j];
        }
        __syncthreads();
        if (team == 0) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int t = 0; t < 9; ++t)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[mb][nb][t][j] += fold[((wave * 18 + nb * 9 + t) * 4 + j) * 64 + lane];
        }
        __syncthreads();
    }
    if (team != 0) return;
    // The sums leave as floats, one copy per pixel group behind the layer's accumulator words (block (ob, ib) of
    // 16 * 9 * 16 values, element (t*4 + j)*64 + lane, as in the accumulators); wgrad16_fold_kernel converts and adds them.
    constexpr int BLOCK_FLOATS = 16 * 9 * 16;
    const int64_t weights = (int64_t)NO * 9 * NI;
    float* part = reinterpret_cast<float*>(gacc + weights) + (int64_t)blockIdx.x * weights;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            float* out = part + (int64_t)((cob * 4 + 2 * wm + mb) * (NI >> 4) + cib * 4 + 2 * wn + nb) * BLOCK_FLOATS + lane;
#pragma unroll
            for (int t = 0; t < 9; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j) out[(t * 4 + j) * 64] = acc[mb][nb][t][j];
        }
}

// Every pixel group's partial sum of a weight is converted to fixed point by itself, range-checked, and the integers are
// added to the layer's accumulator word: the word ends as if every workgroup had added its sums with an atomic, without
// the 9.4 million 64-bit atomics that cost more than the matrix work.  A thread owns four consecutive words; with SL = 4
// (layers with many pixel groups and few weights) wave w takes the groups w, w + 4, ... and the four waves' integers meet
// in LDS.  Eight loads are in flight per thread.  The launch is the only writer of the layer's words while it runs.
template <int SL>
__global__ __launch_bounds__(256) void wgrad16_fold_kernel(fixsum_t* __restrict__ gacc, int64_t weights, int groups, int64_t rstride) {
    if (rstride) gacc = rep_at(gacc, (int64_t)blockIdx.z * rstride);
    const float* part = reinterpret_cast<const float*>(gacc + weights);
    constexpr int QB = 256 / SL;   // quads of words per workgroup and turn
    __shared__ long long red[SL > 1 ? SL - 1 : 1][QB][4];
    __shared__ int red_bad[SL > 1 ? SL - 1 : 1][QB];
    const int ql = threadIdx.x % QB, sl = threadIdx.x / QB;
    const int64_t quads = weights >> 2;
    for (int64_t q0 = (int64_t)blockIdx.x * QB; q0 < quads; q0 += (int64_t)gridDim.x * QB) {
        const int64_t q = q0 + ql;
        const bool on = q < quads;
        long long sum[4] = {0ll, 0ll, 0ll, 0ll};
        bool bad[4] = {false, false, false, false};
        for (int g0 = sl; g0 < groups; g0 += 8 * SL) {
            f32x4 p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                p[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (on && g0 + SL * u < groups) p[u] = *reinterpret_cast<const f32x4*>(part + (int64_t)(g0 + SL * u) * weights + 4 * q);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) fixsum_collect(sum[i], bad[i], (double)p[u][i] * FIX_WGRAD_SCALE, FIX_PARTIAL_LIMIT);
        }
        if (SL > 1) {
            if (sl > 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) red[sl - 1][ql][i] = sum[i];
                red_bad[sl - 1][ql] = (bad[0] ? 1 : 0) | (bad[1] ? 2 : 0) | (bad[2] ? 4 : 0) | (bad[3] ? 8 : 0);
            }
            __syncthreads();
        }
        if (sl == 0 && on) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                long long t = sum[i];
                bool b = bad[i];
                if (SL > 1) {
#pragma unroll
                    for (int w = 0; w < SL - 1; ++w) {
                        t += red[w][ql][i];
                        b = b || ((red_bad[w][ql] >> i) & 1);
                    }
                }
                const long long old = (long long)gacc[4 * q + i];
                gacc[4 * q + i] = (b || old >= FIX_POISON_MIN) ? (fixsum_t)FIX_POISON : (fixsum_t)(old + t);
            }
        }
        if (SL > 1) __syncthreads();
    }
}

// Layers of the narrow network: one 16 x 16 channel block per workgroup.
// ... and layers with 16 input channels, whatever their width (the first block of the wide network)
static bool pair_layer(const ConvShape& cs) { return (cs.c_in <= 64 && cs.c_out <= 64) || cs.c_in == 16; }

// 3x3 layers of more than 64 channels on 8 x 8, 16 x 16 or 32 x 32 maps run on wgrad16_tile_kernel
static bool tile_layer(const ConvShape& cs) { return !pair_layer(cs) && cs.taps == 9 && (cs.h_in == 8 || cs.h_in == 16 || cs.h_in == 32); }

bool wgrad16_covers(int act, const ConvShape& cs) {
    if (act != ACT_BF16 || cs.stride != 1 || cs.c_in_real != cs.c_in || cs.h_in < 4 || cs.h_in > 64) return false;
    if (pair_layer(cs)) return cs.c_in % 16 == 0 && cs.c_out % 16 == 0;
    return cs.c_in % 64 == 0 && cs.c_out % 64 == 0;
}

static ConvGeom wgrad16_geom(const ConvShape& cs) {
    const int tile_px = pair_layer(cs) ? W16P_TILE_PX : W16_TILE_PX;
    return make_geom(cs.B, cs.h_in, cs.h_in, cs.c_out, 1, 0, cs.c_in, tile_px / cs.h_in, cs.taps == 9 ? 1 : 0);
}

// Pixel groups: about 256 workgroups in total (each dumps all its sums once, so fewer groups mean fewer atomics).  The
// tiled kernel takes 128: one of its workgroups fills a compute unit's registers and most of its LDS for its whole life,
// and the launches run beside the convolutions of the main stream, which then find half of the compute units free
// (measured on the WRN-16-8 pass: 22.0 / 20.3 / 20.65 / 21.2 ms with 64 / 128 / 192 / 256 workgroups).
int wgrad16_groups(const ConvShape& cs) {
    const int pairs = pair_layer(cs) ? (cs.c_in / 16) * (cs.c_out / 16) : (cs.c_in / 64) * (cs.c_out / 64);
    const int n_tiles = wgrad16_geom(cs).n_tiles;
    int groups = (tile_layer(cs) ? 128 : 256) / pairs;
    if (groups < 1) groups = 1;
    return groups < n_tiles ? groups : n_tiles;
}

template <typename K>
static void launch_w16(K kern, dim3 grid, size_t lds, hipStream_t s, const KernelTiming* kt, const ConvShape& cs, const void* x, const void* dy,
                       fixsum_t* gacc, const ConvGeom& g, const W16Geom& wg, int tiles_per_group, int replicas, Reps reps) {
    if (lds > 65536) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    // timing events ride on the dispatch itself
    hipExtLaunchKernelGGL(kern, grid, dim3(256), lds, s, kt ? kt->start : nullptr, kt ? kt->stop : nullptr, 0, (const bf16_t*)x, (const bf16_t*)dy, gacc,
                          g, wg, tiles_per_group, cs.c_in, cs.c_out, replicas, reps.stride);
}


template <int WLOG>
static void launch_w16t(dim3 grid, hipStream_t s, const KernelTiming* kt, const ConvShape& cs, const void* x, const void* dy, fixsum_t* gacc, int n_tiles,
                        int tiles_per_group, Reps reps) {
    constexpr int lds = 2 * WtGeom<WLOG>::TEAM_BYTES;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad16_tile_kernel<WLOG>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    hipExtLaunchKernelGGL(wgrad16_tile_kernel<WLOG>, grid, dim3(512), lds, s, kt ? kt->start : nullptr, nullptr, 0, (const bf16_t*)x, (const bf16_t*)dy, gacc,
                          cs.B, cs.c_in, cs.c_out, n_tiles, tiles_per_group, reps.stride);
    const int64_t weights = (int64_t)cs.c_out * 9 * cs.c_in;
    const int groups = (int)grid.x;
    const int qb = groups >= 16 ? 64 : 256;   // many groups: four waves share a word's groups
    int64_t blocks = (weights / 4 + qb - 1) / qb;
    if (blocks > 4096) blocks = 4096;
    auto fold = groups >= 16 ? wgrad16_fold_kernel<4> : wgrad16_fold_kernel<1>;
    hipExtLaunchKernelGGL(fold, dim3((unsigned)blocks, 1, reps.n), dim3(256), 0, s, nullptr, kt ? kt->stop : nullptr, 0, gacc, weights, groups, reps.stride);
}

// Layers whose pixel groups leave float partial sums behind one accumulator replica: the number of accumulator words that
// space takes (0 for the layers that add with atomics into their replicas).
int64_t wgrad16_partial_words(const ConvShape& cs) {
    if (!tile_layer(cs)) return 0;
    return ((int64_t)wgrad16_groups(cs) * cs.c_out * 9 * cs.c_in + 1) / 2;
}

void launch_wgrad16(hipStream_t s, const ConvShape& cs, const void* x, const void* dy, fixsum_t* gacc, int replicas, const KernelTiming* kt,
                    Reps reps) {
    ConvGeom g = wgrad16_geom(cs);
    const bool pair = pair_layer(cs);
    const int tile_px = g.rows_tile * cs.h_in;
    W16Geom wg;
    wg.lwp = cs.taps == 9 ? cs.h_in + 4 : cs.h_in;
    int plane = g.imgs * g.in_rows * wg.lwp;
    plane = (plane + 3) & ~3;
    if (((plane >> 2) & 1) == 0) plane += 4;
    wg.xp = plane;
    wg.dp = tile_px + 4;
    const int groups = wgrad16_groups(cs);
    const int tiles_per_group = (g.n_tiles + groups - 1) / groups;
    if (pair) {
        size_t lds = (size_t)16 * (wg.xp + wg.dp) * sizeof(bf16_t);
        const size_t fold = (size_t)4 * 16 * cs.taps * 16 * sizeof(float);   // the four waves' partial blocks
        if (lds < fold) lds = fold;
        dim3 grid(groups, (cs.c_in / 16) * (cs.c_out / 16), reps.n);
        if (cs.taps == 9) launch_w16(wgrad16_pair_kernel<9>, grid, lds, s, kt, cs, x, dy, gacc, g, wg, tiles_per_group, replicas, reps);
        else launch_w16(wgrad16_pair_kernel<1>, grid, lds, s, kt, cs, x, dy, gacc, g, wg, tiles_per_group, replicas, reps);
        return;
    }
    dim3 grid(groups, (cs.c_in / 64) * (cs.c_out / 64), reps.n);
    if (tile_layer(cs)) {
        if (cs.h_in == 32) launch_w16t<5>(grid, s, kt, cs, x, dy, gacc, g.n_tiles, tiles_per_group, reps);
        else if (cs.h_in == 16) launch_w16t<4>(grid, s, kt, cs, x, dy, gacc, g.n_tiles, tiles_per_group, reps);
        else launch_w16t<3>(grid, s, kt, cs, x, dy, gacc, g.n_tiles, tiles_per_group, reps);
        return;
    }
    const size_t lds = (size_t)64 * (wg.xp + wg.dp) * sizeof(bf16_t);
    if (cs.taps == 9) launch_w16(wgrad16_kernel<9>, grid, lds, s, kt, cs, x, dy, gacc, g, wg, tiles_per_group, replicas, reps);
    else launch_w16(wgrad16_kernel<1>, grid, lds, s, kt, cs, x, dy, gacc, g, wg, tiles_per_group, replicas, reps);
}
