// Weight gradient of wide bf16 layers on the bf16 matrix instruction.
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

// Layers of the narrow network: one 16 x 16 channel block per workgroup.
static bool pair_layer(const ConvShape& cs) { return cs.c_in <= 64 && cs.c_out <= 64; }

bool wgrad16_covers(int act, const ConvShape& cs) {
    if (act != ACT_BF16 || cs.stride != 1 || cs.c_in_real != cs.c_in || cs.h_in < 4 || cs.h_in > 64) return false;
    if (pair_layer(cs)) return cs.c_in % 16 == 0 && cs.c_out % 16 == 0;
    return cs.c_in % 64 == 0 && cs.c_out % 64 == 0;
}

static ConvGeom wgrad16_geom(const ConvShape& cs) {
    const int tile_px = pair_layer(cs) ? W16P_TILE_PX : W16_TILE_PX;
    return make_geom(cs.B, cs.h_in, cs.h_in, cs.c_out, 1, 0, cs.c_in, tile_px / cs.h_in, cs.taps == 9 ? 1 : 0);
}

// Pixel groups: about 256 workgroups in total (each dumps all its sums once, so fewer groups mean fewer atomics)
int wgrad16_groups(const ConvShape& cs) {
    const int pairs = pair_layer(cs) ? (cs.c_in / 16) * (cs.c_out / 16) : (cs.c_in / 64) * (cs.c_out / 64);
    const int n_tiles = wgrad16_geom(cs).n_tiles;
    int groups = 256 / pairs;
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
    const size_t lds = (size_t)64 * (wg.xp + wg.dp) * sizeof(bf16_t);
    dim3 grid(groups, (cs.c_in / 64) * (cs.c_out / 64), reps.n);
    if (cs.taps == 9) launch_w16(wgrad16_kernel<9>, grid, lds, s, kt, cs, x, dy, gacc, g, wg, tiles_per_group, replicas, reps);
    else launch_w16(wgrad16_kernel<1>, grid, lds, s, kt, cs, x, dy, gacc, g, wg, tiles_per_group, replicas, reps);
}
