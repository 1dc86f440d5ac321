// Deterministic loss-based top-k selection (Section 4.2): the k highest-loss samples in rank order.
//
// Every loss is mapped to a 64-bit sort word whose unsigned order is the selection order:
//   high 32 bits: the float's bits made monotone (sign flip), with -0 folded into +0 and every
//                 NaN folded into the largest word, so NaN ranks above +inf;
//   low 32 bits:  ~index, so that among equal losses the smaller index is the larger word.
// All words are distinct, hence exactly one result is correct and no stability argument is needed.
//
// Small pools (N <= TOPK_LDS_MAX) are sorted by one workgroup entirely in LDS with a bitonic
// network.  Larger pools take a multi-workgroup path: radix-select of the k-th word, ordered
// compaction of the selected words, and an LSD radix sort of those k words.
#include <mutex>

#include "common.h"

#define TOPK_LDS_MAX 16384
#define TOPK_THREADS 1024

__device__ __forceinline__ uint32_t loss_key(float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0xffffffffu;  // NaN: above +inf
    if (u == 0x80000000u) u = 0u;                              // -0 == +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t sort_word(float v, uint32_t idx) {
    return ((uint64_t)loss_key(v) << 32) | (uint64_t)(~idx);
}

// One workgroup; M = power of two >= N words in LDS; sorts descending.
__global__ __launch_bounds__(TOPK_THREADS) void topk_lds_bitonic_kernel(const float* __restrict__ losses, int N, int k,
                                                                        int M, int32_t* __restrict__ idx_out,
                                                                        float* __restrict__ val_out) {
    extern __shared__ uint64_t words[];
    const int tid = threadIdx.x;
    for (int i = tid; i < M; i += TOPK_THREADS) words[i] = i < N ? sort_word(losses[i], (uint32_t)i) : 0ull;
    __syncthreads();
    for (int size = 2; size <= M; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int t = tid; t < (M >> 1); t += TOPK_THREADS) {
                int lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                int hi = lo | stride;
                bool descending = (lo & size) == 0;
                uint64_t a = words[lo], b = words[hi];
                if ((a < b) == descending) {
                    words[lo] = b;
                    words[hi] = a;
                }
            }
            __syncthreads();
        }
    }
    for (int r = tid; r < k; r += TOPK_THREADS) {
        uint32_t idx = ~(uint32_t)(words[r] & 0xffffffffull);
        idx_out[r] = (int32_t)idx;
        if (val_out) val_out[r] = losses[idx];
    }
}

// ---- large pools ----------------------------------------------------------------------------------
//
// 1. 2048-bin histogram of the top 11 key bits; the bin b* that contains the k-th largest key follows.
// 2. Every element with bin >= b* (M of them, M >= k, usually M is close to k) is compacted, in index
//    order, into (sort key, index) arrays; the sort key is ~key so that ascending order is rank order.
// 3. Stable LSD radix sort of the M pairs by the 32-bit sort key, 8 bits per pass.  Stability keeps
//    equal losses in ascending index order, which is the tie rule.
// 4. The first k pairs are the result.
// Nothing is read back to the host: grids are sized for the worst case M == N and blocks past M exit.

#define SEL_BINS 2048
#define TILE 2048          // elements per 256-thread block: 8 consecutive elements per thread
#define SCAN_CHUNK 2048
// Radix passes: a block of 256 threads handles RITER * 256 elements (each wave ranks RITER * 64 of them in
// rounds of 64); 8 rounds for moderate pools, 16 for very large ones (longer runs per digit when scattering).

struct SelInfo {
    uint32_t bin;    // b*
    uint32_t M;      // elements with bin >= b*
};

__global__ __launch_bounds__(256) void zero_u32_kernel(uint32_t* p, int64_t n) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

__global__ __launch_bounds__(256) void sel_hist_kernel(const float* __restrict__ losses, int64_t N, uint32_t* __restrict__ hist) {
    __shared__ uint32_t h[SEL_BINS];
    for (int i = threadIdx.x; i < SEL_BINS; i += 256) h[i] = 0u;
    __syncthreads();
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += stride)
        atomicAdd(&h[loss_key(losses[i]) >> 21], 1u);
    __syncthreads();
    for (int i = threadIdx.x; i < SEL_BINS; i += 256)
        if (h[i]) atomicAdd(&hist[i], h[i]);
}

// One block: suffix counts over the bins; b* is the largest bin whose suffix count reaches k.
__global__ __launch_bounds__(256) void sel_threshold_kernel(const uint32_t* __restrict__ hist, uint32_t k, SelInfo* __restrict__ info) {
    __shared__ uint32_t part[256];
    uint32_t mine[8], tot = 0;
    for (int j = 0; j < 8; ++j) {
        mine[j] = hist[threadIdx.x * 8 + j];
        tot += mine[j];
    }
    part[threadIdx.x] = tot;
    __syncthreads();
    // inclusive suffix sum over threads (thread t: bins 8t .. 8t+7)
    for (int o = 1; o < 256; o <<= 1) {
        uint32_t add = (threadIdx.x + o < 256) ? part[threadIdx.x + o] : 0u;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    uint32_t above = part[threadIdx.x] - tot;  // elements in bins of higher threads
    for (int j = 7; j >= 0; --j) {
        uint32_t with = above + mine[j];
        if (above < k && with >= k) {
            info->bin = threadIdx.x * 8 + j;
            info->M = with;
        }
        above = with;
    }
}

__device__ __forceinline__ uint32_t block_exclusive_scan_256(uint32_t v, uint32_t* total) {
    // inclusive scan inside each wave by shuffles, then the four wave totals through LDS
    __shared__ uint32_t wave_total[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t below = __shfl_up(incl, o, 64);
        if (lane >= o) incl += below;
    }
    if (lane == 63) wave_total[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave; ++w) before += wave_total[w];
    const uint32_t all = (wave_total[0] + wave_total[1]) + (wave_total[2] + wave_total[3]);
    __syncthreads();   // wave_total may be written again by the next call
    if (total) *total = all;
    return before + incl - v;
}

__global__ __launch_bounds__(256) void sel_count_kernel(const float* __restrict__ losses, int64_t N, const SelInfo* __restrict__ info,
                                                        uint32_t* __restrict__ counts) {
    const uint32_t bin = info->bin;
    int64_t base = (int64_t)blockIdx.x * TILE + threadIdx.x * 8;
    uint32_t c = 0;
    for (int j = 0; j < 8; ++j)
        if (base + j < N && (loss_key(losses[base + j]) >> 21) >= bin) ++c;
    uint32_t total;
    block_exclusive_scan_256(c, &total);
    if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

// counts has been exclusive-scanned into offsets
__global__ __launch_bounds__(256) void sel_compact_kernel(const float* __restrict__ losses, int64_t N, const SelInfo* __restrict__ info,
                                                          const uint32_t* __restrict__ offsets, uint32_t* __restrict__ keys,
                                                          uint32_t* __restrict__ idx) {
    const uint32_t bin = info->bin;
    int64_t base = (int64_t)blockIdx.x * TILE + threadIdx.x * 8;
    uint32_t key[8], c = 0;
    for (int j = 0; j < 8; ++j) {
        key[j] = base + j < N ? loss_key(losses[base + j]) : 0u;
        if (base + j < N && (key[j] >> 21) >= bin) ++c;
    }
    uint32_t pos = offsets[blockIdx.x] + block_exclusive_scan_256(c, nullptr);
    for (int j = 0; j < 8; ++j)
        if (base + j < N && (key[j] >> 21) >= bin) {
            keys[pos] = ~key[j];
            idx[pos] = (uint32_t)(base + j);
            ++pos;
        }
}

// ---- exclusive scan of a uint32 array (three kernels) -------------------------------------------------

__global__ __launch_bounds__(256) void scan_chunk_sums_kernel(const uint32_t* __restrict__ data, int64_t n, uint32_t* __restrict__ sums) {
    int64_t base = (int64_t)blockIdx.x * SCAN_CHUNK + threadIdx.x * 8;
    uint32_t c = 0;
    for (int j = 0; j < 8; ++j)
        if (base + j < n) c += data[base + j];
    uint32_t total;
    block_exclusive_scan_256(c, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void scan_sums_kernel(uint32_t* __restrict__ sums, int n_chunks) {
    uint32_t carry = 0;
    for (int b0 = 0; b0 < n_chunks; b0 += 256) {
        int i = b0 + threadIdx.x;
        uint32_t v = i < n_chunks ? sums[i] : 0u, total;
        uint32_t ex = block_exclusive_scan_256(v, &total);
        if (i < n_chunks) sums[i] = carry + ex;
        carry += total;
    }
}

__global__ __launch_bounds__(256) void scan_apply_kernel(uint32_t* __restrict__ data, int64_t n, const uint32_t* __restrict__ sums) {
    int64_t base = (int64_t)blockIdx.x * SCAN_CHUNK + threadIdx.x * 8;
    uint32_t v[8], c = 0;
    for (int j = 0; j < 8; ++j) {
        v[j] = base + j < n ? data[base + j] : 0u;
        c += v[j];
    }
    uint32_t run = sums[blockIdx.x] + block_exclusive_scan_256(c, nullptr);
    for (int j = 0; j < 8; ++j)
        if (base + j < n) {
            data[base + j] = run;
            run += v[j];
        }
}

// The same in one launch for arrays of up to 8192 entries (pools of up to about 65 000 losses; above that the strided
// per-thread loads cost more than the two launches saved): thread t of the one workgroup owns entries
// [t * per, (t + 1) * per), all loaded before anything else so that the loads overlap.
#define SCAN_ONE_LAUNCH_MAX 8192
__global__ __launch_bounds__(256) void scan_small_kernel(uint32_t* __restrict__ data, int n, int per) {
    uint32_t v[32];
    const int base = threadIdx.x * per;
#pragma unroll
    for (int j = 0; j < 32; ++j) v[j] = (j < per && base + j < n) ? data[base + j] : 0u;
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) c += v[j];
    uint32_t run = block_exclusive_scan_256(c, nullptr);
#pragma unroll
    for (int j = 0; j < 32; ++j)
        if (j < per && base + j < n) {
            data[base + j] = run;
            run += v[j];
        }
}

static void exclusive_scan_u32(hipStream_t s, uint32_t* data, int64_t n, uint32_t* sums) {
    if (n <= SCAN_ONE_LAUNCH_MAX) {
        hipLaunchKernelGGL(scan_small_kernel, dim3(1), dim3(256), 0, s, data, (int)n, (int)((n + 255) / 256));
        return;
    }
    int n_chunks = (int)((n + SCAN_CHUNK - 1) / SCAN_CHUNK);
    hipLaunchKernelGGL(scan_chunk_sums_kernel, dim3(n_chunks), dim3(256), 0, s, data, n, sums);
    hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(256), 0, s, sums, n_chunks);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(n_chunks), dim3(256), 0, s, data, n, sums);
}

// ---- radix sort passes --------------------------------------------------------------------------------

// table[d * n_blocks + b] = number of elements of block b's tile with digit d (zero for tiles past M)
template <int RITER>
__global__ __launch_bounds__(256) void radix_count_kernel(const uint32_t* __restrict__ keys, const SelInfo* __restrict__ info,
                                                          int shift, uint32_t* __restrict__ table, int n_blocks) {
    __shared__ uint32_t cnt[256];
    cnt[threadIdx.x] = 0u;
    __syncthreads();
    const uint32_t M = info->M;
    constexpr int RTILE = RITER * 256;
    int64_t base = (int64_t)blockIdx.x * RTILE;
    if (base < M)
        for (int j = 0; j < RITER; ++j) {
            int64_t i = base + j * 256 + threadIdx.x;
            if (i < M) atomicAdd(&cnt[(keys[i] >> shift) & 255u], 1u);
        }
    __syncthreads();
    table[(int64_t)threadIdx.x * n_blocks + blockIdx.x] = cnt[threadIdx.x];
}

// table has been exclusive-scanned: table[d * n_blocks + b] = first output slot of digit d in block b.
// Each wave owns RTILE/4 consecutive elements of the tile and ranks them 64 at a time with ballots, so the
// order of equal digits is the input order (stable).  The ranked pairs are first put in digit order in LDS;
// the tile is then written out position by position, so that neighbouring lanes write neighbouring slots of a
// digit's run instead of 64 unrelated addresses per instruction.  Small sorts (RITER = 8, launch-bound) skip the staging
// and write from the ranking loop.
template <int RITER>
__global__ __launch_bounds__(256) void radix_scatter_kernel(const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ idx_in,
                                                            uint32_t* __restrict__ keys_out, uint32_t* __restrict__ idx_out,
                                                            const SelInfo* __restrict__ info, int shift,
                                                            const uint32_t* __restrict__ table, int n_blocks) {
    constexpr int RTILE = RITER * 256;
    constexpr bool STAGED = RITER >= 16;
    __shared__ uint32_t cnt[4][256];
    __shared__ uint32_t to_global[256];   // global slot of a digit's first element minus its slot in the tile
    __shared__ uint32_t kbuf[STAGED ? RTILE : 1], ibuf[STAGED ? RTILE : 1];
    const uint32_t M = info->M;
    const int64_t base = (int64_t)blockIdx.x * RTILE;
    if (base >= M) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int w = 0; w < 4; ++w) cnt[w][threadIdx.x] = 0u;
    __syncthreads();
    const int64_t wbase = base + wave * (RTILE / 4);
    uint32_t key[RITER], id[RITER];
#pragma unroll
    for (int it = 0; it < RITER; ++it) {
        int64_t i = wbase + it * 64 + lane;
        bool valid = i < M;
        key[it] = valid ? keys_in[i] : 0u;
        id[it] = valid ? idx_in[i] : 0u;
        if (valid) atomicAdd(&cnt[wave][(key[it] >> shift) & 255u], 1u);
    }
    __syncthreads();
    {   // per digit: slots of the tile in digit order, waves in order inside a digit
        uint32_t c[4], tile_count = 0;
        for (int w = 0; w < 4; ++w) {
            c[w] = cnt[w][threadIdx.x];
            tile_count += c[w];
        }
        uint32_t run = table[(int64_t)threadIdx.x * n_blocks + blockIdx.x];   // direct: global slots
        if (STAGED) {
            const uint32_t in_tile = block_exclusive_scan_256(tile_count, nullptr);
            to_global[threadIdx.x] = run - in_tile;
            run = in_tile;
        }
        for (int w = 0; w < 4; ++w) {
            cnt[w][threadIdx.x] = run;
            run += c[w];
        }
    }
    __syncthreads();
    const uint64_t lt = lane ? (~0ull >> (64 - lane)) : 0ull;
#pragma unroll
    for (int it = 0; it < RITER; ++it) {
        int64_t i = wbase + it * 64 + lane;
        bool valid = i < M;
        uint32_t d = (key[it] >> shift) & 255u;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            uint64_t v = __ballot((d >> b) & 1u);
            peers &= ((d >> b) & 1u) ? v : ~v;
        }
        if (valid) {
            uint32_t rank = __popcll(peers & lt);
            uint32_t pos = cnt[wave][d] + rank;
            if (STAGED) {
                kbuf[pos] = key[it];
                ibuf[pos] = id[it];
            } else {
                keys_out[pos] = key[it];
                idx_out[pos] = id[it];
            }
        }
        __builtin_amdgcn_wave_barrier();
        if (valid && (peers & lt) == 0ull) cnt[wave][d] += (uint32_t)__popcll(peers);  // lowest peer advances the slot
        __builtin_amdgcn_wave_barrier();
    }
    if (!STAGED) return;
    __syncthreads();
    const int n_valid = (int)(M - base < (uint32_t)RTILE ? M - base : (uint32_t)RTILE);
    for (int j = threadIdx.x; j < n_valid; j += 256) {
        const uint32_t k = kbuf[j];
        const uint32_t pos = to_global[(k >> shift) & 255u] + (uint32_t)j;
        keys_out[pos] = k;
        idx_out[pos] = ibuf[j];
    }
}

// Inverse of loss_key for every key that determines the float uniquely; NaN keys and the zero key
// (shared by +0 and -0) do not, those values are fetched from the loss array.
__device__ __forceinline__ bool key_to_loss(uint32_t key, float* v) {
    if (key == 0xffffffffu || key == 0x80000000u) return false;
    uint32_t u = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
    *v = __uint_as_float(u);
    return true;
}

__global__ __launch_bounds__(256) void topk_emit_kernel(const uint32_t* __restrict__ keys_sorted, const uint32_t* __restrict__ idx_sorted,
                                                        const float* __restrict__ losses, int64_t k, int32_t* __restrict__ idx_out,
                                                        float* __restrict__ val_out) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < k; r += stride) {
        uint32_t i = idx_sorted[r];
        idx_out[r] = (int32_t)i;
        if (val_out) {
            float v;
            if (!key_to_loss(~keys_sorted[r], &v)) v = losses[i];
            val_out[r] = v;
        }
    }
}

struct TopkScratch {
    uint32_t *hist, *counts, *sums, *table, *keys_a, *idx_a, *keys_b, *idx_b;
    SelInfo* info;
    int n_blocks;    // selection tiles (TILE elements)
    int r_iter;      // rounds per wave in the radix passes (8 or 16)
    int r_blocks;    // radix tiles (r_iter * 256 elements)
};

static TopkScratch carve_topk(Carver& c, int64_t N) {
    TopkScratch t;
    t.n_blocks = (int)((N + TILE - 1) / TILE);
    t.r_iter = N >= (int64_t(1) << 22) ? 16 : 8;
    t.r_blocks = (int)((N + t.r_iter * 256 - 1) / (t.r_iter * 256));
    t.hist = c.take<uint32_t>(SEL_BINS);
    t.info = c.take<SelInfo>(1);
    t.counts = c.take<uint32_t>(t.n_blocks);
    t.table = c.take<uint32_t>((size_t)256 * t.r_blocks);
    t.sums = c.take<uint32_t>(((size_t)256 * t.n_blocks + SCAN_CHUNK - 1) / SCAN_CHUNK + 1);
    t.keys_a = c.take<uint32_t>(N);
    t.idx_a = c.take<uint32_t>(N);
    t.keys_b = c.take<uint32_t>(N);
    t.idx_b = c.take<uint32_t>(N);
    return t;
}

size_t topk_scratch_bytes(int64_t N, int64_t k) {
    (void)k;
    if (N <= TOPK_LDS_MAX) return 0;
    Carver c(nullptr);
    carve_topk(c, N);
    return c.off;
}

// `scratch_base`: topk_scratch_bytes(N, k) bytes of device memory, 256-byte aligned; nothing in it needs to be cleared.
static int launch_topk_large(bls_ctx* ctx, char* scratch_base, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out) {
    Carver c(scratch_base);
    TopkScratch t = carve_topk(c, N);
    hipStream_t s = ctx->stream;
    const int nb = t.n_blocks, rb = t.r_blocks;
    int hist_blocks = nb < ctx->num_cus * 8 ? nb : ctx->num_cus * 8;
    hipLaunchKernelGGL(zero_u32_kernel, dim3(8), dim3(256), 0, s, t.hist, (int64_t)SEL_BINS);
    hipLaunchKernelGGL(sel_hist_kernel, dim3(hist_blocks), dim3(256), 0, s, losses, N, t.hist);
    hipLaunchKernelGGL(sel_threshold_kernel, dim3(1), dim3(256), 0, s, t.hist, (uint32_t)k, t.info);
    hipLaunchKernelGGL(sel_count_kernel, dim3(nb), dim3(256), 0, s, losses, N, t.info, t.counts);
    exclusive_scan_u32(s, t.counts, nb, t.sums);
    hipLaunchKernelGGL(sel_compact_kernel, dim3(nb), dim3(256), 0, s, losses, N, t.info, t.counts, t.keys_a, t.idx_a);
    uint32_t *ka = t.keys_a, *ia = t.idx_a, *kb = t.keys_b, *ib = t.idx_b;
    for (int pass = 0; pass < 4; ++pass) {
        if (t.r_iter == 16) hipLaunchKernelGGL(radix_count_kernel<16>, dim3(rb), dim3(256), 0, s, ka, t.info, pass * 8, t.table, rb);
        else hipLaunchKernelGGL(radix_count_kernel<8>, dim3(rb), dim3(256), 0, s, ka, t.info, pass * 8, t.table, rb);
        exclusive_scan_u32(s, t.table, (int64_t)256 * rb, t.sums);
        if (t.r_iter == 16)
            hipLaunchKernelGGL(radix_scatter_kernel<16>, dim3(rb), dim3(256), 0, s, ka, ia, kb, ib, t.info, pass * 8, t.table, rb);
        else
            hipLaunchKernelGGL(radix_scatter_kernel<8>, dim3(rb), dim3(256), 0, s, ka, ia, kb, ib, t.info, pass * 8, t.table, rb);
        uint32_t* tmp = ka; ka = kb; kb = tmp;
        tmp = ia; ia = ib; ib = tmp;
    }
    int64_t eb = (k + 255) / 256;
    if (eb > 2048) eb = 2048;
    hipLaunchKernelGGL(topk_emit_kernel, dim3((unsigned)eb), dim3(256), 0, s, ka, ia, losses, k, idx_out, val_out);
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

static int launch_topk_small(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out) {
    int M = 2;
    while (M < N) M <<= 1;
    size_t lds = (size_t)M * sizeof(uint64_t);
    if (lds > ctx->max_lds) return bls_fail(ctx, BLS_EUNSUPPORTED, "top-k needs %zu bytes of LDS, device allows %zu", lds, ctx->max_lds);
    if (lds > 65536)
        BLS_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(topk_lds_bitonic_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(topk_lds_bitonic_kernel, dim3(1), dim3(TOPK_THREADS), lds, ctx->stream, losses, (int)N, (int)k, M, idx_out,
                       val_out);
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

int launch_topk(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out) {
    if (N <= TOPK_LDS_MAX) return launch_topk_small(ctx, losses, N, k, idx_out, val_out);
    int rc = bls_arena_reserve(ctx, topk_scratch_bytes(N, k));
    if (rc != BLS_OK) return rc;
    return launch_topk_large(ctx, ctx->arena, losses, N, k, idx_out, val_out);
}

// ---- selection without any allocation -----------------------------------------------------------------
//
// The large-pool path above needs device scratch (histogram, block counts, digit tables and two pairs of key / index
// arrays).  For callers that must not allocate, the same launches run on a fixed array in the library's device image.
// Every GPU the library is loaded on holds its own copy of the array at its own address, for the life of the process.

#define TOPK_STATIC_BYTES (size_t(18) << 20)   // >= topk_scratch_bytes(BLS_TOPK_STATIC_MAX_N, .), checked on every call
#define TOPK_STATIC_MAX_DEVICES 64

static __device__ __align__(256) unsigned char scratch[TOPK_STATIC_BYTES];

// Device address of `scratch` per GPU (the array's name in host code is only a handle for the symbol lookup).
static char* g_static_scratch[TOPK_STATIC_MAX_DEVICES];
static std::mutex g_static_scratch_lock;

int topk_static_init(bls_ctx* ctx) {
    if (ctx->device < 0 || ctx->device >= TOPK_STATIC_MAX_DEVICES) return BLS_OK;   // topk_by_loss_static refuses such a device
    std::lock_guard<std::mutex> hold(g_static_scratch_lock);
    if (g_static_scratch[ctx->device]) return BLS_OK;
    void* ptr = nullptr;
    BLS_HIP(ctx, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));   // the context's device is current
    if (!ptr) return bls_fail(ctx, BLS_EHIP, "no device address for the static top-k scratch");
    g_static_scratch[ctx->device] = static_cast<char*>(ptr);
    return BLS_OK;
}

int launch_topk_static(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out) {
    if (N > BLS_TOPK_STATIC_MAX_N || topk_scratch_bytes(N, k) > TOPK_STATIC_BYTES)
        return bls_fail(ctx, BLS_EINVAL, "topk_by_loss_static: N = %lld exceeds the limit of %d", (long long)N, BLS_TOPK_STATIC_MAX_N);
    if (N <= TOPK_LDS_MAX) return launch_topk_small(ctx, losses, N, k, idx_out, val_out);
    char* base = (ctx->device >= 0 && ctx->device < TOPK_STATIC_MAX_DEVICES) ? g_static_scratch[ctx->device] : nullptr;
    if (!base) return bls_fail(ctx, BLS_EUNSUPPORTED, "topk_by_loss_static: no static scratch on device %d", ctx->device);
    return launch_topk_large(ctx, base, losses, N, k, idx_out, val_out);
}
