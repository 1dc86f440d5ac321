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
// 1. Two-level radix select of the k-th largest key: a 2048-bin histogram of the top 11 key bits gives the bin b1 that
//    holds it, a second histogram of the next 11 bits over the members of b1 gives the 22-bit prefix `thr`: the M
//    elements with key >> 10 >= thr are selected (M >= k; the excess is at most the members of one 22-bit prefix).
//    Histograms are aggregated per wave before they touch LDS (losses crowd into a few exponent bins).
// 2. The selected elements are compacted, in index order, into (sort key, index) arrays; the sort key is hi - key
//    (hi bounds every key), so that ascending order is rank order and the keys only span the range that occurs.
// 3. Stable LSD radix sort of the M pairs, 8 bits per pass, with as many passes as that range needs (the later passes
//    exit at once).  Stability keeps equal losses in ascending index order, which is the tie rule.
// 4. The first k pairs are the result.
// Nothing is read back to the host: grids are sized for the worst case M == N and blocks past M exit.

#define SEL_BINS 2048
#define TILE 2048          // elements per 256-thread block: 8 consecutive elements per thread
#define SCAN_CHUNK 2048
// Radix passes: a block of 256 threads handles RITER * 256 elements (each wave ranks RITER * 64 of them in
// rounds of 64); 8 rounds for moderate pools, 16 for very large ones (longer runs per digit when scattering).

struct SelInfo {
    uint32_t bin;        // b1
    uint32_t above;      // elements in bins above b1
    uint32_t thr;        // selected: key >> 10 >= thr
    uint32_t M;          // number of selected elements
    uint32_t hi;         // no key is larger; sort key = hi - key
    uint32_t n_passes;   // 8-bit passes that cover hi - (thr << 10)
};

__global__ __launch_bounds__(256) void zero_u32_kernel(uint32_t* p, int64_t n) {
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}

// Elements 4 q .. 4 q + 3 (zero key, invalid, past N); VEC: the array allows 16-byte loads.
template <bool VEC>
__device__ __forceinline__ void load_keys4(const float* __restrict__ losses, int64_t N, int64_t q, uint32_t (&key)[4], bool (&ok)[4]) {
    const int64_t i0 = q * 4;
    if (VEC && i0 + 3 < N) {
        const float4 v = *reinterpret_cast<const float4*>(losses + i0);
        key[0] = loss_key(v.x); key[1] = loss_key(v.y); key[2] = loss_key(v.z); key[3] = loss_key(v.w);
        ok[0] = ok[1] = ok[2] = ok[3] = true;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            ok[j] = i0 + j < N;
            key[j] = ok[j] ? loss_key(losses[i0 + j]) : 0u;
        }
    }
}

// LEVEL 1: bins of key >> 21 over all elements.  Losses crowd into a handful of exponent bins, so every bin has
// SUB counters in LDS and a lane adds to counter lane % SUB: the lanes of a wave that meet in one bin spread over SUB
// addresses.  LEVEL 2: bins of (key >> 10) & 2047 over the members of info->bin only (those bits are spread evenly).
template <int LEVEL, bool VEC>
__global__ __launch_bounds__(256) void sel_hist_kernel(const float* __restrict__ losses, int64_t N, const SelInfo* __restrict__ info,
                                                       uint32_t* __restrict__ hist) {
    constexpr int SUB = LEVEL == 1 ? 8 : 1;
    __shared__ uint32_t h[SEL_BINS * SUB];
    for (int i = threadIdx.x; i < SEL_BINS * SUB; i += 256) h[i] = 0u;
    __syncthreads();
    const uint32_t b1 = LEVEL == 2 ? info->bin : 0u;
    const uint32_t sub = threadIdx.x & (SUB - 1);
    const int64_t quads = (N + 3) >> 2, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += 2 * stride) {
        uint32_t key[2][4];
        bool ok[2][4] = {{false, false, false, false}, {false, false, false, false}};
        load_keys4<VEC>(losses, N, q, key[0], ok[0]);
        if (q + stride < quads) load_keys4<VEC>(losses, N, q + stride, key[1], ok[1]);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (LEVEL == 1) {
                    if (ok[u][j]) atomicAdd(&h[(key[u][j] >> 21) * SUB + sub], 1u);
                } else {
                    if (ok[u][j] && (key[u][j] >> 21) == b1) atomicAdd(&h[(key[u][j] >> 10) & (SEL_BINS - 1)], 1u);
                }
            }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < SEL_BINS; i += 256) {
        uint32_t c = 0;
#pragma unroll
        for (int u = 0; u < SUB; ++u) c += h[i * SUB + u];
        if (c) atomicAdd(&hist[i], c);
    }
}

// One block: suffix counts over the bins; the bin sought is the largest one whose suffix count reaches `want`.
// LEVEL 1: want = k; stores bin, above and hi.  LEVEL 2: want = k - above over the sub-bins of b1; stores thr, M, n_passes.
template <int LEVEL>
__global__ __launch_bounds__(256) void sel_threshold_kernel(const uint32_t* __restrict__ hist, uint32_t k, SelInfo* __restrict__ info) {
    __shared__ uint32_t part[256];
    __shared__ uint32_t top_bin;
    const uint32_t want = LEVEL == 1 ? k : k - info->above;
    uint32_t mine[8], tot = 0;
    if (threadIdx.x == 0) top_bin = 0u;
    for (int j = 0; j < 8; ++j) {
        mine[j] = hist[threadIdx.x * 8 + j];
        tot += mine[j];
    }
    part[threadIdx.x] = tot;
    __syncthreads();
    if (LEVEL == 1)
        for (int j = 0; j < 8; ++j)
            if (mine[j]) atomicMax(&top_bin, threadIdx.x * 8 + j);
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
        if (above < want && with >= want) {
            const uint32_t b = threadIdx.x * 8 + j;
            if (LEVEL == 1) {
                info->bin = b;
                info->above = above;
                info->hi = top_bin == SEL_BINS - 1 ? 0xffffffffu : ((top_bin + 1u) << 21) - 1u;
            } else {
                const uint32_t thr = (info->bin << 11) | b;
                const uint32_t range = info->hi - (thr << 10);   // sort keys lie in [0, range]
                info->thr = thr;
                info->M = info->above + with;
                info->n_passes = range == 0u ? 0u : (32u - (uint32_t)__clz(range) + 7u) / 8u;
            }
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

// The 8 consecutive elements of a thread (two quads)
template <bool VEC>
__device__ __forceinline__ uint32_t load_tile_keys(const float* __restrict__ losses, int64_t N, uint32_t thr, uint32_t (&key)[8], bool (&sel)[8]) {
    const int64_t q0 = ((int64_t)blockIdx.x * TILE + threadIdx.x * 8) >> 2;
    uint32_t c = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t kq[4];
        bool ok[4];
        load_keys4<VEC>(losses, N, q0 + h, kq, ok);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            key[4 * h + j] = kq[j];
            sel[4 * h + j] = ok[j] && (kq[j] >> 10) >= thr;
            c += sel[4 * h + j] ? 1u : 0u;
        }
    }
    return c;
}

template <bool VEC>
__global__ __launch_bounds__(256) void sel_count_kernel(const float* __restrict__ losses, int64_t N, const SelInfo* __restrict__ info,
                                                        uint32_t* __restrict__ counts) {
    uint32_t key[8];
    bool sel[8];
    const uint32_t c = load_tile_keys<VEC>(losses, N, info->thr, key, sel);
    uint32_t total;
    block_exclusive_scan_256(c, &total);
    if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

// counts has been exclusive-scanned into offsets
template <bool VEC>
__global__ __launch_bounds__(256) void sel_compact_kernel(const float* __restrict__ losses, int64_t N, const SelInfo* __restrict__ info,
                                                          const uint32_t* __restrict__ offsets, uint32_t* __restrict__ keys,
                                                          uint32_t* __restrict__ idx) {
    const uint32_t hi = info->hi;
    const int64_t base = (int64_t)blockIdx.x * TILE + threadIdx.x * 8;
    uint32_t key[8];
    bool sel[8];
    const uint32_t c = load_tile_keys<VEC>(losses, N, info->thr, key, sel);
    uint32_t pos = offsets[blockIdx.x] + block_exclusive_scan_256(c, nullptr);
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (sel[j]) {
            keys[pos] = hi - key[j];
            idx[pos] = (uint32_t)(base + j);
            ++pos;
        }
}

// ---- exclusive scan of a uint32 array (three kernels) -------------------------------------------------

// The scans take an optional (info, pass): a radix pass the key range does not need is skipped by all its kernels.
__device__ __forceinline__ bool pass_skipped(const SelInfo* info, int pass) { return info && (uint32_t)pass >= info->n_passes; }
// Radix tiles that hold selected pairs (the grids and tables are sized for M == N on the host) and the length of a
// pass's digit table, 256 entries per such tile; with rtile == 0 the scan takes the length it was given.
__device__ __forceinline__ int active_tiles(const SelInfo* info, int rtile, int n_blocks) {
    const int64_t a = ((int64_t)info->M + rtile - 1) / rtile;
    return a < n_blocks ? (int)a : n_blocks;
}
__device__ __forceinline__ int64_t scan_length(int64_t n, const SelInfo* info, int rtile) {
    if (!info || rtile == 0) return n;
    const int64_t m = 256 * (((int64_t)info->M + rtile - 1) / rtile);
    return m < n ? m : n;
}

__global__ __launch_bounds__(256) void scan_chunk_sums_kernel(const uint32_t* __restrict__ data, int64_t n, uint32_t* __restrict__ sums,
                                                              const SelInfo* __restrict__ info, int pass, int rtile) {
    if (pass_skipped(info, pass)) return;
    n = scan_length(n, info, rtile);
    if ((int64_t)blockIdx.x * SCAN_CHUNK >= n) return;
    int64_t base = (int64_t)blockIdx.x * SCAN_CHUNK + threadIdx.x * 8;
    uint32_t c = 0;
    for (int j = 0; j < 8; ++j)
        if (base + j < n) c += data[base + j];
    uint32_t total;
    block_exclusive_scan_256(c, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void scan_sums_kernel(uint32_t* __restrict__ sums, int n_chunks, int64_t n, const SelInfo* __restrict__ info, int pass,
                                                        int rtile) {
    if (pass_skipped(info, pass)) return;
    n_chunks = (int)((scan_length(n, info, rtile) + SCAN_CHUNK - 1) / SCAN_CHUNK);
    uint32_t carry = 0;
    for (int b0 = 0; b0 < n_chunks; b0 += 256) {
        int i = b0 + threadIdx.x;
        uint32_t v = i < n_chunks ? sums[i] : 0u, total;
        uint32_t ex = block_exclusive_scan_256(v, &total);
        if (i < n_chunks) sums[i] = carry + ex;
        carry += total;
    }
}

__global__ __launch_bounds__(256) void scan_apply_kernel(uint32_t* __restrict__ data, int64_t n, const uint32_t* __restrict__ sums,
                                                         const SelInfo* __restrict__ info, int pass, int rtile) {
    if (pass_skipped(info, pass)) return;
    n = scan_length(n, info, rtile);
    if ((int64_t)blockIdx.x * SCAN_CHUNK >= n) return;
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
__global__ __launch_bounds__(256) void scan_small_kernel(uint32_t* __restrict__ data, int n, int per, const SelInfo* __restrict__ info, int pass,
                                                         int rtile) {
    if (pass_skipped(info, pass)) return;
    n = (int)scan_length(n, info, rtile);
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

static void exclusive_scan_u32(hipStream_t s, uint32_t* data, int64_t n, uint32_t* sums, const SelInfo* info = nullptr, int pass = 0, int rtile = 0) {
    if (n <= SCAN_ONE_LAUNCH_MAX) {
        hipLaunchKernelGGL(scan_small_kernel, dim3(1), dim3(256), 0, s, data, (int)n, (int)((n + 255) / 256), info, pass, rtile);
        return;
    }
    int n_chunks = (int)((n + SCAN_CHUNK - 1) / SCAN_CHUNK);
    hipLaunchKernelGGL(scan_chunk_sums_kernel, dim3(n_chunks), dim3(256), 0, s, data, n, sums, info, pass, rtile);
    hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(256), 0, s, sums, n_chunks, n, info, pass, rtile);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(n_chunks), dim3(256), 0, s, data, n, sums, info, pass, rtile);
}

// ---- radix sort passes --------------------------------------------------------------------------------

// table[d * tiles + b] = number of elements of block b's tile with digit d, tiles = the tiles that hold pairs (active_tiles)
template <int RITER>
__global__ __launch_bounds__(256) void radix_count_kernel(const uint32_t* __restrict__ keys, const SelInfo* __restrict__ info,
                                                          int shift, uint32_t* __restrict__ table, int n_blocks) {
    if ((uint32_t)(shift >> 3) >= info->n_passes) return;   // the key range does not reach these bits
    __shared__ uint32_t cnt[256];
    cnt[threadIdx.x] = 0u;
    __syncthreads();
    const uint32_t M = info->M;
    constexpr int RTILE = RITER * 256;
    int64_t base = (int64_t)blockIdx.x * RTILE;
    if (base >= M) return;   // the table only has columns for tiles that hold pairs
    for (int j = 0; j < RITER; ++j) {
        int64_t i = base + j * 256 + threadIdx.x;
        if (i < M) atomicAdd(&cnt[(keys[i] >> shift) & 255u], 1u);
    }
    __syncthreads();
    table[(int64_t)threadIdx.x * active_tiles(info, RTILE, n_blocks) + blockIdx.x] = cnt[threadIdx.x];
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
    if ((uint32_t)(shift >> 3) >= info->n_passes) return;   // the key range does not reach these bits
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
        uint32_t run = table[(int64_t)threadIdx.x * active_tiles(info, RTILE, n_blocks) + blockIdx.x];   // direct: global slots
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

// The sorted pairs sit in the first or the second pair of arrays, depending on the number of passes that ran.
__global__ __launch_bounds__(256) void topk_emit_kernel(const uint32_t* __restrict__ keys_a, const uint32_t* __restrict__ idx_a,
                                                        const uint32_t* __restrict__ keys_b, const uint32_t* __restrict__ idx_b,
                                                        const SelInfo* __restrict__ info, const float* __restrict__ losses, int64_t k,
                                                        int32_t* __restrict__ idx_out, float* __restrict__ val_out) {
    const bool second = (info->n_passes & 1u) != 0u;
    const uint32_t* keys_sorted = second ? keys_b : keys_a;
    const uint32_t* idx_sorted = second ? idx_b : idx_a;
    const uint32_t hi = info->hi;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < k; r += stride) {
        uint32_t i = idx_sorted[r];
        idx_out[r] = (int32_t)i;
        if (val_out) {
            float v;
            if (!key_to_loss(hi - keys_sorted[r], &v)) v = losses[i];
            val_out[r] = v;
        }
    }
}

struct TopkScratch {
    uint32_t *hist, *hist2, *counts, *sums, *table, *keys_a, *idx_a, *keys_b, *idx_b;
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
    t.hist = c.take<uint32_t>(2 * SEL_BINS);   // both levels, cleared together
    t.hist2 = t.hist + SEL_BINS;
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
    const int64_t quads = (N + 3) / 4;
    // Histogram workgroups per compute unit: each one clears and folds its LDS bins and adds every non-empty bin to the global
    // histogram (all 2048 of them on the second level), which outweighs the shorter rounds of a finer grid below 2^25 keys
    // (measured, N = 2^20 / 2^24 / 2^26: 118 / 282 / 869 us with two per unit, 133 / 313 / 863 us with eight).
    const int per_cu = N >= (int64_t(1) << 25) ? 8 : 2;
    int hist_blocks = (int)((quads + 255) / 256 < ctx->num_cus * per_cu ? (quads + 255) / 256 : ctx->num_cus * per_cu);
    const bool vec = reinterpret_cast<uintptr_t>(losses) % 16 == 0;   // 16-byte loads where the array allows them
    hipLaunchKernelGGL(zero_u32_kernel, dim3(16), dim3(256), 0, s, t.hist, (int64_t)2 * SEL_BINS);
    if (vec) hipLaunchKernelGGL((sel_hist_kernel<1, true>), dim3(hist_blocks), dim3(256), 0, s, losses, N, t.info, t.hist);
    else hipLaunchKernelGGL((sel_hist_kernel<1, false>), dim3(hist_blocks), dim3(256), 0, s, losses, N, t.info, t.hist);
    hipLaunchKernelGGL(sel_threshold_kernel<1>, dim3(1), dim3(256), 0, s, t.hist, (uint32_t)k, t.info);
    if (vec) hipLaunchKernelGGL((sel_hist_kernel<2, true>), dim3(hist_blocks), dim3(256), 0, s, losses, N, t.info, t.hist2);
    else hipLaunchKernelGGL((sel_hist_kernel<2, false>), dim3(hist_blocks), dim3(256), 0, s, losses, N, t.info, t.hist2);
    hipLaunchKernelGGL(sel_threshold_kernel<2>, dim3(1), dim3(256), 0, s, t.hist2, (uint32_t)k, t.info);
    if (vec) hipLaunchKernelGGL(sel_count_kernel<true>, dim3(nb), dim3(256), 0, s, losses, N, t.info, t.counts);
    else hipLaunchKernelGGL(sel_count_kernel<false>, dim3(nb), dim3(256), 0, s, losses, N, t.info, t.counts);
    exclusive_scan_u32(s, t.counts, nb, t.sums);
    if (vec) hipLaunchKernelGGL(sel_compact_kernel<true>, dim3(nb), dim3(256), 0, s, losses, N, t.info, t.counts, t.keys_a, t.idx_a);
    else hipLaunchKernelGGL(sel_compact_kernel<false>, dim3(nb), dim3(256), 0, s, losses, N, t.info, t.counts, t.keys_a, t.idx_a);
    uint32_t *ka = t.keys_a, *ia = t.idx_a, *kb = t.keys_b, *ib = t.idx_b;
    for (int pass = 0; pass < 4; ++pass) {
        if (t.r_iter == 16) hipLaunchKernelGGL(radix_count_kernel<16>, dim3(rb), dim3(256), 0, s, ka, t.info, pass * 8, t.table, rb);
        else hipLaunchKernelGGL(radix_count_kernel<8>, dim3(rb), dim3(256), 0, s, ka, t.info, pass * 8, t.table, rb);
        exclusive_scan_u32(s, t.table, (int64_t)256 * rb, t.sums, t.info, pass, t.r_iter * 256);
        if (t.r_iter == 16)
            hipLaunchKernelGGL(radix_scatter_kernel<16>, dim3(rb), dim3(256), 0, s, ka, ia, kb, ib, t.info, pass * 8, t.table, rb);
        else
            hipLaunchKernelGGL(radix_scatter_kernel<8>, dim3(rb), dim3(256), 0, s, ka, ia, kb, ib, t.info, pass * 8, t.table, rb);
        uint32_t* tmp = ka; ka = kb; kb = tmp;
        tmp = ia; ia = ib; ib = tmp;
    }
    int64_t eb = (k + 255) / 256;
    if (eb > 2048) eb = 2048;
    hipLaunchKernelGGL(topk_emit_kernel, dim3((unsigned)eb), dim3(256), 0, s, t.keys_a, t.idx_a, t.keys_b, t.idx_b, t.info, losses, k, idx_out, val_out);
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
