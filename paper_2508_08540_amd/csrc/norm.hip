// Batch normalisation around the convolutions: statistics finalisation, normalise + ReLU (+ shortcut),
// and the backward pass (two reductions and one elementwise pass).  Activations are [pixels][C] with
// C a multiple of 16 (at most BN_MAX_C), so every thread works on 4 consecutive channels (16 bytes in fp32, 8 in bf16).
// All kernels are templates on the storage type of the activations; arithmetic is fp32.
#include "act.h"

#define BN_MAX_C 512

// out = relu(gamma*(y-mean)*invstd + beta + shortcut(res)).  In training the statistics come from the
// fixed-point sums: threads 0..C-1 of every workgroup turn them into mean and invstd (double), workgroup 0
// also stores them and moves the running statistics (momentum 0.1, unbiased variance).  In inference (no sums) the
// running statistics are used.
// MAXC: 64 (narrow layers: thread c handles channel c, the form the compiler schedules best: a loop there, even
// with one trip, costs microseconds per launch) or BN_MAX_C (the per-channel prologue loops over 256-channel passes).
// log2 of the number of channel quads when that is a power of two, else -1
static int quads_log2(int C) {
    const int cq = C >> 2;
    if (cq <= 0 || (cq & (cq - 1)) != 0) return -1;
    int l = 0;
    while ((1 << l) < cq) ++l;
    return l;
}

template <typename T, int MAXC>
__global__ __launch_bounds__(256) void bn_apply_kernel(const T* __restrict__ y, int64_t pixels, int C, BnStats st,
                                                       const float* __restrict__ gamma, const float* __restrict__ beta,
                                                       const T* __restrict__ res, int c_res, int res_stride, int h_out,
                                                       T* __restrict__ out, int cq_log2, int64_t rstride) {
    __builtin_amdgcn_s_setprio(2);   // ahead of the weight-gradient kernels of the side stream, which only the update waits for
    if (rstride) {   // one replica of several: every buffer sits blockIdx.z slots further
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        y = rep_at(y, ro); gamma = rep_at(gamma, ro); beta = rep_at(beta, ro); res = rep_at(res, ro); out = rep_at(out, ro);
        st.sums = rep_at(st.sums, ro); st.mean = rep_at(st.mean, ro); st.invstd = rep_at(st.invstd, ro);
        st.running_mean = rep_at(st.running_mean, ro); st.running_var = rep_at(st.running_var, ro);
    }
    constexpr bool WIDE = MAXC > 64;
    __shared__ float s_mean[MAXC], s_invstd[MAXC];
    for (int c0 = 0; c0 < (WIDE ? C : 1); c0 += 256) {
        const int c = c0 + (int)threadIdx.x;
        if (c >= C) continue;
        if (st.sums) {
            const double s1 = (double)fixsum_read(st.sums, C, 0, c) * (1.0 / FIX_FWD_SCALE);
            const double s2 = (double)fixsum_read(st.sums, C, 1, c) * (1.0 / FIX_FWD_SCALE);
            double mu = s1 / st.count;
            double var = s2 / st.count - mu * mu;
            if (var < 0.0) var = 0.0;
            s_mean[c] = (float)mu;
            s_invstd[c] = (float)(1.0 / sqrt(var + BN_EPS));
            if (blockIdx.x == 0) {
                if (fixsum_poisoned(st.sums, C, c)) {   // out of range or not finite: NaN, as a float sum would end
                    s_mean[c] = s_invstd[c] = FIX_NAN;
                    mu = var = (double)FIX_NAN;
                }
                st.mean[c] = s_mean[c];
                st.invstd[c] = s_invstd[c];
                const double unbiased = st.count > 1.0 ? var * st.count / (st.count - 1.0) : var;
                st.running_mean[c] = (float)((1.0 - BN_MOMENTUM) * (double)st.running_mean[c] + BN_MOMENTUM * mu);
                st.running_var[c] = (float)((1.0 - BN_MOMENTUM) * (double)st.running_var[c] + BN_MOMENTUM * unbiased);
            }
        } else {
            s_mean[c] = st.running_mean[c];
            s_invstd[c] = (float)(1.0 / sqrt((double)st.running_var[c] + BN_EPS));
        }
    }
    __syncthreads();
    const int cq = C >> 2;
    int64_t total = pixels * cq;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int lo = (C - c_res) >> 1;
    if (WIDE && cq_log2 >= 0 && (stride & (cq - 1)) == 0 && (res == nullptr || res_stride == 1)) {
        // wide layers: the grid's stride is a multiple of the quads per pixel, so a thread keeps its four channels and their
        // constants for all its pixels (the loop below re-reads 48 bytes of them for every 8 or 16 bytes of payload)
        const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
        const int c = (int)(first & (cq - 1)) << 2;
        const f32x4 ga = *reinterpret_cast<const f32x4*>(gamma + c), be = *reinterpret_cast<const f32x4*>(beta + c);
        const f32x4 mu = *reinterpret_cast<const f32x4*>(&s_mean[c]), is = *reinterpret_cast<const f32x4*>(&s_invstd[c]);
        const bool with_res = res && c >= lo && c < lo + c_res;
        for (int64_t i = first; i < total; i += stride) {
            const int64_t p = i >> cq_log2;
            const f32x4 v = Act<T>::load4(y + p * C + c);
            f32x4 r = {0.f, 0.f, 0.f, 0.f};
            if (with_res) r = Act<T>::load4(res + p * c_res + (c - lo));
            f32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float t = __fmaf_rn((v[j] - mu[j]) * is[j], ga[j], be[j]) + r[j];
                o[j] = relu_keep_nan(t);
            }
            Act<T>::store4(out + p * C + c, o);
        }
        return;
    }
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int64_t p = cq_log2 >= 0 ? i >> cq_log2 : i / cq;   // (a 64-bit division costs as much as the rest of the body)
        int c = (int)(i - p * cq) << 2;
        f32x4 v = Act<T>::load4(y + p * C + c);
        f32x4 ga = *reinterpret_cast<const f32x4*>(gamma + c);
        f32x4 be = *reinterpret_cast<const f32x4*>(beta + c);
        f32x4 r = {0.f, 0.f, 0.f, 0.f};
        if (res && c >= lo && c < lo + c_res) {
            int64_t rp = p;
            if (res_stride != 1) {
                int hw = h_out * h_out;
                int64_t n = p / hw;
                int q = (int)(p - n * hw);
                int h = q / h_out, w = q - h * h_out;
                int h_in = h_out * res_stride;
                rp = (n * h_in + (int64_t)h * res_stride) * h_in + (int64_t)w * res_stride;
            }
            r = Act<T>::load4(res + rp * c_res + (c - lo));
        }
        f32x4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float t = __fmaf_rn((v[j] - s_mean[c + j]) * s_invstd[c + j], ga[j], be[j]) + r[j];
            o[j] = relu_keep_nan(t);
        }
        Act<T>::store4(out + p * C + c, o);
    }
}

void launch_bn_apply(hipStream_t s, int act, const void* y, int64_t pixels, int C, const BnStats& st, const float* gamma,
                     const float* beta, const void* res, int c_res, int res_stride, int h_out, void* out, Reps reps) {
    int64_t total = pixels * (C / 4);
    int64_t blocks = (total + 255) / 256;
    // every workgroup derives the statistics of all C channels first: wide layers take fewer, longer-lived workgroups
    const int64_t cap = C > 64 ? 1024 : 4096;
    if (blocks > cap) blocks = cap;
    const int cq_log2 = quads_log2(C);
    const dim3 grid((unsigned)blocks, 1, reps.n);
    ACT_DISPATCH(act, {
        if (C > 64)
            hipLaunchKernelGGL((bn_apply_kernel<T, BN_MAX_C>), grid, dim3(256), 0, s, (const T*)y, pixels, C, st, gamma, beta,
                               (const T*)res, c_res, res_stride, h_out, (T*)out, cq_log2, reps.stride);
        else
            hipLaunchKernelGGL((bn_apply_kernel<T, 64>), grid, dim3(256), 0, s, (const T*)y, pixels, C, st, gamma, beta,
                               (const T*)res, c_res, res_stride, h_out, (T*)out, cq_log2, reps.stride);
    });
}

__global__ __launch_bounds__(256) void bn_inference_stats_kernel(const float* __restrict__ running_mean, const float* __restrict__ running_var,
                                                                 int C, float* __restrict__ mean, float* __restrict__ invstd) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    mean[c] = running_mean[c];
    invstd[c] = (float)(1.0 / sqrt((double)running_var[c] + BN_EPS));
}

void launch_bn_inference_stats(hipStream_t s, const float* running_mean, const float* running_var, int C, float* mean, float* invstd) {
    hipLaunchKernelGGL(bn_inference_stats_kernel, dim3((C + 255) / 256), dim3(256), 0, s, running_mean, running_var, C, mean, invstd);
}

// ---- backward -------------------------------------------------------------------------------------

// Pixel chunks of the backward reduction: at most 1024 (each of the 16 replicas of a sum then takes 64 partials); 128 pixels
// per chunk, 32 for the layers that are cut into channel slices (they have few pixels).
int bn_bwd_partials(int64_t pixels, int C) {
    int64_t n = pixels / (C > 128 && C % 128 == 0 ? 32 : 128);
    if (n < 1) n = 1;
    if (n > 1024) n = 1024;
    return (int)n;
}
// Channels per workgroup of the backward reduction: layers of more than 128 channels are cut into slices of 128 (blockIdx.y),
// so that a workgroup always has eight or more pixels in flight and a layer of few pixels still fills the chip.
static int bn_bwd_slice(int C) { return (C > 128 && C % 128 == 0) ? 128 : C; }

// Upstream gradient of pixel p, channels c..c+3: either a full tensor of the storage type, or one fp32
// vector per sample shared by all `shared` positions of that sample (gradient of a global average pool).
template <typename T>
__device__ __forceinline__ f32x4 load_dout(const void* __restrict__ dout, int shared, int64_t p, int C, int c) {
    if (shared) return *reinterpret_cast<const f32x4*>(static_cast<const float*>(dout) + (p / shared) * C + c);
    return Act<T>::load4(static_cast<const T*>(dout) + p * C + c);
}

// adds (sum g, sum g*xhat), g = dout * (out > 0), into the fixed-point accumulators sums[2][C]; a workgroup takes a chunk of
// pixels and the CS channels from blockIdx.y * CS on; two pixels per thread are in flight
template <typename T, bool WIDE>
__global__ __launch_bounds__(256) void bn_bwd_reduce_kernel(const void* __restrict__ dout, int shared,
                                                            const T* __restrict__ out, const T* __restrict__ y,
                                                            int64_t pixels, int C, int CS, const float* __restrict__ mean,
                                                            const float* __restrict__ invstd, fixsum_t* __restrict__ sums, int64_t rstride) {
    if (rstride) {
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        dout = rep_at(dout, ro); out = rep_at(out, ro); y = rep_at(y, ro); mean = rep_at(mean, ro); invstd = rep_at(invstd, ro);
        sums = rep_at(sums, ro);
    }
    __shared__ float red[2][256][4];
    const int cq = CS >> 2;             // threads per pixel (CS <= BN_MAX_C: at most 128)
    const int lanes_p = 256 / cq;       // pixels in flight per block; threads beyond lanes_p * cq idle
    const int cg = threadIdx.x % cq, pl = threadIdx.x / cq;
    const int c = blockIdx.y * CS + (cg << 2);
    int64_t chunk = (pixels + gridDim.x - 1) / gridDim.x;
    int64_t p0 = (int64_t)blockIdx.x * chunk, p1 = p0 + chunk < pixels ? p0 + chunk : pixels;
    f32x4 mu = *reinterpret_cast<const f32x4*>(mean + c);
    f32x4 is = *reinterpret_cast<const f32x4*>(invstd + c);
    f32x4 sg = {0.f, 0.f, 0.f, 0.f}, sgx = {0.f, 0.f, 0.f, 0.f};
    if (pl < lanes_p) {
        int64_t p = p0 + pl;
        for (; p + lanes_p < p1; p += 2 * lanes_p) {   // pixels p and p + lanes_p, added in this order
            const int64_t q = p + lanes_p;
            f32x4 d0 = load_dout<T>(dout, shared, p, C, c), d1 = load_dout<T>(dout, shared, q, C, c);
            f32x4 o0 = Act<T>::load4(out + p * C + c), o1 = Act<T>::load4(out + q * C + c);
            f32x4 v0 = Act<T>::load4(y + p * C + c), v1 = Act<T>::load4(y + q * C + c);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float g = o0[j] > 0.f ? d0[j] : 0.f;
                sg[j] += g;
                sgx[j] = __fmaf_rn(g, (v0[j] - mu[j]) * is[j], sgx[j]);
                g = o1[j] > 0.f ? d1[j] : 0.f;
                sg[j] += g;
                sgx[j] = __fmaf_rn(g, (v1[j] - mu[j]) * is[j], sgx[j]);
            }
        }
        if (p < p1) {
            f32x4 d = load_dout<T>(dout, shared, p, C, c);
            f32x4 o = Act<T>::load4(out + p * C + c);
            f32x4 v = Act<T>::load4(y + p * C + c);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float g = o[j] > 0.f ? d[j] : 0.f;
                sg[j] += g;
                sgx[j] = __fmaf_rn(g, (v[j] - mu[j]) * is[j], sgx[j]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        red[0][threadIdx.x][j] = sg[j];
        red[1][threadIdx.x][j] = sgx[j];
    }
    __syncthreads();
    // column (which, channel) is summed over the pixel lanes in a fixed order
    for (int t0 = 0; t0 < (WIDE ? 2 * CS : 1); t0 += 256) {
        const int t = t0 + (int)threadIdx.x;
        if (t >= 2 * CS) continue;
        int which = t / CS, ch = t % CS;
        float acc = 0.f;
        for (int l = 0; l < lanes_p; ++l) acc += red[which][l * cq + (ch >> 2)][ch & 3];
        fixsum_add(sums + ((blockIdx.x % FIX_REPLICAS) * 2 + which) * C + blockIdx.y * CS + ch, (double)acc * FIX_BWD_SCALE);
    }
}

void launch_bn_bwd_reduce(hipStream_t s, int act, const void* dout, int dout_positions_shared, const void* out, const void* y,
                          int64_t pixels, int C, const float* mean, const float* invstd, fixsum_t* sums, Reps reps) {
    int n = bn_bwd_partials(pixels, C);
    const int CS = bn_bwd_slice(C);
    const dim3 grid(n, C / CS, reps.n);
    ACT_DISPATCH(act, {
        if (2 * CS > 256)
            hipLaunchKernelGGL((bn_bwd_reduce_kernel<T, true>), grid, dim3(256), 0, s, dout, dout_positions_shared, (const T*)out,
                               (const T*)y, pixels, C, CS, mean, invstd, sums, reps.stride);
        else
            hipLaunchKernelGGL((bn_bwd_reduce_kernel<T, false>), grid, dim3(256), 0, s, dout, dout_positions_shared, (const T*)out,
                               (const T*)y, pixels, C, CS, mean, invstd, sums, reps.stride);
    });
}

template <typename T, int MAXC, bool HAS_ADD>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(const void* __restrict__ dout, int shared,
                                                           const T* __restrict__ out, const T* __restrict__ y,
                                                           int64_t pixels, int C, const float* __restrict__ mean,
                                                           const float* __restrict__ invstd, const float* __restrict__ gamma,
                                                           const fixsum_t* __restrict__ sums, float* __restrict__ dgamma,
                                                           float* __restrict__ dbeta, float inv_count, T* __restrict__ dy,
                                                           T* __restrict__ g_out, const T* __restrict__ add, int cq_log2, int64_t rstride) {
    __builtin_amdgcn_s_setprio(2);   // ahead of the weight-gradient kernels of the side stream, which only the update waits for
    if (rstride) {
        const int64_t ro = (int64_t)blockIdx.z * rstride;
        dout = rep_at(dout, ro); out = rep_at(out, ro); y = rep_at(y, ro); mean = rep_at(mean, ro); invstd = rep_at(invstd, ro);
        gamma = rep_at(gamma, ro); sums = rep_at(sums, ro); dgamma = rep_at(dgamma, ro); dbeta = rep_at(dbeta, ro); dy = rep_at(dy, ro);
        g_out = rep_at(g_out, ro); add = rep_at(add, ro);
    }
    constexpr bool WIDE = MAXC > 64;
    __shared__ float s_dg[MAXC], s_db[MAXC];
    auto channel_sums = [&](int c) {
        s_db[c] = (float)((double)fixsum_read(sums, C, 0, c) * (1.0 / FIX_BWD_SCALE));
        s_dg[c] = (float)((double)fixsum_read(sums, C, 1, c) * (1.0 / FIX_BWD_SCALE));
        if (blockIdx.x == 0) {
            const bool bad = fixsum_poisoned(sums, C, c);   // out of range or not finite: NaN, as a float sum would end
            dbeta[c] = bad ? FIX_NAN : s_db[c];
            dgamma[c] = bad ? FIX_NAN : s_dg[c];
        }
    };
    if constexpr (WIDE) {
        for (int c = threadIdx.x; c < C; c += 256) channel_sums(c);
    } else {
        if ((int)threadIdx.x < C) channel_sums(threadIdx.x);
    }
    __syncthreads();
    const int cq = C >> 2;
    int64_t total = pixels * cq;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    if (WIDE && cq_log2 >= 0 && (stride & (cq - 1)) == 0) {
        // wide layers: a thread keeps its four channels and their constants for all its pixels (as in bn_apply_kernel)
        const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
        const int c = (int)(first & (cq - 1)) << 2;
        const f32x4 mu = *reinterpret_cast<const f32x4*>(mean + c), is = *reinterpret_cast<const f32x4*>(invstd + c);
        const f32x4 ga = *reinterpret_cast<const f32x4*>(gamma + c);
        const f32x4 db = *reinterpret_cast<const f32x4*>(&s_db[c]), dg = *reinterpret_cast<const f32x4*>(&s_dg[c]);
        for (int64_t i = first; i < total; i += stride) {
            const int64_t p = i >> cq_log2;
            const f32x4 d = load_dout<T>(dout, shared, p, C, c);
            const f32x4 o = Act<T>::load4(out + p * C + c);
            const f32x4 v = Act<T>::load4(y + p * C + c);
            f32x4 r, gq;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float g = o[j] > 0.f ? d[j] : 0.f;
                float xhat = (v[j] - mu[j]) * is[j];
                gq[j] = g;
                r[j] = ga[j] * is[j] * (g - db[j] * inv_count - xhat * (dg[j] * inv_count));
            }
            if (HAS_ADD) r += Act<T>::load4(add + p * C + c);  // gradient arriving through an identity shortcut
            Act<T>::store4(dy + p * C + c, r);
            if (g_out) Act<T>::store4(g_out + p * C + c, gq);
        }
        return;
    }
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int64_t p = cq_log2 >= 0 ? i >> cq_log2 : i / cq;
        int c = (int)(i - p * cq) << 2;
        f32x4 d = load_dout<T>(dout, shared, p, C, c);
        f32x4 o = Act<T>::load4(out + p * C + c);
        f32x4 v = Act<T>::load4(y + p * C + c);
        f32x4 mu = *reinterpret_cast<const f32x4*>(mean + c);
        f32x4 is = *reinterpret_cast<const f32x4*>(invstd + c);
        f32x4 ga = *reinterpret_cast<const f32x4*>(gamma + c);
        f32x4 r, gq;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float g = o[j] > 0.f ? d[j] : 0.f;
            float xhat = (v[j] - mu[j]) * is[j];
            gq[j] = g;
            r[j] = ga[j] * is[j] * (g - s_db[c + j] * inv_count - xhat * (s_dg[c + j] * inv_count));
        }
        if (HAS_ADD) r += Act<T>::load4(add + p * C + c);  // gradient arriving through an identity shortcut
        Act<T>::store4(dy + p * C + c, r);
        if (g_out) Act<T>::store4(g_out + p * C + c, gq);
    }
}

void launch_bn_bwd_apply(hipStream_t s, int act, const void* dout, int dout_positions_shared, const void* out, const void* y,
                         int64_t pixels, int C, const float* mean, const float* invstd, const float* gamma,
                         const fixsum_t* sums, float* dgamma, float* dbeta, void* dy, void* g_out, const void* add, Reps reps) {
    int64_t total = pixels * (C / 4);
    int64_t blocks = (total + 255) / 256;
    const int64_t cap = (C > 64 || add) ? 1024 : 4096;   // as in launch_bn_apply
    if (blocks > cap) blocks = cap;
#define BN_BWD_APPLY(MAXC, HAS_ADD)                                                                                                   \
    hipLaunchKernelGGL((bn_bwd_apply_kernel<T, MAXC, HAS_ADD>), dim3((unsigned)blocks, 1, reps.n), dim3(256), 0, s, dout, dout_positions_shared,   \
                       (const T*)out, (const T*)y, pixels, C, mean, invstd, gamma, sums, dgamma, dbeta, 1.f / (float)pixels, (T*)dy,  \
                       (T*)g_out, (const T*)add, cq_log2, reps.stride)
    const int cq_log2 = quads_log2(C);
    ACT_DISPATCH(act, {
        if (C > 64 || add) {
            if (add) BN_BWD_APPLY(BN_MAX_C, true);
            else BN_BWD_APPLY(BN_MAX_C, false);
        } else {
            BN_BWD_APPLY(64, false);
        }
    });
#undef BN_BWD_APPLY
}
