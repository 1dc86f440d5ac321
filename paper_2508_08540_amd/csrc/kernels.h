// Launchers of the network kernels.  Every function enqueues on `s` and returns nothing; argument
// shapes are validated by the callers in net.hip before any launch.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Storage type of activations in the launchers below (pointers to activations are void*).
enum { ACT_F32 = 0, ACT_BF16 = 1 };
static inline size_t act_bytes(int act) { return act == ACT_BF16 ? 2 : 4; }

// Per-channel sums that cross workgroups are accumulated as 64-bit fixed-point integers with atomic adds:
// integer addition is associative, so the result does not depend on the order in which workgroups arrive
// (bit-reproducible), and no partial-sum rows or finalisation kernels are needed.  A float partial p
// contributes llrint(p * scale); forward statistics use 2^30 (resolution 2^-30), backward sums 2^44, weight
// gradients 2^40.  The accumulators must be zero before the producing kernel.
//
// Range.  A word takes at most FIX_WORD_CONTRIBUTIONS partials (the launchers cap their grids accordingly; the
// convolution's epilogue, whose grid is capped at 512 workgroups over 16 replicas, half as many), each below
// FIX_PARTIAL_LIMIT (there: twice that) in scaled units, so a word stays below 2^59 in magnitude: neither a word nor
// the sum of its 16 replicas can wrap.  A partial that is not finite or not below the limit does not add: it raises
// the word to FIX_POISON with a signed atomic maximum (later additions cannot bring it back below FIX_POISON_MIN).
// Workgroup 0 of every consumer, the one that stores the statistics, checks for poisoned words and stores NaN then; the
// update turns a poisoned weight-gradient word into a NaN gradient.  An overflow or a non-finite value therefore ends,
// as in floating point, in NaN statistics, gradients, parameters and losses instead of in finite garbage.  Limits of a
// partial in real units: 2^24 for forward sums (the sum of squares of one tile of 256 outputs: rms below 256), 2^9 for
// backward sums (2^10 from a convolution's epilogue), 2^13 for weight-gradient sums.
typedef unsigned long long fixsum_t;
#define FIX_WORD_CONTRIBUTIONS 64
#define FIX_PARTIAL_LIMIT 9007199254740992.0   // 2^53 = 2^59 / FIX_WORD_CONTRIBUTIONS
#define FIX_POISON (1ll << 62)
#define FIX_POISON_MIN (1ll << 61)
__device__ __forceinline__ void fixsum_add(fixsum_t* dst, double scaled, double limit = FIX_PARTIAL_LIMIT) {
    if (fabs(scaled) < limit) atomicAdd(dst, (fixsum_t)__double2ll_rn(scaled));
    else atomicMax(reinterpret_cast<long long*>(dst), FIX_POISON);   // also taken by NaN
}
// The same in two steps for a workgroup that walks several tiles: every tile's partial is converted and range-checked by
// itself and added up as integers in a register, one atomic goes out at the end.  The word then receives exactly what
// one workgroup per tile would have added, so the result does not depend on how tiles are dealt to workgroups.
__device__ __forceinline__ void fixsum_collect(long long& sum, bool& poisoned, double scaled, double limit) {
    if (fabs(scaled) < limit) sum += __double2ll_rn(scaled);
    else poisoned = true;   // also taken by NaN
}
__device__ __forceinline__ void fixsum_flush(fixsum_t* dst, long long sum, bool poisoned) {
    if (poisoned) atomicMax(reinterpret_cast<long long*>(dst), FIX_POISON);
    else atomicAdd(dst, (fixsum_t)sum);
}
// ReLU that keeps NaN (the hardware maximum returns the other operand): a poisoned statistic or a diverged weight has to
// reach the losses instead of being clamped to zero on the way.
__device__ __forceinline__ float relu_keep_nan(float t) { return t < 0.f ? 0.f : t; }
// Each accumulator is replicated FIX_REPLICAS times (workgroup b adds into replica b % FIX_REPLICAS) to
// spread the atomic traffic; readers add the replicas (integer, exact).  One set = FIX_SET entries.
#define FIX_REPLICAS 16
#define FIX_SET (FIX_REPLICAS * 2 * 64)
__device__ __forceinline__ long long fixsum_read(const fixsum_t* sums, int C, int which, int c) {
    long long t = 0;
#pragma unroll
    for (int r = 0; r < FIX_REPLICAS; ++r) t += (long long)sums[(r * 2 + which) * C + c];
    return t;
}
// True if either sum of channel c holds a poisoned word (checked by the one workgroup that stores the statistics).
__device__ __forceinline__ bool fixsum_poisoned(const fixsum_t* sums, int C, int c) {
    long long top = 0;   // all loads in flight at once: the words are in cache, the other workgroups have just read them
#pragma unroll
    for (int r = 0; r < 2 * FIX_REPLICAS; ++r) {
        const long long w = (long long)sums[r * C + c];
        top |= w & ~(w >> 63);   // bits of the non-negative words (a poisoned word is positive)
    }
    return top >= FIX_POISON_MIN;
}
#define FIX_NAN __int_as_float(0x7fc00000)
#define FIX_FWD_SCALE 1073741824.0
#define FIX_BWD_SCALE 17592186044416.0

// Several replicas of a network in one launch (the workers of a communication round side by side): every buffer of
// replica r sits `stride` bytes after the same buffer of replica r - 1 (parameters, statistics, activations, sums:
// one slot per replica, all laid out alike), the launchers below take the pointers of replica 0 and add a grid
// dimension (blockIdx.z = replica); a kernel shifts its pointers by blockIdx.z * stride before anything else.
// The default is one replica and no shift.
struct Reps {
    int n = 1;
    int64_t stride = 0;
};
// Pointer p of replica 0 as replica r sees it (`ro` = r * stride bytes); null stays null.
template <typename P>
__device__ __forceinline__ P rep_at(P p, int64_t ro) {
    return p ? (P)((const char*)p + ro) : p;
}
// Per-replica selection lists of a batched gather (the only per-replica arguments that are not slot-relative).
#define GATHER_MAX_REPS 64
struct GatherReps {
    const int32_t* sel[GATHER_MAX_REPS];
    int64_t k[GATHER_MAX_REPS];
};

// Optional pair of events that a launcher attaches to its kernel dispatch (start and end of that kernel).
struct KernelTiming {
    hipEvent_t start, stop;
};

// ---- elementwise.hip ----------------------------------------------------------------------------
// dst[b][0..row) = src[idx[(start + b) % k]][0..row_src) zero-padded to `row` floats per `group`:
// each source row is `row_src/group_src`... see gather_rows for the image variant.
void launch_gather_rows(hipStream_t s, const float* src, const int32_t* y_src, const int32_t* sel, int64_t k,
                        int64_t start, int batch, int64_t row, float* dst, int32_t* y_dst);
// Images float [n][pixels][c_src] -> storage type `act` [batch][pixels][c_dst] with zero-filled extra channels; sel == nullptr copies
// images first .. first+batch-1, otherwise image b is sel[(start + b) % k].
void launch_gather_images(hipStream_t s, const float* src, const int32_t* y_src, const int32_t* sel, int64_t k,
                          int64_t start, int64_t first, int batch, int pixels, int c_src, int c_dst, int act, void* dst,
                          int32_t* y_dst);
// The same for several replicas at once: replica r gathers by lists.sel[r] / lists.k[r] into its own dst / y_dst.
void launch_gather_images_reps(hipStream_t s, const float* src, const int32_t* y_src, const GatherReps& lists, int64_t start, int batch,
                               int pixels, int c_src, int c_dst, int act, void* dst, int32_t* y_dst, Reps reps);
void launch_sgd(hipStream_t s, float* params, float* momentum, const float* grad, int64_t d, float lr, float mu,
                float wd);
// out[n] = sum_b in[b][n]
void launch_colsum(hipStream_t s, const float* in, int rows, int cols, float* out);
void launch_fill_zero(hipStream_t s, float* p, int64_t n, Reps reps = Reps{});

// ---- gemm.hip ---------------------------------------------------------------------------------------
// C[m][n] = sum_k A(m,k) * B(n,k); A(m,k) = a_kmajor ? A[k*lda+m] : A[m*lda+k], likewise B.
// Split over `splits` K-ranges into part[splits][M][N], then reduced in split order into out with
// optional bias[n] add, ReLU, and multiplication by (mask[m][n] > 0).
size_t gemm_partial_floats(int M, int N, int splits);
void launch_gemm(hipStream_t s, const float* A, int lda, bool a_kmajor, const float* B, int ldb, bool b_kmajor, int M,
                 int N, int K, int splits, float* part, float* out, const float* bias, bool relu, const float* mask);

// ---- head.hip ---------------------------------------------------------------------------------------
// One wave per sample: feature = mean over `positions` of act[b][p][F] (storage type act_type); logits = W feature + bias;
// loss = softmax cross-entropy.  Training outputs (all optional, nullptr to skip): feat [B][F],
// dlogits [B][C] scaled by grad_scale, dact [B][F] = (W^T dlogits) / positions, masked by feature > 0
// when relu_mask is set.
void launch_head_forward(hipStream_t s, int act_type, const void* act, int B, int positions, int F, const float* W, const float* bias,
                         int C, const int32_t* y, float* loss, float* feat, float* dlogits, float* dfeat,
                         float grad_scale, bool relu_mask, Reps reps = Reps{});
// dW[c][f] = sum_b dlogits[b][c] feat[b][f]; db[c] = sum_b dlogits[b][c]
void launch_head_wgrad(hipStream_t s, const float* dlogits, const float* feat, int B, int C, int F, float* dW, float* db, Reps reps = Reps{});

// ---- norm.hip ---------------------------------------------------------------------------------------
// Where the normalisation statistics of bn_apply come from.  Training: `sums` holds the fixed-point
// (sum, sum of squares) of y over `count` values; every workgroup derives mean and invstd from them, and
// workgroup 0 also stores them into mean/invstd and moves the running statistics.  Inference: sums == nullptr
// and the running statistics are used.  At most 512 channels.
#define BN_EPS 1e-5        // variance offset of the batch norm (Section 5.1: PyTorch defaults)
#define BN_MOMENTUM 0.1    // weight of the batch statistics in the running ones
struct BnStats {
    const fixsum_t* sums;
    double count;
    float *mean, *invstd, *running_mean, *running_var;
};
// mean[c] = running_mean[c], invstd[c] = 1 / sqrt(running_var[c] + BN_EPS) rounded as bn_apply_kernel rounds it: the
// constants of a batch norm in inference, for kernels that apply it in their epilogue
void launch_bn_inference_stats(hipStream_t s, const float* running_mean, const float* running_var, int C, float* mean, float* invstd);
// a = relu(gamma * (y - mean) * invstd + beta [+ shortcut(res)]); res has c_res channels at res_stride x resolution
void launch_bn_apply(hipStream_t s, int act, const void* y, int64_t pixels, int C, const BnStats& st, const float* gamma,
                     const float* beta, const void* res, int c_res, int res_stride, int h_out, void* out, Reps reps = Reps{});
// Backward of relu(bn(y) [+ shortcut]) for a layer whose upstream gradient does not come from an input-gradient
// kernel: g = dout * (out > 0); dout is a tensor of the storage type, or, with dout_positions_shared > 0, an fp32
// [samples][C] matrix whose rows are shared by that many positions; adds (sum g, sum g*xhat) into the fixed-point accumulators `sums` [2][C].
void launch_bn_bwd_reduce(hipStream_t s, int act, const void* dout, int dout_positions_shared, const void* out, const void* y,
                          int64_t pixels, int C, const float* mean, const float* invstd, fixsum_t* sums, Reps reps = Reps{});
// dy = gamma*invstd*(g - dbeta/M - xhat*dgamma/M) with g = dout * (out > 0) and (dbeta, dgamma) read from `sums`;
// workgroup 0 stores dgamma and dbeta; g_out (optional) receives g; `add` (optional, shape of dy) is added to dy.
void launch_bn_bwd_apply(hipStream_t s, int act, const void* dout, int dout_positions_shared, const void* out, const void* y,
                         int64_t pixels, int C, const float* mean, const float* invstd, const float* gamma,
                         const fixsum_t* sums, float* dgamma, float* dbeta, void* dy, void* g_out, const void* add = nullptr, Reps reps = Reps{});
// ---- conv.hip ---------------------------------------------------------------------------------------
struct ConvShape {
    int B, h_in, c_in, c_out, stride;  // square maps; 3x3, padding 1; c_in, c_out in {16, 32, 64}
    int c_in_real;                     // weights hold this many input channels (<= c_in); the rest are zero
    int taps = 9;                      // 9: 3x3 filter with padding 1; 1: 1x1 filter (weight-gradient and wide kernels only)
};
// Packed (lane-major) weight copies for the convolution kernels; see pack_weights_kernel.
#define PACK_MAX_ENTRIES 72
struct PackEntry {
    int64_t w_off;     // offset of w[c_out][3][3][c_in_real] in the parameter vector
    int64_t pack_off;  // offset of this entry in the packed buffer, in quads (4 values of the storage type)
    int c_in, c_out, c_in_real, dgrad;
    int taps, pad_;    // 9 (3x3) or 1 (1x1)
};
struct PackTable {
    int n;
    int64_t total_vec4;
    PackEntry e[PACK_MAX_ENTRIES];
};
void launch_pack_weights(hipStream_t s, int act, const float* params, void* packed, const PackTable& tab, Reps reps = Reps{});
// Fused epilogue of the convolution kernels (see conv_kernel).  `sums` points at [replica][2][channels] accumulators:
// forward (sum, sum of squares) of the output; input gradient (sum g, sum g*xhat) of the layer below.
struct ConvEpi {
    fixsum_t* sums;
    double scale;
    double tile_limit;   // bound of one tile's scaled partial sum (set by the launcher)
    // input gradient: shortcut gradient to add (sc_g may be nullptr), then the ReLU of the layer below (the output is stored
    // with zeros where a_prev is zero: the gradient behind that ReLU), then batch-norm backward sums of the layer below
    const void* sc_g;  // activations (storage type of the launch)
    int sc_c, sc_lo, sc_stride;
    const void *a_prev, *y_prev;  // activations
    const float *mean_prev, *invstd_prev;
    // inference forward (gamma != nullptr): out = relu(bn(y) + shortcut) with mean_prev = running mean, invstd_prev =
    // running variance, sc_g = shortcut source (c channels sc_c, first output channel sc_lo, spatial stride sc_stride)
    const float *gamma, *beta;
    // training forward with in_sums != nullptr: the input x is the raw convolution output of the layer below.  The kernel
    // turns that layer's sums into statistics (workgroup 0 stores them and updates the running statistics, as bn_apply
    // does), applies its batch norm (+ shortcut) and ReLU while staging, and writes the activation to a_out for the backward pass.
    // 3x3 layers of either stride; the values are those bn_apply would have stored.
    const fixsum_t* in_sums;
    double in_count;
    float *in_mean, *in_invstd, *in_rmean, *in_rvar;
    const float *in_gamma, *in_beta;
    const void* in_res;   // optional shortcut added before the ReLU (the end of a block): in_res_c channels that go to
    int in_res_c, in_res_lo, in_res_stride;   // x's channels in_res_lo .. (zeros elsewhere), read at every in_res_stride-th pixel
    void* a_out;
    // input gradient with bw_dout != nullptr (stride-1 layers): the launch's input dy does not exist yet.  The kernel computes
    // it while staging, as bn_bwd_apply does, from the gradient bw_dout behind the layer's ReLU (zero where the activation
    // is: the input-gradient launch of the layer above stored it that way), the layer's convolution output bw_y, its
    // statistics and the backward sums bw_sums [2][C] (workgroup 0 stores the scale and shift gradients), and stores it to
    // bw_dy_out for the weight gradient.
    const void *bw_dout, *bw_y;
    const float *bw_mean, *bw_invstd, *bw_gamma;
    const fixsum_t* bw_sums;
    float *bw_dgamma, *bw_dbeta;
    float bw_inv_count;
    void* bw_dy_out;
};
int conv_fwd_tiles(const ConvShape& cs);
// x, y, dy, dx are activations of storage type `act`.  In the three launchers below `w` is the packed copy (forward form for fwd, input-gradient form for dgrad).
// y = conv(x, w); with `stats` the kernel also accumulates (sum, sum of squares) of y per channel, or, when
// stats->gamma is set, applies inference batch norm + shortcut + ReLU before storing.
void launch_conv_fwd(hipStream_t s, int act, const ConvShape& cs, const void* x, const void* w, void* y, const ConvEpi* stats,
                     const KernelTiming* kt = nullptr, Reps reps = Reps{});
// dx = conv_transpose(dy, w) [+ shortcut gradient]; with `bn_below` also the batch-norm backward sums of the layer
// that produced x.
void launch_conv_dgrad(hipStream_t s, int act, const ConvShape& cs, const void* dy, const void* w, void* dx, const ConvEpi* bn_below,
                       const KernelTiming* kt = nullptr, Reps reps = Reps{});
// Adds dy (x) shifted x over all pixels into gacc: [replica][c_out/16][c_in/16][2304] fixed-point accumulators
// (conv_wgrad_accumulators entries, zero before the call) ...
int64_t conv_wgrad_accumulators(int act, const ConvShape& cs);
int conv_wgrad_replicas(int act, const ConvShape& cs);
void launch_conv_wgrad(hipStream_t s, int act, const ConvShape& cs, const void* x, const void* dy, fixsum_t* gacc,
                       const KernelTiming* kt = nullptr, Reps reps = Reps{});
// End of a local step in one launch (see update_kernel): gradient of every parameter (convolution weights from the
// accumulators, which are cleared; the rest from grad[]), SGD update, refresh of the packed weight copies, and
// clearing of the n_sums batch-norm accumulators.
#define WGRAD_MAX_ENTRIES 40
struct UpdateEntry {
    int64_t w_off, n;     // w[c_out][3][3][c_in_real] in the parameter vector
    int64_t acc_off;      // this layer's accumulators in gacc
    int64_t fwd_quad;     // quad offset of the forward packed copy
    int64_t dgrad_quad;   // quad offset of the input-gradient packed copy, -1 if the layer has none
    int c_in, c_out, c_in_real, taps;
    int replicas, pad_;   // accumulator replicas of this layer (conv_wgrad_replicas)
};
struct UpdateTable {
    int n;
    UpdateEntry e[WGRAD_MAX_ENTRIES];
};
// Parameters begin .. end - 1 (end < 0: d); the batch-norm accumulators `sums` (n_sums words, may be 0) are cleared as well.
void launch_update(hipStream_t s, int act, float* params, float* momentum, const float* grad, int64_t d, float lr, float mu,
                   float wd, fixsum_t* gacc, void* packed, const UpdateTable& tab, fixsum_t* sums, int64_t n_sums, Reps reps = Reps{},
                   int64_t begin = 0, int64_t end = -1);

// ---- wconv.hip --------------------------------------------------------------------------------------
// Convolution for wide layers: y = conv(x, w) [+ add] with a 3x3 (taps 9, padding 1) or 1x1 (taps 1) filter;
// c_in is 16 or a multiple of 32, c_out a multiple of 16; `w` is the packed copy (forward form, or input-gradient
// form when the call computes an input gradient: then c_in / c_out are the layer's output / input channels,
// stride is 1 and ups = 1 reads x with zeros inserted, which undoes a stride-2 layer).  With `sums` the
// (sum, sum of squares) of the stored values are added into [replica][2][c_out] accumulators scaled by `scale`.
// Returns 0, or -1 for a shape the kernel does not cover (nothing is launched).
// With `bn` (inference) the batch norm with running statistics and the ReLU of the layer that reads the result are applied
// before the store: y = relu(bn(r)) with r the result rounded to the storage type, which also goes to bn->raw when that is
// not null (a later identity shortcut adds it).  The arithmetic is bn_apply_kernel's.  Not together with `sums`.
struct WconvBn {
    const float *mean, *invstd, *gamma, *beta;   // per output channel
    void* raw;
};
int launch_wconv(hipStream_t s, int act, int taps, int B, int h_in, int h_out, int c_in, int c_out, int stride, int ups, const void* x,
                 const void* w, void* y, const void* add, fixsum_t* sums, double scale, const WconvBn* bn = nullptr);

// ---- gemm_tiled.hip -----------------------------------------------------------------------------------
// C[m][n] = alpha * sum_k A(m,k) B(n,k) [+ bias[n]] [+ R[m][n]]; A(m,k) = a_kmajor ? A[k*lda + m] : A[m*lda + k], same for B.
// Batched over z = z1 * inner + z2 (z1 < batch / inner): pointer offsets z1*s?1 + z2*s?2 (R uses C's).  splits > 1 splits
// K into partials in `part` (batch must be 1) that are added in order.  Fields below the line are filled by the launcher.
struct GemmDesc {
    const float *A, *B;
    float* C;
    const float *bias, *R;
    float* part;
    float* G;   // optional second output gelu(C), same layout as C (single matrix, no split)
    int M, N, K, lda, ldb, ldc;
    int a_kmajor, b_kmajor;
    int batch, inner, splits;
    int64_t sa1, sa2, sb1, sb2, sc1, sc2;
    float alpha;
    // ----
    int k_chunk, a_vec, b_vec;
    int64_t part_stride;
};
size_t gemm_tiled_partial_floats(int M, int N, int splits);
void launch_gemm_tiled(hipStream_t s, GemmDesc d);

// true where the bf16 weight-gradient kernel (wgrad16.hip) takes the layer
bool wgrad16_covers(int act, const ConvShape& cs);

// ---- gemm16.hip --------------------------------------------------------------------------------------
// The same product with both operands stored in bf16 (uint16_t bit patterns).  Outputs: C fp32, C16 bf16, G16 = gelu(C)
// in bf16, any of them NULL; ldc and the batch strides sc1/sc2 apply to all of them and to R.  splits > 1 needs
// batch == 1 and writes C only.  Fields below the line are filled by the launcher.
struct Gemm16Desc {
    const uint16_t *A, *B;
    float* C;
    uint16_t *C16, *G16;
    const float *bias, *R;
    float* part;
    int M, N, K, lda, ldb, ldc;
    int a_kmajor, b_kmajor;
    int batch, inner, splits;
    int64_t sa1, sa2, sb1, sb2, sc1, sc2;
    int64_t sbias1;   // floats between the bias vectors of consecutive z1 (unsplit products only)
    float alpha;
    // optional softmax statistics of the rows of C (single matrix, no split): per row and per 64-column block the pair
    // (max, sum exp(C - max)) into ce_part[2 * ceil(N / 128)][M][2], and C[m][ce_targets[m]] into ce_tlogit[m]
    float* ce_part;
    const int32_t* ce_targets;
    float* ce_tlogit;
    // ----
    int k_chunk, a_vec, b_vec, c_vec;
    int64_t part_stride;
};
void launch_gemm16(hipStream_t s, Gemm16Desc d);

// ---- seq.hip ------------------------------------------------------------------------------------------
// Accumulator ranges that fix_finalize turns into gradients: grad[grad_off + i] = acc[acc_off + i] / 2^44, acc cleared.
#define FIX_MAX_RANGES 112
struct FixRange {
    int64_t acc_off, grad_off, n;
};
struct FixRangeTable {
    int n;
    FixRange r[FIX_MAX_RANGES];
};
void launch_embed(hipStream_t s, const int32_t* tokens, int64_t T, int L, int D, const float* tok, const float* pos, float* h, uint16_t* h16);
void launch_to_bf16(hipStream_t s, const float* in, uint16_t* out, int64_t n);
void launch_embed_grad(hipStream_t s, const int32_t* tokens, int64_t T, int D, const float* dh, fixsum_t* acc_tok);
// Column sums in two halves, the second half of many of them in one launch: partial sums of row chunks land in one
// buffer (part_off), the table kernel folds each job's rows in a fixed order into out[out_off ..].
#define COLSUM_TABLE_MAX 64
struct ColsumJob {
    int64_t part_off, out_off;
    int rows, N, pitch;   // pitch = floats between the rows of the partial sums
};
struct ColsumTable {
    ColsumJob j[COLSUM_TABLE_MAX];
    int n;
};
int launch_colsum_partial(hipStream_t s, const float* X, int64_t M, int N, float* part);
void launch_colsum_table(hipStream_t s, const ColsumTable& tab, const float* part, float* out);
int launch_layernorm_bwd_partial(hipStream_t s, const float* dy, const float* x, const float* stats, int64_t T, int D, const float* g, float* dx,
                                 uint16_t* dx16, float* part);
size_t colsum_partial_floats(int64_t M, int N);
void launch_colsum_tokens(hipStream_t s, const float* X, int64_t M, int N, float* part, float* out);
void launch_fix_finalize(hipStream_t s, const FixRangeTable& tab, fixsum_t* acc, float* grad);
void launch_layernorm(hipStream_t s, const float* x, int64_t T, int D, const float* g, const float* b, float* y, uint16_t* y16, float* stats);
size_t layernorm_bwd_partial_floats(int64_t T, int D);
void launch_layernorm_bwd(hipStream_t s, const float* dy, const float* x, const float* stats, int64_t T, int D, const float* g, float* dx,
                          uint16_t* dx16, float* part, float* dgb);
// Fused self-attention with bf16 factors for short sequences (L <= 128, L % 8 == 0, dh 32 or 64): ctx = softmax(alpha q k^T) v per
// (sample, head); P / P16 (nullable) keep the probabilities as [B][H][L][L].  Returns false, having launched nothing, for
// anything else.
bool launch_attention16(hipStream_t s, const uint16_t* q, const uint16_t* k, const uint16_t* v, int ld, int B, int H, int L, int dh, float alpha,
                        uint16_t* ctx, int ldc, float* P, uint16_t* P16);
// Its backward pass from dctx (bf16) and the fp32 probabilities: dq, dk, dv as fp32 and bf16, same shapes and limits.
// colsum (optional) takes partial column sums for the bias gradients: three [4 B][H dh] arrays (dq, dk, dv in that order), row
// 4 b + w = the sum over the rows of sample b that wave w of its workgroups owned.
bool launch_attention16_bwd(hipStream_t s, const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* dctx, const float* P, int ld, int B,
                            int H, int L, int dh, float alpha, float* dq, float* dk, float* dv, uint16_t* dq16, uint16_t* dk16, uint16_t* dv16,
                            float* colsum);
void launch_softmax_rows(hipStream_t s, float* sc, uint16_t* p16, bool store_f32, int64_t rows, int n);
void launch_softmax_bwd_rows(hipStream_t s, float* dp, const float* p, uint16_t* ds16, int64_t rows, int n, float scale);
void launch_gelu_bwd(hipStream_t s, float* dg, const float* u, uint16_t* du16, int64_t n);
// The same on a [M][N] tensor, leaving partial column sums of the result (returned number of rows x N floats) in part;
// returns 0 and launches nothing where its vector accesses do not fit
size_t gelu_bwd_colsum_floats(int64_t M, int N);
int launch_gelu_bwd_colsum(hipStream_t s, float* dg, const float* u, uint16_t* du16, int64_t M, int N, float* part);
// Cross-entropy from the statistics the vocabulary projection left behind: folds the n_parts pairs of a row in index
// order; tok_loss[t] = max + log(sum) - tlogit[t]; row_stats[t] = (max, sum) if given.
void launch_ce_combine(hipStream_t s, const float* ce_part, int n_parts, const float* tlogit, int64_t T, float* tok_loss, float* row_stats);
// d16[t][c] = bf16((exp(logits[t][c] - max_t) / sum_t - [c == target_t]) * grad_scale)
void launch_ce_grad(hipStream_t s, const float* logits, const int32_t* targets, const float* row_stats, int64_t T, int V, float grad_scale,
                    uint16_t* d16);
void launch_token_ce(hipStream_t s, float* logits, const int32_t* targets, int64_t T, int V, float* tok_loss, float grad_scale, uint16_t* d16);
void launch_sample_mean(hipStream_t s, const float* tok_loss, int B, int L, float* loss);
