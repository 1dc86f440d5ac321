/*
 * bls.h - C ABI of the biased-local-SGD fast path for AMD MI355X (gfx950).
 *
 * The four operations are the fast worker's share of one communication round of the
 * system-aware biased local SGD framework (arXiv 2508.08540, Algorithm 1):
 *
 *   score_losses        one loss value per candidate sample (Section 4.2: samples are ranked
 *                       by loss value; Section 4.3 limitations: one float per sample)
 *   topk_by_loss        deterministic selection of the k highest-loss samples (Section 4.2,
 *                       first sampling step of Algorithm 1)
 *   local_step          tau local mini-batch SGD updates on the selected samples, recording the
 *                       individual losses of the processed samples (Section 2 update rule;
 *                       local-update and loss-recording steps of Algorithm 1)
 *   weighted_aggregate  x_{t+1} = sum_i (tau_i / sum_j tau_j) x^i_t (Section 4.3, Eq. 4)
 *
 * Conventions for every call
 *   - "device" pointers are HIP device memory on the context's GPU, owned by the caller and not
 *     retained after the call returns; "host" pointers are ordinary memory, read before return.
 *   - Work is enqueued on the context's stream and the call returns without waiting; the caller
 *     synchronises the stream before reading results.  Scratch memory belongs to the context.
 *   - Return value: BLS_OK (0) or a negative bls_status.  Argument errors are detected on the
 *     host before anything is enqueued and leave all outputs untouched; bls_last_error() then
 *     describes the problem.  Nothing is printed and nothing aborts.
 *   - Results are bit-reproducible run to run (no floating-point atomics).  Sums over a whole batch that many
 *     workgroups contribute to (batch-norm statistics, the two sums of the batch-norm backward pass, convolution
 *     weight gradients, token-embedding gradients) are accumulated as 64-bit fixed-point integers, which bounds what one
 *     tile of a launch may contribute (bls_sum_limits): 2^24 to a forward sum (the sum of squares of 256 convolution
 *     outputs, i.e. an rms below 256 per tile), 2^9 to a backward sum, 2^13 to a weight-gradient sum; convolution
 *     launches of more than 512 tiles (batches above 128 images of 32 x 32) halve the first two with every doubling
 *     of the tile count.  A contribution beyond its
 *     limit, or one that is not finite, does not wrap around and is not dropped: the sum becomes NaN, and with it the
 *     statistics, gradients, parameters and every later loss, as an overflow in floating point would end.  Inputs
 *     normalised to unit scale (the convention of the paper's image pipelines) stay four orders of magnitude below
 *     the limits; raw 8-bit pixel values (0 .. 255) are within them.
 *   - One context must not be used from two threads at once.
 */
#ifndef BLS_H
#define BLS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BLS_OK = 0,
    BLS_EINVAL = -1,       /* bad argument (NULL, size out of range, k > N, ...)          */
    BLS_ENOMEM = -2,       /* device or host allocation failed                            */
    BLS_EHIP = -3,         /* a HIP runtime call failed; see bls_last_error()              */
    BLS_EUNSUPPORTED = -4  /* valid request outside what the kernels are built for        */
} bls_status;

typedef struct bls_ctx bls_ctx;     /* device, stream (borrowed) and library-owned scratch */
typedef struct bls_model bls_model; /* architecture and flat-parameter layout (host only)  */

enum { BLS_MODEL_MLP = 0, BLS_MODEL_RESNET_CIFAR = 1, BLS_MODEL_WRN = 2, BLS_MODEL_ENCODER = 3 };

/* Storage type of the activations (and of the copies of the convolution weights the kernels read).
 * Parameters, momentum, gradients, batch-norm statistics, losses and every reduction stay fp32: with
 * BLS_ACT_BF16 the parameter vector is the fp32 master copy of a mixed-precision run. */
enum { BLS_ACT_F32 = 0, BLS_ACT_BF16 = 1 };

/* Architecture description.
 *   MLP:           image_hw*image_hw*in_channels -> hidden (ReLU) -> classes.
 *   RESNET_CIFAR:  3x3 stem conv to widths[0], three stages of `blocks` two-convolution residual
 *                  blocks with widths[0..2] (stride 2 and a parameter-free zero-padded shortcut at
 *                  the start of stages 2 and 3), batch norm after every convolution, global
 *                  average pooling, linear classifier.  ResNet20 (Section 5) is widths 16/32/64,
 *                  blocks 3, image_hw 32, in_channels 3, classes 10.
 *   WRN:           pre-activation wide residual network (the WRN16 of Section 5): 3x3 stem conv to `hidden`
 *                  channels, three stages of `blocks` blocks  out = shortcut + conv2(relu(bn2(conv1(relu(bn1(x))))))
 *                  with widths[0..2], stride 2 at the start of stages 2 and 3, identity shortcut where the block
 *                  keeps its shape and a 1x1 convolution of relu(bn1(x)) otherwise; batch norm, ReLU, global
 *                  average pooling, linear classifier.  WRN-16-8 is hidden 16, widths 128/256/512, blocks 2,
 *                  image_hw 32, classes 100.  Tensor order: stem.conv; per block bn1, conv1, bn2, conv2,
 *                  [shortcut]; final.bn; fc.
 *   ENCODER:       transformer encoder language model standing in for the language workload of Section 5: token and
 *                  learned position embeddings, `blocks` post-layer-norm layers  h = LN1(h + MHA(h)),
 *                  h = LN2(h + W2 gelu(W1 h + b1) + b2)  with unmasked self-attention, erf GELU, layer-norm eps 1e-5,
 *                  and a bias-free projection to the vocabulary.  A sample is one sequence; its loss is the mean of
 *                  its per-position cross-entropies (Section 4.3 ranks one loss per sample).
 *                  classes = vocabulary size (2 .. 2^20), image_hw = sequence length (1 .. 1024), hidden = model
 *                  width (multiple of 4, at most 1024), widths[0] = heads (divides hidden), widths[1] = feed-forward
 *                  width (multiple of 4), blocks = layers (1 .. 16); in_channels and widths[2] are ignored.
 *                  With BLS_ACT_BF16 both factors of every matrix product (linear layers, attention scores and
 *                  values, and all their gradients) are bf16, rounded to nearest even by the kernel that produces
 *                  them, and multiplied on the bf16 matrix cores with fp32 sums; tensors that are only ever factors
 *                  are stored in bf16 alone.  Everything else (residual sums, layer norm, softmax, the GELU
 *                  derivative, bias and layer-norm gradients, losses, parameters, momentum, the update) is fp32.
 *                  Tensor order: tok_emb, pos_emb; per layer attn.q/k/v/o (weight, bias), ln1, ffn.fc1, ffn.fc2,
 *                  ln2; head.weight. */
typedef struct {
    int32_t kind;        /* BLS_MODEL_*                                    */
    int32_t classes;     /* 2 .. 64 (WRN: 2 .. 128)                        */
    int32_t image_hw;    /* square images; RESNET: 8, 16, 32 or 64; WRN: 8, 16 or 32 */
    int32_t in_channels; /* RESNET, WRN: 1 .. 4                            */
    int32_t hidden;      /* MLP: multiple of 16, 16 .. 1024; WRN: stem channels, 16 or a multiple of 32 up to 512 */
    int32_t widths[3];   /* RESNET: each of 16, 32 or 64; WRN: each 16 or a multiple of 32 up to 512 */
    int32_t blocks;      /* RESNET: 1 .. 6; WRN: 1 .. 4                    */
    int32_t act_dtype;   /* BLS_ACT_*; the MLP supports BLS_ACT_F32 only   */
} bls_model_desc;

/* One tensor of the flat parameter vector (is_buffer = 0) or of the flat buffer vector that
 * holds batch-norm running means and variances (is_buffer = 1).  Offsets count floats.
 * Convolution weights are [C_out, 3, 3, C_in]; linear weights are [out, in]. */
typedef struct {
    char name[56];
    int64_t offset;
    int32_t ndim;
    int32_t shape[4];
    int32_t is_buffer;
} bls_tensor_info;

/* SGD hyper-parameters with the semantics of the optimiser the paper trains with (Appendix A.1):
 * g += weight_decay * x;  buf = momentum * buf + g;  x -= lr * buf. */
typedef struct {
    float lr;
    float momentum;
    float weight_decay;
} bls_sgd;

enum {
    BLS_AGG_NORMALISE = 1, /* divide the weights by their sum instead of requiring sum == 1 */
    BLS_AGG_BROADCAST = 2  /* also store the result into every replica (start of next round) */
};

/* ---- context ------------------------------------------------------------------------------ */

/* Creates a context on HIP device `device`.  `hip_stream` is a hipStream_t owned by the caller
 * (NULL = the default stream); all work of this context is enqueued there. */
int bls_ctx_create(bls_ctx** out, int device, void* hip_stream);
/* Number of workers communication_round runs side by side (1 .. 16, default 1).  With more than one lane the library
 * owns that many extra streams (default priority), each with its own scratch memory; the workers of a round are dealt
 * to them in turn and the context's stream waits for all of them before it aggregates.  Results do not depend on the
 * number of lanes.  Waits for the context's stream. */
int bls_ctx_set_lanes(bls_ctx* ctx, int lanes);
/* Waits for the stream, frees the scratch memory and the context.  NULL is allowed. */
void bls_ctx_destroy(bls_ctx* ctx);
/* Text of the most recent error on this context ("" if none).  Owned by the context. */
const char* bls_last_error(const bls_ctx* ctx);
/* Blocks until everything enqueued on the context's stream has finished. */
int bls_ctx_synchronize(bls_ctx* ctx);

/* Optional per-class kernel timing for benchmarks.  Between begin and end the convolution kernels carry
 * start/stop events on their own dispatch (duration of that kernel alone) and every other group of
 * launches is bracketed by HIP events on the stream it runs on (this slows the calls down; do not
 * time throughput while it is on).  bls_profile_end waits for the stream, adds the elapsed time and the
 * number of bracketed groups per class into the caller's host arrays (capacity entries each,
 * either may be NULL) and returns the number of classes.  Class order: 0 conv forward, 1 conv input
 * gradient, 2 conv weight gradient kernel, 3 batch norm kernels, 4 classifier head, 5 fully connected
 * GEMM, 6 SGD update and weight packing, 7 batch gather, 8 top-k, 9 aggregation, 10 reduction of the
 * weight-gradient partial sums. */
int bls_profile_begin(bls_ctx* ctx);
int bls_profile_end(bls_ctx* ctx, double* ms_by_class, int64_t* launches_by_class, int capacity);

/* ---- model description (host only; no GPU needed) ------------------------------------------- */

int bls_model_create(const bls_model_desc* desc, bls_model** out);
void bls_model_destroy(bls_model* model);
/* d: number of trainable floats.  Buffers: batch-norm running statistics (0 for the MLP). */
int64_t bls_model_num_params(const bls_model* model);
int64_t bls_model_num_buffers(const bls_model* model);
/* Device scratch memory the context grows to (once; it is kept until the context is destroyed): with training != 0 for
 * local_step at batch size n, otherwise for score_losses over a pool of n samples (large pools are scored in chunks, so
 * the figure stops growing).  Activations kept for the backward pass, gradients, partial sums and the kernels' weight
 * copies live there (Algorithm 1's worker holds its model, momentum and data; everything else is this scratch).
 * Host only.  BLS_EINVAL for a NULL model or n outside [1, 2^24]. */
int64_t bls_model_workspace_bytes(const bls_model* model, int64_t n, int training);
/* Number of tensors (parameters and buffers together). */
int32_t bls_model_num_tensors(const bls_model* model);
/* Fills out[0 .. capacity-1]; returns the number of tensors written or BLS_EINVAL. */
int bls_model_tensor_layout(const bls_model* model, bls_tensor_info* out, int32_t capacity);

/* ---- the four operations ------------------------------------------------------------------ */

/* Loss of every candidate under the current parameters (Section 4.2).
 *   params   device float[d]; buffers device float[num_buffers] (may be NULL for the MLP)
 *   x        device float[N, H, W, C] (channels last); y device int32[N], labels in [0, classes)
 *            ENCODER: x device int32[N, L] token ids, y device int32[N, L] target ids, both in [0, classes)
 *   losses_out device float[N]: softmax cross-entropy of sample i, natural logarithm (ENCODER: mean over positions)
 * Batch-norm layers use their running statistics, so a score does not depend on the rest of the
 * pool.  N == 0 is a no-op.  Labels are not range-checked on the device. */
int score_losses(bls_ctx* ctx, const bls_model* model, const float* params, const float* buffers,
                 const void* x, const int32_t* y, int64_t N, float* losses_out);

/* Indices of the k largest losses in rank order (Section 4.2; deterministic).
 *   losses device float[N]; idx_out device int32[k]; val_out device float[k] or NULL
 * Total order: NaN ranks above +inf, -0 equals +0, equal losses rank by ascending index.
 * 0 <= k <= N < 2^31; k == 0 is a no-op.  val_out[r] = losses[idx_out[r]] bit for bit. */
int topk_by_loss(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out);

/* topk_by_loss for callers that cannot allocate device memory (code under HIP graph capture, serving loops and harnesses
 * that forbid hipMalloc): same arguments, same result bit for bit, and no allocation of any kind on the device.  Pools
 * above 16384 losses work in a fixed array of 18 MiB that is part of the library's device image (every GPU the library
 * runs on holds it until the process ends), which limits N to BLS_TOPK_STATIC_MAX_N; a larger N is BLS_EINVAL.  All calls
 * on one GPU share that array: calls that overlap in time on one GPU (two contexts, two streams) race; calls in stream
 * order on one stream do not.  Nothing in the array has to survive between calls, and the launches clear what they count
 * in.  Its device address is looked up when a context is created on the GPU. */
enum { BLS_TOPK_STATIC_MAX_N = 1 << 20 };
int topk_by_loss_static(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out);

/* tau mini-batch SGD updates on the selected samples (Algorithm 1, fast-worker branch).
 *   params, momentum  device float[d], updated in place; buffers device float[num_buffers],
 *                     updated in place (batch norm trains with batch statistics)
 *   x_pool, y_pool    the candidate pool as in score_losses (N samples)
 *   sel_idx           device int32[k], indices into the pool (e.g. from topk_by_loss)
 *   step j (0 <= j < tau) trains on sel_idx[(j*batch + b) mod k], b = 0 .. batch-1; the batch loss
 *   is the mean of the per-sample losses
 *   step_losses_out   device float[tau * batch] or NULL: the loss of every processed sample
 * Requires 1 <= k, 1 <= batch; tau == 0 is a no-op.  A zero momentum vector before the first step
 * gives buf = g there.  Indices are not range-checked on the device. */
int local_step(bls_ctx* ctx, const bls_model* model, float* params, float* buffers, float* momentum,
               const void* x_pool, const int32_t* y_pool, int64_t N, const int32_t* sel_idx, int64_t k,
               int64_t batch, int64_t tau, const bls_sgd* opt, float* step_losses_out);

/* out[j] = sum_i w_i * replicas[i][j], i ascending, in fp32 (Eq. 4).
 *   replicas host array of P device pointers to float[d]; weights host float[P], finite,
 *   non-negative, summing to 1 within 1e-5 unless BLS_AGG_NORMALISE is given
 *   out device float[d]; may be one of the replicas
 * 1 <= P <= 64.  d == 0 is a no-op.  Non-finite parameter values propagate (IEEE). */
int weighted_aggregate(bls_ctx* ctx, const float* const* replicas, const float* weights, int P, int64_t d,
                       float* out, int flags);

/* ---- one communication round (Algorithm 1: local steps of every worker, loss recording, aggregation) ---- */

/* One worker of a round.  All pointers are device pointers.
 *   tau        local steps this round (0: the worker neither trains nor counts)
 *   idx, n_idx the samples assigned to it (a segment of sample_epoch's output); entries distinct
 *   params, buffers  storage for its replica, float[d] / float[num_buffers]; overwritten with the global model when the
 *              round starts, they hold the trained replica afterwards
 *   momentum   float[d], the worker's own optimiser state, kept from round to round by the caller */
typedef struct {
    int64_t tau;
    const int32_t* idx;
    int64_t n_idx;
    float* params;
    float* buffers;
    float* momentum;
} bls_worker;

/* Every worker with tau > 0, in the order given: replica <- global model; tau local steps on its samples as in
 * local_step (batches walk idx cyclically); then  global_params <- sum_i (tau_i / sum_j tau_j) * params_i  (Eq. 4), and
 * the same for the batch-norm running statistics in global_buffers.
 *   workers     host array of P descriptions, 1 <= P <= 64
 *   loss_table  device float[N] or NULL: the loss of every processed sample is stored at its index (the loss-recording
 *               step of Algorithm 1); a sample processed more than once keeps the loss recorded last, in the order
 *               workers, steps, positions; other entries are left alone
 * The weights are computed in double from the step counts and rounded once, as by bls_weights_from_tau.
 * The workers are the parallel loop of Algorithm 1.  For RESNET_CIFAR models (and no lanes set) they run side by side
 * inside the kernels: one launch per layer covers every worker that still has steps to take, each worker in a scratch
 * slot of its own (bls_model_workspace_bytes(model, batch, 1) plus two parameter vectors per worker).  Otherwise they run
 * one after the other on the context's stream, or on the lanes set with bls_ctx_set_lanes.  The recorded losses, the
 * replicas and the aggregate are the same bits on every path.  Errors as for local_step and weighted_aggregate;
 * workers that take a step must not share params, buffers or momentum storage with each other or with the global
 * vectors (BLS_EINVAL).  flags: 0 or a sum of BLS_ROUND_* values. */
enum {
    BLS_ROUND_UNIFORM_WEIGHTS = 1, /* aggregate with the balanced average (1/m) sum_i x^i of Section 4.3 over the m workers
                                      that took part instead of Eq. 4: the setting without the aggregation bias of the
                                      appendix's feature-wise evaluation */
    BLS_ROUND_SEQUENTIAL = 2       /* run the workers one after the other even where the library could run them side by side
                                      in one launch per layer (one scratch slot instead of one per worker; same results) */
};
int communication_round(bls_ctx* ctx, const bls_model* model, float* global_params, float* global_buffers,
                        const bls_worker* workers, int P, const void* x_pool, const int32_t* y_pool, int64_t N, int64_t batch,
                        const bls_sgd* opt, float* loss_table, int flags);

/* ---- epoch sampler (Section 4.2; sampling steps at the top of every epoch of Algorithm 1) ------- */

/* Sizes of one epoch's allocation.  N_F = floor(N tau_F P_F / (tau_F P_F + tau_S P_S)) samples go to the
 * fast workers, the first k = floor(lambda N_F) of them by loss; N_S = N - N_F go to the slow workers.
 * Host only.  0 <= N < 2^31, 1 <= tau_F <= 2^20, 0 <= tau_S <= 2^20, 1 <= P_F <= 1024, 0 <= P_S <= 1024,
 * 0 < lambda <= 1; outputs may be NULL. */
int bls_epoch_allocation(int64_t N, int64_t tau_f, int P_f, int64_t tau_s, int P_s, double lambda, int64_t* n_fast,
                         int64_t* k_high, int64_t* n_slow);
/* n ranked items dealt round-robin to P workers (worker p receives ranks p, p + P, ...): worker p's
 * items sit at [offset, offset + count) of the worker-major output of sample_epoch.  Host only. */
int bls_worker_share(int64_t n, int P, int p, int64_t* offset, int64_t* count);

/* One epoch's sample assignment.
 *   losses  device float[N]: current loss of every sample
 *   u_fast, u_slow device float[N]: one finite random key per sample and per group, drawn by the caller
 *           (uniform, independent); u_fast may be NULL when lambda selects everything by loss
 *   fast_idx_out device int32[N_F], slow_idx_out device int32[N_S] (sizes from bls_epoch_allocation),
 *           worker-major: the segment of worker p is given by bls_worker_share
 * Fast workers: the k highest losses in rank order (as topk_by_loss), then the N_F - k samples with the
 * largest u_fast among those not yet selected (uniform without replacement); equal keys rank by lower
 * index.  Slow workers: the N_S samples with the largest u_slow among all N, independent of the fast
 * draw.  Both lists are dealt round-robin by rank.  N == 0 is a no-op. */
int sample_epoch(bls_ctx* ctx, const float* losses, const float* u_fast, const float* u_slow, int64_t N, int64_t tau_f,
                 int P_f, int64_t tau_s, int P_s, double lambda, int32_t* fast_idx_out, int32_t* slow_idx_out);

/* The sampling schemes compared in the appendix (sampling-scheme comparison and its table of data-allocation rows).
 *   scheme        BLS_SAMPLING_SEPARATED: as sample_epoch.  BLS_SAMPLING_UNIFIED: the group that samples by loss goes
 *                 first and the other group trains on the remaining data: it receives exactly the samples the first
 *                 group did not take (N - N_F resp. N - N_S of them), in descending order of its own keys.
 *   high_loss_to  BLS_HIGH_LOSS_TO_FAST: as sample_epoch.  BLS_HIGH_LOSS_TO_SLOW: the slow workers receive the
 *                 floor(lambda N_S) highest losses and a uniform fill from the rest (keys u_slow); the fast workers draw
 *                 uniformly by u_fast, from all N or, unified, from what the slow workers left.
 *                 BLS_HIGH_LOSS_TO_NONE: nobody samples by loss (the unbiased column of that table; the settings of the
 *                 feature-wise evaluation without the sampling bias): the fast workers draw their N_F samples uniformly
 *                 by u_fast, the slow workers their N_S by u_slow from all N or, unified, from what the fast workers
 *                 left; losses may be NULL and lambda only has to be valid.
 * Sizes, layout of the outputs, ties and errors as for sample_epoch, which is the (SEPARATED, TO_FAST) case.  Keys are
 * finite; a key of -inf is treated as the lowest finite float (a sample already drawn is never drawn again). */
enum { BLS_SAMPLING_SEPARATED = 0, BLS_SAMPLING_UNIFIED = 1 };
enum { BLS_HIGH_LOSS_TO_FAST = 0, BLS_HIGH_LOSS_TO_SLOW = 1, BLS_HIGH_LOSS_TO_NONE = 2 };
int sample_epoch_variant(bls_ctx* ctx, const float* losses, const float* u_fast, const float* u_slow, int64_t N, int64_t tau_f,
                         int P_f, int64_t tau_s, int P_s, double lambda, int scheme, int high_loss_to, int32_t* fast_idx_out,
                         int32_t* slow_idx_out);

/* ---- the outer loop of Algorithm 1 on one GPU: E epochs of sampling and communication rounds ---------------------- */

/* Settings of a run (the inputs of Algorithm 1 and the optimiser settings of Appendix A.1).
 *   epochs      E >= 0
 *   tau_f, P_f, tau_s, P_s, lambda, scheme, high_loss_to   as for sample_epoch_variant; the P_f fast workers come first
 *   round_flags as for communication_round
 *   batch       mini-batch size B
 *   opt         opt.lr is the initial learning rate; momentum and weight decay are constant
 *   milestones  host array of n_milestones epoch numbers (counted from 0); during epoch t the learning rate is
 *               opt.lr * lr_gamma^(number of milestones <= t)  (the MultiStepLR schedule named in Appendix A.1) */
typedef struct {
    int64_t epochs;
    int64_t tau_f;
    int64_t tau_s;
    int32_t P_f;
    int32_t P_s;
    double lambda;
    int32_t scheme;
    int32_t high_loss_to;
    int32_t round_flags;
    int32_t n_milestones;
    int64_t batch;
    bls_sgd opt;
    float lr_gamma;
    const int64_t* milestones;
} bls_epoch_plan;

/* Runs the epochs: at the top of epoch t the sampler assigns the fast and the slow workers their samples from the current
 * loss table and the keys u_fast[t], u_slow[t]; round r then hands worker i the next tau_i * B samples of its share, the
 * workers with a non-empty hand run communication_round (a shorter last hand still takes tau_i steps, its batches wrap
 * around the hand; a worker whose share is used up sits the round out), and the epoch ends when every share is consumed.
 *   global_params, global_buffers  device, in/out: the global model
 *   worker_params  device float[P, d], worker_buffers device float[P, num_buffers] (NULL without buffers): replica storage
 *   worker_momentum device float[P, d], in/out: every worker keeps its optimiser state across rounds and epochs
 *   u_fast, u_slow device float[E, N]: the random keys of every epoch (finite; drawn by the caller)
 *   loss_table     device float[N], in/out: the loss the sampler ranks (fill it before the first epoch, e.g. with
 *                  score_losses); processed samples get their recorded loss
 *   idx_work       device int32[N]: holds the epoch's assignment while its rounds run
 *   rounds_out     host, may be NULL: number of communication rounds that were run
 * P = P_f + P_s <= 64.  Everything is enqueued on the context's stream; errors as for the calls it is made of. */
int train_epochs(bls_ctx* ctx, const bls_model* model, const bls_epoch_plan* plan, float* global_params, float* global_buffers,
                 float* worker_params, float* worker_buffers, float* worker_momentum, const void* x_pool, const int32_t* y_pool,
                 int64_t N, const float* u_fast, const float* u_slow, float* loss_table, int32_t* idx_work, int64_t* rounds_out);

/* Largest magnitude one tile may add to a forward statistic (sum or sum of squares of a tile of a convolution output),
 * to a batch-norm backward sum, and one workgroup to a weight-gradient sum (see the conventions at the top); any pointer
 * may be NULL.  Host only. */
int bls_sum_limits(double* forward_partial, double* backward_partial, double* weight_gradient_partial);

/* w_i = tau_i / sum_j tau_j (Eq. 4), computed in double and rounded once.  Host only. */
int bls_weights_from_tau(const int64_t* tau, int P, float* weights_out);

#ifdef __cplusplus
}
#endif
#endif /* BLS_H */
