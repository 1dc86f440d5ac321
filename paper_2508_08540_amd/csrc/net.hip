// Network passes: scoring (inference-mode forward + per-sample loss) and the local SGD steps
// (train-mode forward, backward, update) for the MLP and the CIFAR residual network.
#include "net.h"
#include <utility>

#include "kernels.h"

// Runs `call` with a KernelTiming* named kt that is non-null while profiling is on.
#define PROF_KERNEL(ctx, cls, call)                                   \
    do {                                                              \
        ProfKernel pk_(ctx, cls);                                     \
        KernelTiming kt_{pk_.span.start, pk_.span.stop};              \
        const KernelTiming* kt = pk_.on ? &kt_ : nullptr;             \
        call;                                                         \
    } while (0)

#define PROF(ctx, cls, call) \
    do {                     \
        ProfScope prof_(ctx, cls); \
        call;                \
    } while (0)

namespace {

constexpr int PAD_C = 16;       // the stem's input is zero-padded to 16 channels so it runs on the same kernels
constexpr int SCORE_CHUNK = 2048;
constexpr int FUSED_BWD_MIN_C = 16;   // channel count from which the batch-norm backward rides in the input gradient's staging
constexpr int MLP_SPLITS = 8;

int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }

ConvShape shape_of(const ConvBn& l, int B) {
    ConvShape cs;
    cs.B = B; cs.h_in = l.h_in; cs.c_out = l.c_out; cs.stride = l.stride;
    cs.c_in = l.c_in < PAD_C ? PAD_C : l.c_in;
    cs.c_in_real = l.c_in;
    return cs;
}

int64_t out_elems(const ConvBn& l, int B) { return (int64_t)B * l.h_out * l.h_out * l.c_out; }

typedef uint8_t act_t;  // activations are addressed as bytes; the model's storage type gives the element size

// ---- MLP ----------------------------------------------------------------------------------------

struct MlpScratch {
    float *xb, *h, *part, *loss, *dlogits, *dpre, *grad;
    int32_t* yb;
};

MlpScratch carve_mlp(Carver& c, const bls_model* m, int B, bool train) {
    MlpScratch s{};
    const int hid = m->desc.hidden;
    s.h = c.take<float>((size_t)B * hid);
    s.part = c.take<float>(max64(gemm_partial_floats(B, hid, MLP_SPLITS), train ? gemm_partial_floats(hid, m->d_in, 1) : 0));
    s.loss = c.take<float>(B);
    if (train) {
        s.xb = c.take<float>((size_t)B * m->d_in);
        s.yb = c.take<int32_t>(B);
        s.dlogits = c.take<float>((size_t)B * m->desc.classes);
        s.dpre = c.take<float>((size_t)B * hid);
        s.grad = c.take<float>(m->num_params);
    }
    return s;
}

void mlp_hidden(bls_ctx* ctx, hipStream_t st, const bls_model* m, const float* params, const float* x, int B, const MlpScratch& s) {
    PROF(ctx, PROF_GEMM, launch_gemm(st, x, m->d_in, false, params + m->fc1_w, m->d_in, false, B, m->desc.hidden, m->d_in, MLP_SPLITS, s.part,
                s.h, params + m->fc1_b, true, nullptr));
}

// ---- residual network ---------------------------------------------------------------------------------

struct ResScratch {
    Reps reps;                         // replicas that every launch covers (one, or the workers of a batched round)
    int act;                           // storage type of activations and packed weights
    act_t* wpack;                      // packed weights: forward copies of all layers, then input-gradient copies
    std::vector<int64_t> fwd_off, dgrad_off;  // byte offsets into wpack per layer
    PackTable tab;
    act_t* xpad;
    int32_t* yb;
    act_t* xpad_next;                  // training: the batch of the next step, gathered on the side stream meanwhile
    int32_t* yb_next;
    std::vector<act_t*> y, a, dy;      // per layer
    std::vector<float*> mean, invstd;  // per layer
    act_t *stats, *d1, *d2, *g;
    float* grad;
    fixsum_t* wacc;  // weight-gradient accumulators of all layers (kept zero between uses)
    int64_t wacc_count;
    UpdateTable utab;  // per layer: where its weights, accumulators and packed copies are
    fixsum_t* sums;  // per layer: a forward and a backward set of fixed-point accumulators, zeroed every step
    float *loss, *feat, *dlogits, *dfeat;
};

ResScratch carve_resnet(Carver& c, const bls_model* m, int B, bool train) {
    ResScratch s{};
    const int L = (int)m->layers.size();
    const int hw = m->desc.image_hw;
    s.act = m->desc.act_dtype == BLS_ACT_BF16 ? ACT_BF16 : ACT_F32;
    const size_t esz = act_bytes(s.act);
    s.fwd_off.assign(L, 0);
    s.dgrad_off.assign(L, 0);
    s.tab.n = 0;
    int64_t vec4 = 0;
    for (int pass = 0; pass < (train ? 2 : 1); ++pass)
        for (int l = (pass == 0 ? 0 : 1); l < L; ++l) {
            const ConvBn& cb = m->layers[l];
            PackEntry& e = s.tab.e[s.tab.n++];
            e.w_off = cb.w_off;
            e.pack_off = vec4;
            e.c_in = cb.c_in < PAD_C ? PAD_C : cb.c_in;
            e.c_out = cb.c_out;
            e.c_in_real = cb.c_in;
            e.dgrad = pass;
            e.taps = 9; e.pad_ = 0;
            (pass == 0 ? s.fwd_off : s.dgrad_off)[l] = vec4 * 4 * (int64_t)esz;
            vec4 += (int64_t)e.c_in * e.c_out * 9 / 4;
        }
    s.tab.total_vec4 = vec4;
    s.wpack = c.take<act_t>(vec4 * 4 * esz);
    s.xpad = c.take<act_t>((size_t)B * hw * hw * PAD_C * esz);
    s.yb = c.take<int32_t>(B);
    if (train) {
        s.xpad_next = c.take<act_t>((size_t)B * hw * hw * PAD_C * esz);
        s.yb_next = c.take<int32_t>(B);
    }
    s.loss = c.take<float>(B);
    s.y.resize(L); s.a.resize(L); s.mean.resize(L); s.invstd.resize(L); s.dy.assign(L, nullptr);
    int64_t max_act = 0, max_wpart = 0;
    s.utab.n = 0;
    for (int l = 0; l < L; ++l) {
        const ConvBn& cb = m->layers[l];
        ConvShape cs = shape_of(cb, B);
        max_act = max64(max_act, out_elems(cb, B));
        {
            UpdateEntry& ue = s.utab.e[s.utab.n++];
            ue.w_off = cb.w_off; ue.n = (int64_t)cs.c_out * 9 * cs.c_in_real; ue.acc_off = max_wpart;
            ue.fwd_quad = s.fwd_off[l] / (4 * (int64_t)esz);
            ue.dgrad_quad = (train && l > 0) ? s.dgrad_off[l] / (4 * (int64_t)esz) : -1;
            ue.c_in = cs.c_in; ue.c_out = cs.c_out; ue.c_in_real = cs.c_in_real; ue.taps = 9;
            ue.replicas = conv_wgrad_replicas(s.act, cs); ue.pad_ = 0;
            max_wpart += conv_wgrad_accumulators(s.act, cs);
        }
        s.mean[l] = c.take<float>(cb.c_out);
        s.invstd[l] = c.take<float>(cb.c_out);
    }
    if (train) {
        for (int l = 0; l < L; ++l) {
            s.y[l] = c.take<act_t>(out_elems(m->layers[l], B) * esz);
            s.a[l] = c.take<act_t>(out_elems(m->layers[l], B) * esz);
            s.dy[l] = c.take<act_t>(out_elems(m->layers[l], B) * esz);  // kept per layer: the side stream reads it later
        }
        s.stats = nullptr;
        s.sums = c.take<fixsum_t>((size_t)L * 2 * FIX_SET);
        s.d1 = c.take<act_t>(max_act * esz);
        s.d2 = c.take<act_t>(max_act * esz);
        s.g = c.take<act_t>(max_act * esz);
        s.wacc = c.take<fixsum_t>(max_wpart);
        s.wacc_count = max_wpart;
        s.grad = c.take<float>(m->num_params);
        s.feat = c.take<float>((size_t)B * m->final_c);
        s.dlogits = c.take<float>((size_t)B * m->desc.classes);
        s.dfeat = c.take<float>((size_t)B * m->final_c);
    } else {
        // inference keeps no activations: four rotating buffers are enough
        act_t* pool[4];
        for (act_t*& p : pool) p = c.take<act_t>(max_act * esz);
        for (int l = 0; l < L; ++l) {
            // layer l writes y into pool[(2l) % 4 .. ]: see resnet_forward for the rotation
            s.y[l] = nullptr;
            s.a[l] = nullptr;
        }
        s.d1 = pool[0]; s.d2 = pool[1]; s.g = pool[2]; s.stats = pool[3];
        s.sums = nullptr;
    }
    return s;
}

// Forward pass over a batch already gathered into s.xpad.  Train mode keeps every layer's
// convolution output and activation for the backward pass and updates the running statistics.
// Returns the final activation.
// `prepare`: build the packed weight copies from the parameters and clear the batch-norm accumulators first (the update
// at the end of a local step leaves both ready for the next step).
const act_t* resnet_forward(bls_ctx* ctx, hipStream_t st, const bls_model* m, const float* params, float* buffers, int B, ResScratch& s,
                            bool train, bool prepare) {
    const int L = (int)m->layers.size();
    act_t* rot[4] = {s.d1, s.d2, s.g, s.stats};  // inference-only rotation
    int next = 0;
    auto take = [&](const act_t* keep0, const act_t* keep1) {
        for (;;) {
            act_t* p = rot[next];
            next = (next + 1) & 3;
            if (p != keep0 && p != keep1) return p;
        }
    };
    if (prepare) {
        PROF(ctx, PROF_UPDATE, launch_pack_weights(st, s.act, params, s.wpack, s.tab, s.reps));
        if (train) PROF(ctx, PROF_UPDATE, launch_fill_zero(st, reinterpret_cast<float*>(s.sums), (int64_t)m->layers.size() * 2 * FIX_SET * 2, s.reps));
    }
    const act_t* block_in = nullptr;
    const act_t* cur = s.xpad;
    // Training: the batch norm + ReLU of a layer without a shortcut (the stem and the first convolution of every block)
    // is applied by the next convolution while it stages its input, which also stores the activation for the backward
    // pass; `pending` is that layer, whose raw convolution output the next launch reads.
    int pending = -1;
    const act_t* pending_res = nullptr;   // shortcut that goes with it (the end of a block), or nullptr; its channels and stride
    int pending_res_c = 0, pending_res_stride = 1;
    for (int l = 0; l < L; ++l) {
        const ConvBn& cb = m->layers[l];
        ConvShape cs = shape_of(cb, B);
        const bool is_conv2 = l > 0 && (l % 2 == 0);
        if (l > 0 && !is_conv2) block_in = cur;
        act_t* y = train ? s.y[l] : take(cur, block_in);
        const int64_t pixels = (int64_t)B * cb.h_out * cb.h_out;
        if (train) {
            // the convolution accumulates the sums of its output; bn_apply turns them into statistics
            ConvEpi e{};
            e.sums = s.sums + (size_t)l * 2 * FIX_SET;
            e.scale = FIX_FWD_SCALE;
            const act_t* x_in = cur;
            if (pending >= 0) {
                const ConvBn& pb = m->layers[pending];
                e.in_sums = s.sums + (size_t)pending * 2 * FIX_SET;
                e.in_count = (double)((int64_t)B * pb.h_out * pb.h_out);
                e.in_mean = s.mean[pending]; e.in_invstd = s.invstd[pending];
                e.in_rmean = buffers + pb.rmean_off; e.in_rvar = buffers + pb.rvar_off;
                e.in_gamma = params + pb.gamma_off; e.in_beta = params + pb.beta_off;
                e.in_res = pending_res;
                e.in_res_c = pending_res_c; e.in_res_lo = (pb.c_out - pending_res_c) / 2; e.in_res_stride = pending_res_stride;
                e.a_out = s.a[pending];
                x_in = s.y[pending];
                pending = -1;
            }
            PROF_KERNEL(ctx, PROF_CONV_FWD, launch_conv_fwd(st, s.act, cs, x_in, s.wpack + s.fwd_off[l], y, &e, kt, s.reps));
        } else {
            // inference: one kernel per layer, batch norm (running statistics), shortcut and ReLU in the epilogue
            ConvEpi e{};
            e.mean_prev = buffers + cb.rmean_off; e.invstd_prev = buffers + cb.rvar_off;
            e.gamma = params + cb.gamma_off; e.beta = params + cb.beta_off;
            if (is_conv2) {
                const ConvBn& c1 = m->layers[l - 1];
                e.sc_g = block_in; e.sc_c = c1.c_in; e.sc_lo = (cb.c_out - c1.c_in) / 2; e.sc_stride = c1.stride;
            }
            PROF_KERNEL(ctx, PROF_CONV_FWD, launch_conv_fwd(st, s.act, cs, cur, s.wpack + s.fwd_off[l], y, &e, kt));
            cur = y;
            continue;
        }
        // the next convolution can normalise on load (adding the block's shortcut, identity or subsampled and zero-padded)
        // when it reads all of this layer's channels
        if (l + 1 < L && m->layers[l + 1].c_in == cb.c_out && cb.c_out <= 64) {
            pending = l;      // the next convolution writes s.a[l]
            pending_res = is_conv2 ? block_in : nullptr;
            pending_res_c = is_conv2 ? m->layers[l - 1].c_in : 0;
            pending_res_stride = is_conv2 ? m->layers[l - 1].stride : 1;
            cur = s.a[l];
            continue;
        }
        BnStats bs{};
        bs.sums = s.sums + (size_t)l * 2 * FIX_SET;
        bs.count = (double)pixels;
        bs.mean = s.mean[l]; bs.invstd = s.invstd[l];
        bs.running_mean = buffers + cb.rmean_off; bs.running_var = buffers + cb.rvar_off;
        act_t* a = train ? s.a[l] : take(y, block_in);
        const act_t* res = nullptr;
        int c_res = cb.c_out, res_stride = 1;
        if (is_conv2) {
            const ConvBn& c1 = m->layers[l - 1];
            res = block_in;
            c_res = c1.c_in;
            res_stride = c1.stride;
        }
        PROF(ctx, PROF_NORM, launch_bn_apply(st, s.act, y, pixels, cb.c_out, bs, params + cb.gamma_off, params + cb.beta_off, res,
                        c_res, res_stride, cb.h_out, a, s.reps));
        cur = a;
    }
    return cur;
}

// The weight gradients are off the critical path (only the update needs them), so they run on the
// context's side stream, each after the event that marks its dy as ready; the caller joins the side
// stream before the update.
// `early_from`: the caller updates the parameters of layers early_from .. L-1 (and everything behind the last layer) as soon
// as their weight gradients are in, while those of the layers below still run; the events that mark the two moments are
// fork_events[L] / [L + 1] (one per side stream) and the join events.
int resnet_backward(bls_ctx* ctx, hipStream_t st, const bls_model* m, const float* params, int B, ResScratch& s, int early_from) {
    const int L = (int)m->layers.size();
    while ((int)ctx->fork_events.size() < L + 2) {
        hipEvent_t e;
        BLS_HIP(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
        ctx->fork_events.push_back(e);
    }
    // the second side stream exists only where it is used: idle streams still take part in the mapping of streams to
    // hardware queues and cost concurrent workers (lanes) 15 % of their throughput
    const bool two_sides = s.act == ACT_BF16;
    if (two_sides && !ctx->aux2) BLS_HIP(ctx, hipStreamCreateWithFlags(&ctx->aux2, hipStreamNonBlocking));
    const ConvBn& last = m->layers[L - 1];
    const void* dout = s.dfeat;
    int shared = last.h_out * last.h_out;
    // Every input-gradient launch stores the gradient behind the ReLU of the layer below (zero where that activation is).
    // The one a block's second convolution receives is also the gradient of the block's shortcut: `block_g` keeps it until
    // the input-gradient launch of the block's first convolution has added it, so the three tensors rotate.
    act_t* const ring[3] = {s.d1, s.d2, s.g};
    const void* block_g = nullptr;
    for (int l = L - 1; l >= 0; --l) {
        const ConvBn& cb = m->layers[l];
        ConvShape cs = shape_of(cb, B);
        const int64_t pixels = (int64_t)B * cb.h_out * cb.h_out;
        const bool is_conv2 = l > 0 && (l % 2 == 0);
        const act_t* x_in = l == 0 ? s.xpad : s.a[l - 1];
        if (l == L - 1) {
            // top layer: its upstream gradient comes from the head; lower layers get these sums from the
            // input-gradient kernel of the layer above
            PROF(ctx, PROF_NORM, launch_bn_bwd_reduce(st, s.act, dout, shared, s.a[l], s.y[l], pixels, cb.c_out, s.mean[l], s.invstd[l],
                                                      s.sums + ((size_t)l * 2 + 1) * FIX_SET, s.reps));
        }
        // Layers whose upstream gradient is a tensor (all but the top one): the input-gradient convolution computes dy itself
        // while staging (for a stride-2 layer at the even positions of the zero-inserted image), the element-wise kernel goes
        const bool fused_bwd = l > 0 && !shared && cb.c_out <= 64 && cb.c_out >= FUSED_BWD_MIN_C;
        auto weight_gradient = [&]() -> int {
            BLS_HIP(ctx, hipEventRecord(ctx->fork_events[l], st));
            // With bf16 storage the main stream's kernels are shorter than the weight gradients (which multiply in fp32), the
            // side stream is the long pole and neighbouring layers' weight gradients alternate between two streams; with
            // fp32 storage a third queue only slows the critical path (measured: +1.7 % per pass).
            hipStream_t side = (two_sides && (l & 1)) ? ctx->aux2 : ctx->aux;
            BLS_HIP(ctx, hipStreamWaitEvent(side, ctx->fork_events[l], 0));
            PROF_KERNEL(ctx, PROF_CONV_WGRAD, launch_conv_wgrad(side, s.act, cs, x_in, s.dy[l], s.wacc + s.utab.e[l].acc_off, kt, s.reps));
            // the last weight gradient of the early part on this stream (two streams take the layers in turn)
            if (l >= early_from && l < early_from + (two_sides ? 2 : 1)) BLS_HIP(ctx, hipEventRecord(ctx->fork_events[L + (side == ctx->aux ? 0 : 1)], side));
            return BLS_OK;
        };
        if (is_conv2 && !shared) block_g = dout;   // as stored by the launch of the layer above
        if (!fused_bwd) {
            // the head's gradient is one row per sample: the element-wise kernel leaves the gradient behind the ReLU as a tensor
            act_t* g_out = (is_conv2 && shared) ? s.g : nullptr;
            PROF(ctx, PROF_NORM, launch_bn_bwd_apply(st, s.act, dout, shared, s.a[l], s.y[l], pixels, cb.c_out, s.mean[l], s.invstd[l], params + cb.gamma_off,
                                s.sums + ((size_t)l * 2 + 1) * FIX_SET, s.grad + cb.gamma_off, s.grad + cb.beta_off, s.dy[l], g_out, nullptr, s.reps));
            if (g_out) block_g = g_out;
            int rcw = weight_gradient();
            if (rcw != BLS_OK) return rcw;
        }
        if (l == 0) break;
        act_t* dx = nullptr;   // neither the tensor the fused staging reads nor the shortcut gradient still to be added
        for (act_t* cand : ring)
            if (cand != dout && cand != block_g) dx = cand;
        {
            // input gradient; its epilogue adds the shortcut gradient (conv1 of a block) and reduces the
            // batch-norm backward sums of layer l-1
            ConvEpi e{};
            e.sums = s.sums + ((size_t)(l - 1) * 2 + 1) * FIX_SET;
            e.scale = FIX_BWD_SCALE;
            e.a_prev = s.a[l - 1]; e.y_prev = s.y[l - 1]; e.mean_prev = s.mean[l - 1]; e.invstd_prev = s.invstd[l - 1];
            if (!is_conv2) {
                const ConvBn& c2 = m->layers[l + 1];
                e.sc_g = block_g; e.sc_c = c2.c_out; e.sc_lo = (c2.c_out - cb.c_in) / 2; e.sc_stride = cb.stride;
            }
            if (fused_bwd) {
                e.bw_dout = dout; e.bw_y = s.y[l];
                e.bw_mean = s.mean[l]; e.bw_invstd = s.invstd[l]; e.bw_gamma = params + cb.gamma_off;
                e.bw_sums = s.sums + ((size_t)l * 2 + 1) * FIX_SET;
                e.bw_dgamma = s.grad + cb.gamma_off; e.bw_dbeta = s.grad + cb.beta_off;
                e.bw_inv_count = 1.f / (float)pixels;
                e.bw_dy_out = s.dy[l];
            }
            PROF_KERNEL(ctx, PROF_CONV_DGRAD, launch_conv_dgrad(st, s.act, cs, s.dy[l], s.wpack + s.dgrad_off[l], dx, &e, kt, s.reps));
        }
        if (fused_bwd) {
            int rcw = weight_gradient();   // dy[l] exists once the input gradient has run
            if (rcw != BLS_OK) return rcw;
        }
        if (!is_conv2) block_g = nullptr;   // added by this launch
        dout = dx;
        shared = 0;
    }
    BLS_HIP(ctx, hipEventRecord(ctx->join_event, ctx->aux));
    if (two_sides) BLS_HIP(ctx, hipEventRecord(ctx->join_event2, ctx->aux2));
    return BLS_OK;
}

// One training step on the batch already gathered into s.xpad / s.yb: forward, head, backward, update.  All launches cover
// s.reps replicas (params, buffers, momentum, loss and the scratch are replica 0's).
int resnet_train_step(bls_ctx* ctx, hipStream_t st, const bls_model* m, float* params, float* buffers, float* momentum, int B, ResScratch& s,
                      float* loss, const bls_sgd& opt, bool first) {
    const int C = m->desc.classes;
    const float inv_b = 1.f / (float)B;
    const act_t* fin = resnet_forward(ctx, st, m, params, buffers, B, s, true, first);
    PROF(ctx, PROF_HEAD, launch_head_forward(st, s.act, fin, B, m->final_hw * m->final_hw, m->final_c, params + m->fc_w, params + m->fc_b, C, s.yb,
                        loss, s.feat, s.dlogits, s.dfeat, inv_b, false, s.reps));
    // the head's weight gradient is only needed by the update: side stream, joined at the end of the backward pass
    BLS_HIP(ctx, hipEventRecord(ctx->head_event, st));
    BLS_HIP(ctx, hipStreamWaitEvent(ctx->aux, ctx->head_event, 0));
    {
        ProfScope prof_(ctx, PROF_HEAD, ctx->aux);
        launch_head_wgrad(ctx->aux, s.dlogits, s.feat, B, C, m->final_c, s.grad + m->fc_w, s.grad + m->fc_b, s.reps);
    }
    // The update comes in two launches: the layers from `early` up (nearly all parameters) as soon as their weight gradients
    // are in, behind which the side stream still works on the weight gradients of the first layers; those layers, and the
    // clearing of the batch-norm accumulators, after the join.
    const int L = (int)m->layers.size();
    const int early = L > 3 ? 3 : L;
    const bool two_sides = s.act == ACT_BF16;
    int rc = resnet_backward(ctx, st, m, params, B, s, early);
    if (rc != BLS_OK) return rc;
    const int64_t split = early < L ? m->layers[early].w_off : m->layers[L - 1].beta_off + m->layers[L - 1].c_out;
    // gradients of the convolution weights are still in the accumulators: the update reads them there
    if (early < L) {
        BLS_HIP(ctx, hipStreamWaitEvent(st, ctx->fork_events[L], 0));
        if (two_sides && early + 1 < L) BLS_HIP(ctx, hipStreamWaitEvent(st, ctx->fork_events[L + 1], 0));
    } else {
        BLS_HIP(ctx, hipStreamWaitEvent(st, ctx->join_event, 0));   // nothing below: the head's weight gradient is all there is to wait for
    }
    PROF(ctx, PROF_UPDATE, launch_update(st, s.act, params, momentum, s.grad, m->num_params, opt.lr, opt.momentum, opt.weight_decay,
                                         s.wacc, s.wpack, s.utab, nullptr, 0, s.reps, split, -1));
    BLS_HIP(ctx, hipStreamWaitEvent(st, ctx->join_event, 0));
    if (two_sides) BLS_HIP(ctx, hipStreamWaitEvent(st, ctx->join_event2, 0));
    PROF(ctx, PROF_UPDATE, launch_update(st, s.act, params, momentum, s.grad, m->num_params, opt.lr, opt.momentum, opt.weight_decay,
                                         s.wacc, s.wpack, s.utab, s.sums, (int64_t)L * 2 * FIX_SET, s.reps, 0, split));
    return BLS_OK;
}

// ---- the workers of a communication round side by side ----------------------------------------------------------------
// Worker r lives in slot r of the arena: its parameters, running statistics, momentum, recorded losses and the whole
// training scratch, every slot laid out alike, so that one launch per layer covers all workers (Reps).
struct SlotHead {
    float *params, *buffers, *momentum, *losses;
};

SlotHead carve_slot_head(Carver& c, const bls_model* m, int B, int64_t tau_max) {
    SlotHead h{};
    h.params = c.take<float>(m->num_params);
    h.buffers = c.take<float>(m->num_buffers > 0 ? m->num_buffers : 1);
    h.momentum = c.take<float>(m->num_params);
    h.losses = c.take<float>((size_t)tau_max * B);
    return h;
}

#define ROUND_MAX_REPS 64
struct RoundIO {   // the workers' own storage, by slot
    float* params[ROUND_MAX_REPS];
    float* buffers[ROUND_MAX_REPS];
    float* momentum[ROUND_MAX_REPS];
    float* losses[ROUND_MAX_REPS];     // where the recorded losses of the slot go (or nullptr)
    int64_t n_losses[ROUND_MAX_REPS];
};

// Start of a round: every slot takes the global model and its worker's momentum.
__global__ __launch_bounds__(256) void round_copy_in_kernel(const float* __restrict__ gparams, const float* __restrict__ gbuffers, RoundIO io,
                                                            SlotHead h, int64_t d, int64_t nb, int64_t rstride) {
    const int r = blockIdx.z;
    const int64_t ro = (int64_t)r * rstride;
    float *sp = rep_at(h.params, ro), *sb = rep_at(h.buffers, ro), *sm = rep_at(h.momentum, ro);
    const float* wm = io.momentum[r];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x, first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = first; i < d; i += stride) {
        sp[i] = gparams[i];
        sm[i] = wm[i];
    }
    for (int64_t i = first; i < nb; i += stride) sb[i] = gbuffers[i];
}

// End of a round: the trained replica, its running statistics, momentum and recorded losses go to the worker's storage.
__global__ __launch_bounds__(256) void round_copy_out_kernel(RoundIO io, SlotHead h, int64_t d, int64_t nb, int64_t rstride) {
    const int r = blockIdx.z;
    const int64_t ro = (int64_t)r * rstride;
    const float *sp = rep_at(h.params, ro), *sb = rep_at(h.buffers, ro), *sm = rep_at(h.momentum, ro), *sl = rep_at(h.losses, ro);
    float *wp = io.params[r], *wb = io.buffers[r], *wm = io.momentum[r], *wl = io.losses[r];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x, first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = first; i < d; i += stride) {
        wp[i] = sp[i];
        wm[i] = sm[i];
    }
    if (wb)
        for (int64_t i = first; i < nb; i += stride) wb[i] = sb[i];
    if (wl)
        for (int64_t i = first; i < io.n_losses[r]; i += stride) wl[i] = sl[i];
}

size_t round_slot_bytes(const bls_model* m, int B, int64_t tau_max) {
    Carver c(nullptr);
    carve_slot_head(c, m, B, tau_max);
    carve_resnet(c, m, B, true);
    return (c.off + 255) & ~size_t(255);
}

size_t scratch_bytes(const bls_model* m, int B, bool train) {
    Carver c(nullptr);
    if (m->desc.kind == BLS_MODEL_MLP) carve_mlp(c, m, B, train);
    else carve_resnet(c, m, B, train);
    return c.off;
}

}  // namespace

size_t net_workspace_bytes(const bls_model* m, int64_t n, bool train) {
    return scratch_bytes(m, (int)(train || n < SCORE_CHUNK ? n : SCORE_CHUNK), train);
}

int net_score(bls_ctx* ctx, const bls_model* m, const float* params, const float* buffers, const float* x,
              const int32_t* y, int64_t N, float* losses_out) {
    const int chunk = (int)(N < SCORE_CHUNK ? N : SCORE_CHUNK);
    int rc = bls_arena_reserve(ctx, scratch_bytes(m, chunk, false));
    if (rc != BLS_OK) return rc;
    hipStream_t st = ctx->stream;
    Carver c(ctx->arena);
    if (m->desc.kind == BLS_MODEL_MLP) {
        MlpScratch s = carve_mlp(c, m, chunk, false);
        for (int64_t first = 0; first < N; first += chunk) {
            int B = (int)(N - first < chunk ? N - first : chunk);
            mlp_hidden(ctx, st, m, params, x + first * m->d_in, B, s);
            PROF(ctx, PROF_HEAD, launch_head_forward(st, ACT_F32, s.h, B, 1, m->desc.hidden, params + m->fc2_w, params + m->fc2_b, m->desc.classes,
                                y + first, losses_out + first, nullptr, nullptr, nullptr, 0.f, false));
        }
    } else {
        ResScratch s = carve_resnet(c, m, chunk, false);
        const int hw = m->desc.image_hw;
        for (int64_t first = 0; first < N; first += chunk) {
            int B = (int)(N - first < chunk ? N - first : chunk);
            PROF(ctx, PROF_GATHER, launch_gather_images(st, x, y, nullptr, 1, 0, first, B, hw * hw, m->desc.in_channels, PAD_C, s.act, s.xpad, s.yb));
            const act_t* fin = resnet_forward(ctx, st, m, params, const_cast<float*>(buffers), B, s, false, first == 0);
            PROF(ctx, PROF_HEAD, launch_head_forward(st, s.act, fin, B, m->final_hw * m->final_hw, m->final_c, params + m->fc_w, params + m->fc_b,
                                m->desc.classes, s.yb, losses_out + first, nullptr, nullptr, nullptr, 0.f, false));
        }
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

int net_local_step(bls_ctx* ctx, const bls_model* m, float* params, float* buffers, float* momentum, const float* x_pool,
                   const int32_t* y_pool, int64_t N, const int32_t* sel, int64_t k, int64_t batch, int64_t tau,
                   const bls_sgd& opt, float* step_losses_out) {
    (void)N;
    const int B = (int)batch;
    int rc = bls_arena_reserve(ctx, scratch_bytes(m, B, true));
    if (rc != BLS_OK) return rc;
    hipStream_t st = ctx->stream;
    Carver c(ctx->arena);
    if (m->desc.kind == BLS_MODEL_MLP) {
        const float inv_b = 1.f / (float)B;
        MlpScratch s = carve_mlp(c, m, B, true);
        const int hid = m->desc.hidden, C = m->desc.classes;
        for (int64_t j = 0; j < tau; ++j) {
            float* loss = step_losses_out ? step_losses_out + j * B : s.loss;
            PROF(ctx, PROF_GATHER, launch_gather_rows(st, x_pool, y_pool, sel, k, j * B, B, m->d_in, s.xb, s.yb));
            mlp_hidden(ctx, st, m, params, s.xb, B, s);
            PROF(ctx, PROF_HEAD, launch_head_forward(st, ACT_F32, s.h, B, 1, hid, params + m->fc2_w, params + m->fc2_b, C, s.yb, loss, nullptr, s.dlogits,
                                s.dpre, inv_b, true));
            PROF(ctx, PROF_HEAD, launch_head_wgrad(st, s.dlogits, s.h, B, C, hid, s.grad + m->fc2_w, s.grad + m->fc2_b));
            PROF(ctx, PROF_GEMM, launch_gemm(st, s.dpre, hid, true, s.xb, m->d_in, true, hid, m->d_in, B, 1, s.part, s.grad + m->fc1_w, nullptr,
                        false, nullptr));
            PROF(ctx, PROF_UPDATE, launch_colsum(st, s.dpre, B, hid, s.grad + m->fc1_b));
            PROF(ctx, PROF_UPDATE, launch_sgd(st, params, momentum, s.grad, m->num_params, opt.lr, opt.momentum, opt.weight_decay));
        }
    } else {
        ResScratch s = carve_resnet(c, m, B, true);
        const int hw = m->desc.image_hw;
        // the weight-gradient accumulators start at zero; every reduction leaves them at zero again
        PROF(ctx, PROF_UPDATE, launch_fill_zero(st, reinterpret_cast<float*>(s.wacc), s.wacc_count * 2));
        // The batch of step j + 1 does not depend on step j: it is gathered on the side stream while step j runs, into the
        // other pair of buffers.  That stream is in order and every step joins it before its update, so the gather follows
        // the last reader of its buffers (the stem's weight gradient of step j - 1) and precedes the first of step j + 1.
        PROF(ctx, PROF_GATHER, launch_gather_images(st, x_pool, y_pool, sel, k, 0, 0, B, hw * hw, m->desc.in_channels, PAD_C, s.act, s.xpad, s.yb));
        for (int64_t j = 0; j < tau; ++j) {
            float* loss = step_losses_out ? step_losses_out + j * B : s.loss;
            if (j + 1 < tau) {
                if (j == 0) {   // the side stream has not seen this call's work yet: behind the first gather, whose launch is the latest so far
                    BLS_HIP(ctx, hipEventRecord(ctx->head_event, st));
                    BLS_HIP(ctx, hipStreamWaitEvent(ctx->aux, ctx->head_event, 0));
                }
                ProfScope prof_(ctx, PROF_GATHER, ctx->aux);
                launch_gather_images(ctx->aux, x_pool, y_pool, sel, k, (j + 1) * B, 0, B, hw * hw, m->desc.in_channels, PAD_C, s.act, s.xpad_next,
                                     s.yb_next);
            }
            rc = resnet_train_step(ctx, st, m, params, buffers, momentum, B, s, loss, opt, j == 0);
            if (rc != BLS_OK) return rc;
            std::swap(s.xpad, s.xpad_next);
            std::swap(s.yb, s.yb_next);
        }
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

bool net_round_batched_covers(const bls_model* m) { return m->desc.kind == BLS_MODEL_RESNET_CIFAR; }

int net_round_batched(bls_ctx* ctx, const bls_model* m, const float* global_params, const float* global_buffers, const bls_worker* workers, int P,
                      const float* x_pool, const int32_t* y_pool, int64_t batch, const bls_sgd& opt, float* losses_out, const int64_t* loss_off) {
    // slots in order of decreasing step count: the workers still training after step j are then the first R_j slots
    int order[ROUND_MAX_REPS], R = 0;
    for (int i = 0; i < P; ++i)
        if (workers[i].tau > 0) order[R++] = i;
    if (R < 1 || R > ROUND_MAX_REPS) return bls_fail(ctx, BLS_EINVAL, "batched round: %d workers take a step, 1 .. %d supported", R, ROUND_MAX_REPS);
    for (int a = 1; a < R; ++a)   // stable insertion sort by tau, descending
        for (int b = a; b > 0 && workers[order[b]].tau > workers[order[b - 1]].tau; --b) {
            const int t = order[b]; order[b] = order[b - 1]; order[b - 1] = t;
        }
    const int B = (int)batch;
    const int64_t tau_max = workers[order[0]].tau;
    const size_t slot = round_slot_bytes(m, B, tau_max);
    int rc = bls_arena_reserve(ctx, slot * R);
    if (rc != BLS_OK) return rc;
    hipStream_t st = ctx->stream;
    Carver c(ctx->arena);
    SlotHead h = carve_slot_head(c, m, B, tau_max);
    ResScratch s = carve_resnet(c, m, B, true);
    s.reps.n = R;
    s.reps.stride = (int64_t)slot;
    RoundIO io{};
    GatherReps lists{};
    int t_seen = 0;
    for (int i = 0; i < P; ++i) {   // loss_off counts the workers that take a step, in the caller's order
        if (workers[i].tau == 0) continue;
        for (int r = 0; r < R; ++r)
            if (order[r] == i) {
                io.losses[r] = losses_out ? losses_out + loss_off[t_seen] : nullptr;
                io.n_losses[r] = workers[i].tau * batch;
            }
        ++t_seen;
    }
    for (int r = 0; r < R; ++r) {
        const bls_worker& w = workers[order[r]];
        io.params[r] = w.params; io.buffers[r] = w.buffers; io.momentum[r] = w.momentum;
        lists.sel[r] = w.idx; lists.k[r] = w.n_idx;
    }
    const int64_t d = m->num_params, nb = m->num_buffers;
    int64_t blocks = (d + 255) / 256;
    if (blocks > 256) blocks = 256;
    PROF(ctx, PROF_UPDATE, hipLaunchKernelGGL(round_copy_in_kernel, dim3((unsigned)blocks, 1, R), dim3(256), 0, st, global_params, global_buffers, io, h,
                                              d, nb, s.reps.stride));
    // the weight-gradient accumulators start at zero; every update leaves them at zero again
    PROF(ctx, PROF_UPDATE, launch_fill_zero(st, reinterpret_cast<float*>(s.wacc), s.wacc_count * 2, s.reps));
    const int hw = m->desc.image_hw;
    // replicas still training at step j: the first R_j slots
    auto training_at = [&](int64_t j) {
        int rj = 0;
        while (rj < R && workers[order[rj]].tau > j) ++rj;
        return rj;
    };
    // as in net_local_step: the batches of step j + 1 are gathered on the side stream while step j runs
    s.reps.n = training_at(0);
    PROF(ctx, PROF_GATHER, launch_gather_images_reps(st, x_pool, y_pool, lists, 0, B, hw * hw, m->desc.in_channels, PAD_C, s.act, s.xpad, s.yb, s.reps));
    for (int64_t j = 0; j < tau_max; ++j) {
        if (j + 1 < tau_max) {
            if (j == 0) {
                BLS_HIP(ctx, hipEventRecord(ctx->head_event, st));
                BLS_HIP(ctx, hipStreamWaitEvent(ctx->aux, ctx->head_event, 0));
            }
            Reps next = s.reps;
            next.n = training_at(j + 1);
            ProfScope prof_(ctx, PROF_GATHER, ctx->aux);
            launch_gather_images_reps(ctx->aux, x_pool, y_pool, lists, (j + 1) * B, B, hw * hw, m->desc.in_channels, PAD_C, s.act, s.xpad_next,
                                      s.yb_next, next);
        }
        s.reps.n = training_at(j);
        rc = resnet_train_step(ctx, st, m, h.params, h.buffers, h.momentum, B, s, h.losses + j * B, opt, j == 0);
        if (rc != BLS_OK) return rc;
        std::swap(s.xpad, s.xpad_next);
        std::swap(s.yb, s.yb_next);
    }
    s.reps.n = R;
    PROF(ctx, PROF_UPDATE, hipLaunchKernelGGL(round_copy_out_kernel, dim3((unsigned)blocks, 1, R), dim3(256), 0, st, io, h, d, nb, s.reps.stride));
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

void net_release(bls_ctx*) {}
