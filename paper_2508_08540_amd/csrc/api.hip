// C ABI entry points: argument checking, scratch sizing and dispatch to the kernel launchers.
#include <math.h>
#include <stdarg.h>
#include <string.h>

#include <new>

#include "common.h"
#include "model.h"
#include "net.h"
#include "kernels.h"

int bls_fail(bls_ctx* ctx, int code, const char* fmt, ...) {
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        ctx->error = buf;
    }
    return code;
}

int bls_arena_reserve(bls_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->arena_bytes) return BLS_OK;
    BLS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->aux) BLS_HIP(ctx, hipStreamSynchronize(ctx->aux));
    if (ctx->aux2) BLS_HIP(ctx, hipStreamSynchronize(ctx->aux2));
    if (ctx->arena) BLS_HIP(ctx, hipFree(ctx->arena));
    ctx->arena = nullptr;
    ctx->arena_bytes = 0;
    size_t want = bytes + bytes / 8;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&ctx->arena), want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return bls_fail(ctx, BLS_ENOMEM, "scratch allocation of %zu bytes failed: %s", want, hipGetErrorString(e));
    }
    ctx->arena_bytes = want;
    return BLS_OK;
}

#pragma GCC visibility push(default)
extern "C" {

int bls_ctx_create(bls_ctx** out, int device, void* hip_stream) {
    if (!out) return BLS_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) {
        (void)hipGetLastError();
        return BLS_EHIP;
    }
    if (hipSetDevice(device) != hipSuccess) return BLS_EHIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return BLS_EHIP;
    bls_ctx* ctx = new (std::nothrow) bls_ctx();
    if (!ctx) return BLS_ENOMEM;
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->num_cus = prop.multiProcessorCount;
    ctx->max_lds = prop.sharedMemPerBlock;
    int optin = 0;
    if (hipDeviceGetAttribute(&optin, hipDeviceAttributeSharedMemPerBlockOptin, device) == hipSuccess &&
        (size_t)optin > ctx->max_lds)
        ctx->max_lds = (size_t)optin;
    (void)hipGetLastError();
    if (hipStreamCreateWithFlags(&ctx->aux, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->join_event, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->join_event2, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->head_event, hipEventDisableTiming) != hipSuccess) {
        delete ctx;
        return BLS_EHIP;
    }
    if (topk_static_init(ctx) != BLS_OK) {
        bls_ctx_destroy(ctx);
        return BLS_EHIP;
    }
    *out = ctx;
    return BLS_OK;
}

void bls_ctx_destroy(bls_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (bls_ctx* lane : ctx->lanes) bls_ctx_destroy(lane);
    ctx->lanes.clear();
    for (hipEvent_t e : ctx->lane_events) (void)hipEventDestroy(e);
    if (ctx->round_start) (void)hipEventDestroy(ctx->round_start);
    net_release(ctx);
    if (ctx->aux) {
        (void)hipStreamSynchronize(ctx->aux);
        (void)hipStreamDestroy(ctx->aux);
    }
    if (ctx->aux2) {
        (void)hipStreamSynchronize(ctx->aux2);
        (void)hipStreamDestroy(ctx->aux2);
    }
    for (hipEvent_t e : ctx->fork_events) (void)hipEventDestroy(e);
    if (ctx->join_event) (void)hipEventDestroy(ctx->join_event);
    if (ctx->join_event2) (void)hipEventDestroy(ctx->join_event2);
    if (ctx->head_event) (void)hipEventDestroy(ctx->head_event);
    if (ctx->arena) (void)hipFree(ctx->arena);
    if (ctx->round_losses) (void)hipFree(ctx->round_losses);
    if (ctx->owns_stream) (void)hipStreamDestroy(ctx->stream);
    delete ctx;
}

int bls_ctx_set_lanes(bls_ctx* ctx, int lanes) {
    if (!ctx) return BLS_EINVAL;
    if (lanes < 1 || lanes > 16) return bls_fail(ctx, BLS_EINVAL, "bls_ctx_set_lanes: need 1 <= lanes <= 16");
    BLS_HIP(ctx, hipSetDevice(ctx->device));
    BLS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const int want = lanes == 1 ? 0 : lanes;   // one lane = the context's own stream
    while ((int)ctx->lanes.size() > want) {
        bls_ctx_destroy(ctx->lanes.back());
        ctx->lanes.pop_back();
    }
    while ((int)ctx->lanes.size() < want) {
        hipStream_t st = nullptr;
        BLS_HIP(ctx, hipStreamCreateWithFlags(&st, hipStreamNonBlocking));   // default priority
        bls_ctx* lane = nullptr;
        int rc = bls_ctx_create(&lane, ctx->device, st);
        if (rc != BLS_OK) {
            (void)hipStreamDestroy(st);
            return bls_fail(ctx, rc, "bls_ctx_set_lanes: could not create lane %d", (int)ctx->lanes.size());
        }
        lane->owns_stream = true;
        ctx->lanes.push_back(lane);
    }
    if (!ctx->round_start) BLS_HIP(ctx, hipEventCreateWithFlags(&ctx->round_start, hipEventDisableTiming));
    return BLS_OK;
}

const char* bls_last_error(const bls_ctx* ctx) { return ctx ? ctx->error.c_str() : ""; }

int bls_ctx_synchronize(bls_ctx* ctx) {
    if (!ctx) return BLS_EINVAL;
    BLS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return BLS_OK;
}

int bls_profile_begin(bls_ctx* ctx) {
    if (!ctx) return BLS_EINVAL;
    ctx->profiling = true;
    return BLS_OK;
}

int bls_profile_end(bls_ctx* ctx, double* ms_by_class, int64_t* launches_by_class, int capacity) {
    if (!ctx) return BLS_EINVAL;
    ctx->profiling = false;
    BLS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (int i = 0; i < capacity; ++i) {
        if (ms_by_class) ms_by_class[i] = 0.0;
        if (launches_by_class) launches_by_class[i] = 0;
    }
    for (ProfSpan& sp : ctx->spans) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sp.start, sp.stop) == hipSuccess && sp.cls < capacity) {
            if (ms_by_class) ms_by_class[sp.cls] += (double)ms;
            if (launches_by_class) launches_by_class[sp.cls] += 1;
        }
        (void)hipEventDestroy(sp.start);
        (void)hipEventDestroy(sp.stop);
    }
    ctx->spans.clear();
    return PROF_NUM_CLASSES;
}

// ---- model ----------------------------------------------------------------------------------------

static void add_tensor(bls_model* m, const std::string& name, bool is_buffer, int ndim, int s0, int s1 = 1, int s2 = 1,
                       int s3 = 1) {
    TensorSlot t;
    t.name = name;
    t.ndim = ndim;
    t.shape[0] = s0; t.shape[1] = s1; t.shape[2] = s2; t.shape[3] = s3;
    t.is_buffer = is_buffer;
    int64_t& total = is_buffer ? m->num_buffers : m->num_params;
    t.offset = total;
    total += t.count();
    m->tensors.push_back(t);
}

static void add_conv_bn(bls_model* m, const std::string& conv, const std::string& bn, int c_in, int c_out, int stride,
                        int h_in) {
    ConvBn l;
    l.c_in = c_in; l.c_out = c_out; l.stride = stride; l.h_in = h_in; l.h_out = (h_in - 1) / stride + 1;
    l.w_off = m->num_params;
    add_tensor(m, conv + ".weight", false, 4, c_out, 3, 3, c_in);
    l.gamma_off = m->num_params;
    add_tensor(m, bn + ".weight", false, 1, c_out);
    l.beta_off = m->num_params;
    add_tensor(m, bn + ".bias", false, 1, c_out);
    l.rmean_off = m->num_buffers;
    add_tensor(m, bn + ".running_mean", true, 1, c_out);
    l.rvar_off = m->num_buffers;
    add_tensor(m, bn + ".running_var", true, 1, c_out);
    m->layers.push_back(l);
}

int bls_model_create(const bls_model_desc* desc, bls_model** out) {
    if (!desc || !out) return BLS_EINVAL;
    *out = nullptr;
    const int max_classes = desc->kind == BLS_MODEL_ENCODER ? (1 << 20) : desc->kind == BLS_MODEL_WRN ? 128 : 64;
    if (desc->classes < 2 || desc->classes > max_classes) return BLS_EINVAL;
    if (desc->act_dtype != BLS_ACT_F32 && desc->act_dtype != BLS_ACT_BF16) return BLS_EINVAL;
    if (desc->kind == BLS_MODEL_MLP && desc->act_dtype != BLS_ACT_F32) return BLS_EUNSUPPORTED;
    // a convolution's input width must be 16 or a multiple of 32 in the wide network
    auto wide_ok = [](int c) { return c == 16 || (c >= 32 && c <= 512 && c % 32 == 0); };
    bls_model* m = new (std::nothrow) bls_model();
    if (!m) return BLS_ENOMEM;
    m->desc = *desc;
    if (desc->kind == BLS_MODEL_MLP) {
        if (desc->image_hw < 1 || desc->in_channels < 1 || desc->hidden < 16 || desc->hidden > 1024 ||
            desc->hidden % 16 != 0 || (int64_t)desc->image_hw * desc->image_hw * desc->in_channels > (1 << 20)) {
            delete m;
            return BLS_EINVAL;
        }
        m->d_in = desc->image_hw * desc->image_hw * desc->in_channels;
        m->fc1_w = m->num_params; add_tensor(m, "fc1.weight", false, 2, desc->hidden, m->d_in);
        m->fc1_b = m->num_params; add_tensor(m, "fc1.bias", false, 1, desc->hidden);
        m->fc2_w = m->num_params; add_tensor(m, "fc2.weight", false, 2, desc->classes, desc->hidden);
        m->fc2_b = m->num_params; add_tensor(m, "fc2.bias", false, 1, desc->classes);
    } else if (desc->kind == BLS_MODEL_RESNET_CIFAR) {
        bool ok = (desc->image_hw == 8 || desc->image_hw == 16 || desc->image_hw == 32 || desc->image_hw == 64) && desc->in_channels >= 1 &&
                  desc->in_channels <= 4 && desc->blocks >= 1 && desc->blocks <= 6;
        for (int s = 0; s < 3; ++s) {
            int w = desc->widths[s];
            ok = ok && (w == 16 || w == 32 || w == 64);
            // the zero-padded shortcut needs an even number of extra channels and never fewer
            if (s > 0) ok = ok && w >= desc->widths[s - 1] && (w - desc->widths[s - 1]) % 2 == 0;
        }
        if (!ok) {
            delete m;
            return BLS_EINVAL;
        }
        int hw = desc->image_hw;
        add_conv_bn(m, "stem.conv", "stem.bn", desc->in_channels, desc->widths[0], 1, hw);
        int c_prev = desc->widths[0];
        for (int s = 0; s < 3; ++s) {
            int c = desc->widths[s];
            for (int b = 0; b < desc->blocks; ++b) {
                int stride = (b == 0 && s > 0) ? 2 : 1;
                char p[32];
                snprintf(p, sizeof p, "s%d.b%d", s + 1, b);
                add_conv_bn(m, std::string(p) + ".conv1", std::string(p) + ".bn1", c_prev, c, stride, hw);
                hw = (hw - 1) / stride + 1;
                add_conv_bn(m, std::string(p) + ".conv2", std::string(p) + ".bn2", c, c, 1, hw);
                c_prev = c;
            }
        }
        m->final_c = c_prev;
        m->final_hw = hw;
        m->fc_w = m->num_params; add_tensor(m, "fc.weight", false, 2, desc->classes, c_prev);
        m->fc_b = m->num_params; add_tensor(m, "fc.bias", false, 1, desc->classes);
    } else if (desc->kind == BLS_MODEL_WRN) {
        bool ok = (desc->image_hw == 8 || desc->image_hw == 16 || desc->image_hw == 32) && desc->in_channels >= 1 &&
                  desc->in_channels <= 4 && desc->blocks >= 1 && desc->blocks <= 4 && wide_ok(desc->hidden);
        for (int s = 0; s < 3; ++s) ok = ok && wide_ok(desc->widths[s]);
        if (!ok) {
            delete m;
            return BLS_EINVAL;
        }
        auto add_bn = [&](const std::string& name, int c) {
            BnSlot b;
            b.c = c;
            b.gamma_off = m->num_params; add_tensor(m, name + ".weight", false, 1, c);
            b.beta_off = m->num_params; add_tensor(m, name + ".bias", false, 1, c);
            b.rmean_off = m->num_buffers; add_tensor(m, name + ".running_mean", true, 1, c);
            b.rvar_off = m->num_buffers; add_tensor(m, name + ".running_var", true, 1, c);
            return b;
        };
        auto add_conv = [&](const std::string& name, int c_in, int c_out, int stride, int taps, int h_in) {
            ConvSlot c;
            c.c_in = c_in; c.c_out = c_out; c.stride = stride; c.taps = taps; c.h_in = h_in; c.h_out = (h_in - 1) / stride + 1;
            c.w_off = m->num_params;
            const int k = taps == 9 ? 3 : 1;
            add_tensor(m, name + ".weight", false, 4, c_out, k, k, c_in);
            return c;
        };
        int hw = desc->image_hw;
        m->wrn_stem = add_conv("stem.conv", desc->in_channels, desc->hidden, 1, 9, hw);
        int c_prev = desc->hidden;
        for (int s = 0; s < 3; ++s) {
            int c = desc->widths[s];
            for (int b = 0; b < desc->blocks; ++b) {
                int stride = (b == 0 && s > 0) ? 2 : 1;
                char pn[32];
                snprintf(pn, sizeof pn, "s%d.b%d", s + 1, b);
                const std::string p(pn);
                WrnBlock blk{};
                blk.proj = c_prev != c || stride != 1;
                blk.bn1 = add_bn(p + ".bn1", c_prev);
                blk.conv1 = add_conv(p + ".conv1", c_prev, c, stride, 9, hw);
                const int h_out = (hw - 1) / stride + 1;
                blk.bn2 = add_bn(p + ".bn2", c);
                blk.conv2 = add_conv(p + ".conv2", c, c, 1, 9, h_out);
                if (blk.proj) blk.shortcut = add_conv(p + ".shortcut", c_prev, c, stride, 1, hw);
                m->wrn_blocks.push_back(blk);
                hw = h_out;
                c_prev = c;
            }
        }
        m->wrn_final_bn = add_bn("final.bn", c_prev);
        m->final_c = c_prev;
        m->final_hw = hw;
        m->fc_w = m->num_params; add_tensor(m, "fc.weight", false, 2, desc->classes, c_prev);
        m->fc_b = m->num_params; add_tensor(m, "fc.bias", false, 1, desc->classes);
    } else if (desc->kind == BLS_MODEL_ENCODER) {
        const int V = desc->classes, L = desc->image_hw, D = desc->hidden, H = desc->widths[0], F = desc->widths[1];
        if (L < 1 || L > 1024 || D < 4 || D > 1024 || D % 4 != 0 || H < 1 || D % H != 0 || F < 4 || F % 4 != 0 || F > 8192 ||
            desc->blocks < 1 || desc->blocks > 16) {
            delete m;
            return BLS_EINVAL;
        }
        m->enc_V = V; m->enc_L = L; m->enc_D = D; m->enc_H = H; m->enc_F = F;
        m->enc_tok = m->num_params; add_tensor(m, "tok_emb.weight", false, 2, V, D);
        m->enc_pos = m->num_params; add_tensor(m, "pos_emb.weight", false, 2, L, D);
        for (int l = 0; l < desc->blocks; ++l) {
            char pn[16];
            snprintf(pn, sizeof pn, "l%d.", l);
            const std::string p(pn);
            EncLayer e;
            auto lin = [&](const std::string& name, int out_f, int in_f, int64_t& w, int64_t& b) {
                w = m->num_params; add_tensor(m, p + name + ".weight", false, 2, out_f, in_f);
                b = m->num_params; add_tensor(m, p + name + ".bias", false, 1, out_f);
            };
            lin("attn.q", D, D, e.wq, e.bq);
            lin("attn.k", D, D, e.wk, e.bk);
            lin("attn.v", D, D, e.wv, e.bv);
            lin("attn.o", D, D, e.wo, e.bo);
            e.ln1_g = m->num_params; add_tensor(m, p + "ln1.weight", false, 1, D);
            e.ln1_b = m->num_params; add_tensor(m, p + "ln1.bias", false, 1, D);
            lin("ffn.fc1", F, D, e.w1, e.b1);
            lin("ffn.fc2", D, F, e.w2, e.b2);
            e.ln2_g = m->num_params; add_tensor(m, p + "ln2.weight", false, 1, D);
            e.ln2_b = m->num_params; add_tensor(m, p + "ln2.bias", false, 1, D);
            m->enc_layers.push_back(e);
        }
        m->enc_head = m->num_params; add_tensor(m, "head.weight", false, 2, V, D);
    } else {
        delete m;
        return BLS_EINVAL;
    }
    *out = m;
    return BLS_OK;
}

void bls_model_destroy(bls_model* model) { delete model; }
int64_t bls_model_num_params(const bls_model* model) { return model ? model->num_params : BLS_EINVAL; }
int64_t bls_model_num_buffers(const bls_model* model) { return model ? model->num_buffers : BLS_EINVAL; }
int32_t bls_model_num_tensors(const bls_model* model) { return model ? (int32_t)model->tensors.size() : BLS_EINVAL; }

int64_t bls_model_workspace_bytes(const bls_model* model, int64_t n, int training) {
    if (!model || n < 1 || n > (int64_t(1) << 24)) return BLS_EINVAL;
    const bool train = training != 0;
    if (model->desc.kind == BLS_MODEL_ENCODER) {
        if (train && n * model->enc_L >= (int64_t(1) << 31) / 8) return BLS_EINVAL;
        return (int64_t)seq_workspace_bytes(model, n, train);
    }
    if (model->desc.kind == BLS_MODEL_WRN) return (int64_t)wrn_workspace_bytes(model, n, train);
    return (int64_t)net_workspace_bytes(model, n, train);
}

int bls_model_tensor_layout(const bls_model* model, bls_tensor_info* out, int32_t capacity) {
    if (!model || !out || capacity < 0) return BLS_EINVAL;
    int n = (int)model->tensors.size() < capacity ? (int)model->tensors.size() : capacity;
    for (int i = 0; i < n; ++i) {
        const TensorSlot& t = model->tensors[i];
        memset(&out[i], 0, sizeof out[i]);
        strncpy(out[i].name, t.name.c_str(), sizeof out[i].name - 1);
        out[i].offset = t.offset;
        out[i].ndim = t.ndim;
        for (int j = 0; j < 4; ++j) out[i].shape[j] = j < t.ndim ? t.shape[j] : 1;
        out[i].is_buffer = t.is_buffer ? 1 : 0;
    }
    return n;
}

// ---- operations -----------------------------------------------------------------------------------

int score_losses(bls_ctx* ctx, const bls_model* model, const float* params, const float* buffers, const void* x_any,
                 const int32_t* y, int64_t N, float* losses_out) {
    if (!ctx) return BLS_EINVAL;
    if (!model || N < 0) return bls_fail(ctx, BLS_EINVAL, "score_losses: model is NULL or N < 0");
    if (N == 0) return BLS_OK;
    if (!params || !x_any || !y || !losses_out) return bls_fail(ctx, BLS_EINVAL, "score_losses: NULL pointer");
    if (model->num_buffers > 0 && !buffers) return bls_fail(ctx, BLS_EINVAL, "score_losses: this model needs buffers");
    if (N >= (int64_t(1) << 31)) return bls_fail(ctx, BLS_EINVAL, "score_losses: N must be below 2^31");
    BLS_HIP(ctx, hipSetDevice(ctx->device));
    if (model->desc.kind == BLS_MODEL_ENCODER) return seq_score(ctx, model, params, static_cast<const int32_t*>(x_any), y, N, losses_out);
    const float* x = static_cast<const float*>(x_any);
    if (model->desc.kind == BLS_MODEL_WRN) return wrn_score(ctx, model, params, buffers, x, y, N, losses_out);
    return net_score(ctx, model, params, buffers, x, y, N, losses_out);
}

int topk_by_loss(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out) {
    if (!ctx) return BLS_EINVAL;
    if (N < 0 || k < 0 || k > N) return bls_fail(ctx, BLS_EINVAL, "topk_by_loss: need 0 <= k <= N (N=%lld, k=%lld)", (long long)N, (long long)k);
    if (N >= (int64_t(1) << 31)) return bls_fail(ctx, BLS_EINVAL, "topk_by_loss: N must be below 2^31");
    if (k == 0) return BLS_OK;
    if (!losses || !idx_out) return bls_fail(ctx, BLS_EINVAL, "topk_by_loss: NULL pointer");
    BLS_HIP(ctx, hipSetDevice(ctx->device));
    ProfScope prof(ctx, PROF_TOPK);
    return launch_topk(ctx, losses, N, k, idx_out, val_out);
}

int topk_by_loss_static(bls_ctx* ctx, const float* losses, int64_t N, int64_t k, int32_t* idx_out, float* val_out) {
    if (!ctx) return BLS_EINVAL;
    if (N < 0 || k < 0 || k > N) return bls_fail(ctx, BLS_EINVAL, "topk_by_loss_static: need 0 <= k <= N (N=%lld, k=%lld)", (long long)N, (long long)k);
    if (k == 0) return BLS_OK;
    if (!losses || !idx_out) return bls_fail(ctx, BLS_EINVAL, "topk_by_loss_static: NULL pointer");
    BLS_HIP(ctx, hipSetDevice(ctx->device));
    ProfScope prof(ctx, PROF_TOPK);
    return launch_topk_static(ctx, losses, N, k, idx_out, val_out);
}

int local_step(bls_ctx* ctx, const bls_model* model, float* params, float* buffers, float* momentum,
               const void* x_any, const int32_t* y_pool, int64_t N, const int32_t* sel_idx, int64_t k, int64_t batch,
               int64_t tau, const bls_sgd* opt, float* step_losses_out) {
    if (!ctx) return BLS_EINVAL;
    if (!model || !opt) return bls_fail(ctx, BLS_EINVAL, "local_step: model or opt is NULL");
    if (N < 1 || k < 1 || batch < 1 || tau < 0) return bls_fail(ctx, BLS_EINVAL, "local_step: need N, k, batch >= 1 and tau >= 0");
    if (N >= (int64_t(1) << 31) || batch > 65536) return bls_fail(ctx, BLS_EINVAL, "local_step: N < 2^31 and batch <= 65536 required");
    if (!(isfinite(opt->lr) && isfinite(opt->momentum) && isfinite(opt->weight_decay)))
        return bls_fail(ctx, BLS_EINVAL, "local_step: non-finite optimiser setting");
    if (tau == 0) return BLS_OK;
    if (!params || !momentum || !x_any || !y_pool || !sel_idx) return bls_fail(ctx, BLS_EINVAL, "local_step: NULL pointer");
    if (model->num_buffers > 0 && !buffers) return bls_fail(ctx, BLS_EINVAL, "local_step: this model needs buffers");
    if (model->desc.kind != BLS_MODEL_MLP && model->desc.kind != BLS_MODEL_ENCODER && batch * model->final_hw * model->final_hw < 2)
        return bls_fail(ctx, BLS_EINVAL, "local_step: batch norm needs more than one value per channel");
    BLS_HIP(ctx, hipSetDevice(ctx->device));
    if (model->desc.kind == BLS_MODEL_ENCODER)
        return seq_local_step(ctx, model, params, momentum, static_cast<const int32_t*>(x_any), y_pool, N, sel_idx, k, batch, tau, *opt,
                              step_losses_out);
    const float* x_pool = static_cast<const float*>(x_any);
    if (model->desc.kind == BLS_MODEL_WRN)
        return wrn_local_step(ctx, model, params, buffers, momentum, x_pool, y_pool, N, sel_idx, k, batch, tau, *opt, step_losses_out);
    return net_local_step(ctx, model, params, buffers, momentum, x_pool, y_pool, N, sel_idx, k, batch, tau, *opt,
                          step_losses_out);
}

int weighted_aggregate(bls_ctx* ctx, const float* const* replicas, const float* weights, int P, int64_t d, float* out,
                       int flags) {
    if (!ctx) return BLS_EINVAL;
    if (P < 1 || P > 64 || d < 0) return bls_fail(ctx, BLS_EINVAL, "weighted_aggregate: need 1 <= P <= 64 and d >= 0");
    if (!replicas || !weights) return bls_fail(ctx, BLS_EINVAL, "weighted_aggregate: NULL pointer");
    if (flags & ~(BLS_AGG_NORMALISE | BLS_AGG_BROADCAST)) return bls_fail(ctx, BLS_EINVAL, "weighted_aggregate: unknown flag");
    double sum = 0.0;
    for (int i = 0; i < P; ++i) {
        if (!isfinite(weights[i]) || weights[i] < 0.f)
            return bls_fail(ctx, BLS_EINVAL, "weighted_aggregate: weight %d is negative or not finite", i);
        sum += (double)weights[i];
    }
    float w[64];
    if (flags & BLS_AGG_NORMALISE) {
        if (!(sum > 0.0)) return bls_fail(ctx, BLS_EINVAL, "weighted_aggregate: weights sum to zero");
        for (int i = 0; i < P; ++i) w[i] = (float)((double)weights[i] / sum);
    } else {
        if (fabs(sum - 1.0) > 1e-5) return bls_fail(ctx, BLS_EINVAL, "weighted_aggregate: weights sum to %.9g, not 1", sum);
        for (int i = 0; i < P; ++i) w[i] = weights[i];
    }
    if (d == 0) return BLS_OK;
    if (!out) return bls_fail(ctx, BLS_EINVAL, "weighted_aggregate: NULL output");
    for (int i = 0; i < P; ++i)
        if (!replicas[i]) return bls_fail(ctx, BLS_EINVAL, "weighted_aggregate: replica %d is NULL", i);
    BLS_HIP(ctx, hipSetDevice(ctx->device));
    ProfScope prof(ctx, PROF_AGGREGATE);
    return launch_weighted_aggregate(ctx, replicas, w, P, d, out, (flags & BLS_AGG_BROADCAST) != 0);
}

int bls_epoch_allocation(int64_t N, int64_t tau_f, int P_f, int64_t tau_s, int P_s, double lambda, int64_t* n_fast,
                         int64_t* k_high, int64_t* n_slow) {
    if (N < 0 || N >= (int64_t(1) << 31) || tau_f < 1 || tau_f > (1 << 20) || tau_s < 0 || tau_s > (1 << 20) || P_f < 1 ||
        P_f > 1024 || P_s < 0 || P_s > 1024 || !(lambda > 0.0 && lambda <= 1.0))
        return BLS_EINVAL;
    const int64_t fast = tau_f * P_f, slow = tau_s * P_s;
    const int64_t nf = N * fast / (fast + slow);
    if (n_fast) *n_fast = nf;
    if (k_high) *k_high = (int64_t)floor(lambda * (double)nf);
    if (n_slow) *n_slow = N - nf;
    return BLS_OK;
}

int bls_worker_share(int64_t n, int P, int p, int64_t* offset, int64_t* count) {
    if (n < 0 || P < 1 || p < 0 || p >= P) return BLS_EINVAL;
    const int64_t base = n / P, rem = n % P;
    if (offset) *offset = p * base + (p < rem ? p : rem);
    if (count) *count = base + (p < rem ? 1 : 0);
    return BLS_OK;
}

int sample_epoch_variant(bls_ctx* ctx, const float* losses, const float* u_fast, const float* u_slow, int64_t N, int64_t tau_f, int P_f,
                         int64_t tau_s, int P_s, double lambda, int scheme, int high_loss_to, int32_t* fast_idx_out, int32_t* slow_idx_out) {
    if (!ctx) return BLS_EINVAL;
    if ((scheme != BLS_SAMPLING_SEPARATED && scheme != BLS_SAMPLING_UNIFIED) ||
        (high_loss_to != BLS_HIGH_LOSS_TO_FAST && high_loss_to != BLS_HIGH_LOSS_TO_SLOW && high_loss_to != BLS_HIGH_LOSS_TO_NONE))
        return bls_fail(ctx, BLS_EINVAL, "sample_epoch_variant: unknown scheme or group");
    int64_t nf, k, ns;
    if (bls_epoch_allocation(N, tau_f, P_f, tau_s, P_s, lambda, &nf, &k, &ns) != BLS_OK)
        return bls_fail(ctx, BLS_EINVAL, "sample_epoch: need 0 <= N < 2^31, 1 <= tau_F, 0 <= tau_S, 1 <= P_F, 0 <= P_S, 0 < lambda <= 1");
    if (ns > 0 && P_s < 1) return bls_fail(ctx, BLS_EINVAL, "sample_epoch: slow samples but no slow worker");
    if (N == 0) return BLS_OK;
    const bool to_fast = high_loss_to != BLS_HIGH_LOSS_TO_SLOW;   // without a by-loss part the fast group still draws first
    if (!to_fast) k = (int64_t)floor(lambda * (double)ns);   // the by-loss part of the slow allocation
    if (high_loss_to == BLS_HIGH_LOSS_TO_NONE) k = 0;
    const int64_t n_biased = to_fast ? nf : ns, n_other = to_fast ? ns : nf;
    const float *u_biased = to_fast ? u_fast : u_slow, *u_other = to_fast ? u_slow : u_fast;
    if ((k > 0 && !losses) || (n_biased > k && !u_biased) || (n_other > 0 && !u_other) || (nf > 0 && !fast_idx_out) || (ns > 0 && !slow_idx_out))
        return bls_fail(ctx, BLS_EINVAL, "sample_epoch: NULL pointer");
    BLS_HIP(ctx, hipSetDevice(ctx->device));
    ProfScope prof(ctx, PROF_TOPK);
    return launch_sample_epoch(ctx, losses, u_biased, u_other, N, n_biased, k, n_other, to_fast ? P_f : P_s, to_fast ? P_s : P_f,
                               scheme == BLS_SAMPLING_UNIFIED, to_fast ? fast_idx_out : slow_idx_out, to_fast ? slow_idx_out : fast_idx_out);
}

int sample_epoch(bls_ctx* ctx, const float* losses, const float* u_fast, const float* u_slow, int64_t N, int64_t tau_f,
                 int P_f, int64_t tau_s, int P_s, double lambda, int32_t* fast_idx_out, int32_t* slow_idx_out) {
    return sample_epoch_variant(ctx, losses, u_fast, u_slow, N, tau_f, P_f, tau_s, P_s, lambda, BLS_SAMPLING_SEPARATED, BLS_HIGH_LOSS_TO_FAST,
                                fast_idx_out, slow_idx_out);
}

// table[idx[e mod n_idx]] = losses[e] for the last entry e of every cyclic position: the local steps walk idx cyclically,
// so entry e is overwritten later exactly when e + n_idx < n.
__global__ __launch_bounds__(256) void record_losses_kernel(const int32_t* __restrict__ idx, int64_t n_idx, int64_t n,
                                                            const float* __restrict__ losses, float* __restrict__ table) {
    const int64_t first = n > n_idx ? n - n_idx : 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) table[idx[e % n_idx]] = losses[e];
}

// True when [a, a + na) and [b, b + nb) floats share an address.
static bool ranges_overlap(const float* a, int64_t na, const float* b, int64_t nb) {
    if (!a || !b || na <= 0 || nb <= 0) return false;
    return a < b + nb && b < a + na;
}

int communication_round(bls_ctx* ctx, const bls_model* model, float* global_params, float* global_buffers, const bls_worker* workers, int P,
                        const void* x_pool, const int32_t* y_pool, int64_t N, int64_t batch, const bls_sgd* opt, float* loss_table, int flags) {
    if (!ctx) return BLS_EINVAL;
    if (!model || !opt || !workers || !global_params) return bls_fail(ctx, BLS_EINVAL, "communication_round: NULL pointer");
    if (P < 1 || P > 64 || batch < 1 || batch > 65536) return bls_fail(ctx, BLS_EINVAL, "communication_round: need 1 <= P <= 64, 1 <= batch <= 65536");
    if (flags & ~(BLS_ROUND_UNIFORM_WEIGHTS | BLS_ROUND_SEQUENTIAL)) return bls_fail(ctx, BLS_EINVAL, "communication_round: unknown flag");
    for (int i = 0; i < P; ++i)   // local_step's own checks, made here once for every path
        if (workers[i].tau > 0 && (N < 1 || N >= (int64_t(1) << 31) || !x_pool || !y_pool))
            return bls_fail(ctx, BLS_EINVAL, "communication_round: need a pool of 1 <= N < 2^31 samples");
    if (!(isfinite(opt->lr) && isfinite(opt->momentum) && isfinite(opt->weight_decay)))
        return bls_fail(ctx, BLS_EINVAL, "communication_round: non-finite optimiser setting");
    if (model->desc.kind != BLS_MODEL_MLP && model->desc.kind != BLS_MODEL_ENCODER && batch * model->final_hw * model->final_hw < 2)
        return bls_fail(ctx, BLS_EINVAL, "communication_round: batch norm needs more than one value per channel");
    if (model->num_buffers > 0 && !global_buffers) return bls_fail(ctx, BLS_EINVAL, "communication_round: this model needs buffers");
    const bool uniform = (flags & BLS_ROUND_UNIFORM_WEIGHTS) != 0;
    const int64_t d = model->num_params, nb = model->num_buffers;
    double weight_sum = 0.0;
    int64_t total = 0;
    for (int i = 0; i < P; ++i) {
        const bls_worker& w = workers[i];
        if (w.tau < 0 || w.tau > (int64_t(1) << 20)) return bls_fail(ctx, BLS_EINVAL, "communication_round: tau of worker %d out of range", i);
        if (w.tau == 0) continue;
        if (!w.idx || w.n_idx < 1 || !w.params || !w.momentum || (nb > 0 && !w.buffers))
            return bls_fail(ctx, BLS_EINVAL, "communication_round: worker %d lacks samples or storage", i);
        if (ranges_overlap(w.params, d, global_params, d) || ranges_overlap(w.momentum, d, global_params, d) ||
            ranges_overlap(w.params, d, w.momentum, d) || ranges_overlap(w.buffers, nb, global_buffers, nb))
            return bls_fail(ctx, BLS_EINVAL, "communication_round: storage of worker %d overlaps the global model or itself", i);
        for (int j = 0; j < i; ++j) {
            const bls_worker& v = workers[j];
            if (v.tau == 0) continue;
            if (ranges_overlap(w.params, d, v.params, d) || ranges_overlap(w.params, d, v.momentum, d) || ranges_overlap(w.momentum, d, v.params, d) ||
                ranges_overlap(w.momentum, d, v.momentum, d) || ranges_overlap(w.buffers, nb, v.buffers, nb))
                return bls_fail(ctx, BLS_EINVAL, "communication_round: workers %d and %d share storage", j, i);
        }
        weight_sum += uniform ? 1.0 : (double)w.tau;
        total += w.tau * batch;
    }
    if (!(weight_sum > 0.0)) return bls_fail(ctx, BLS_EINVAL, "communication_round: no worker takes a step");
    BLS_HIP(ctx, hipSetDevice(ctx->device));
    if (loss_table && (size_t)total > ctx->round_losses_count) {
        BLS_HIP(ctx, hipStreamSynchronize(ctx->stream));
        for (bls_ctx* lane : ctx->lanes) BLS_HIP(ctx, hipStreamSynchronize(lane->stream));
        if (ctx->round_losses) BLS_HIP(ctx, hipFree(ctx->round_losses));
        ctx->round_losses = nullptr;
        ctx->round_losses_count = 0;
        BLS_HIP(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->round_losses), (size_t)total * sizeof(float)));
        ctx->round_losses_count = (size_t)total;
    }
    const int n_lanes = (int)ctx->lanes.size();
    while ((int)ctx->lane_events.size() < P) {
        hipEvent_t e;
        BLS_HIP(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
        ctx->lane_events.push_back(e);
    }
    const float* trained[64];
    const float* trained_buffers[64];
    float weights[64];
    int64_t loss_off[64];
    int n_trained = 0;
    int64_t off = 0;
    for (int i = 0; i < P; ++i) {
        const bls_worker& w = workers[i];
        if (w.tau == 0) continue;
        trained[n_trained] = w.params;
        trained_buffers[n_trained] = w.buffers;
        weights[n_trained] = (float)((uniform ? 1.0 : (double)w.tau) / weight_sum);   // Eq. 4 in double, rounded once
        loss_off[n_trained] = off;
        off += w.tau * batch;
        ++n_trained;
    }
    // Networks with a batched path run all workers in one launch per layer (the same kernels on the same data per worker,
    // hence the same bits as one after the other); it needs one scratch slot per worker.
    const bool batched = n_lanes == 0 && !(flags & BLS_ROUND_SEQUENTIAL) && n_trained >= 2 && net_round_batched_covers(model);
    if (batched) {
        int rc = net_round_batched(ctx, model, global_params, global_buffers, workers, P, static_cast<const float*>(x_pool), y_pool, batch, *opt,
                                   loss_table ? ctx->round_losses : nullptr, loss_off);
        if (rc != BLS_OK) return rc;
    } else {
        if (n_lanes > 0) BLS_HIP(ctx, hipEventRecord(ctx->round_start, ctx->stream));   // the global model is ready
        int t = 0;
        for (int i = 0; i < P; ++i) {
            const bls_worker& w = workers[i];
            if (w.tau == 0) continue;
            bls_ctx* lane = n_lanes > 0 ? ctx->lanes[t % n_lanes] : ctx;
            if (lane != ctx) BLS_HIP(ctx, hipStreamWaitEvent(lane->stream, ctx->round_start, 0));
            // every worker starts the round from the global model (the aggregate of the previous round)
            BLS_HIP(ctx, hipMemcpyAsync(w.params, global_params, (size_t)d * sizeof(float), hipMemcpyDeviceToDevice, lane->stream));
            if (nb > 0) BLS_HIP(ctx, hipMemcpyAsync(w.buffers, global_buffers, (size_t)nb * sizeof(float), hipMemcpyDeviceToDevice, lane->stream));
            int rc = local_step(lane, model, w.params, w.buffers, w.momentum, x_pool, y_pool, N, w.idx, w.n_idx, batch, w.tau, opt,
                                loss_table ? ctx->round_losses + loss_off[t] : nullptr);
            if (rc != BLS_OK) return lane == ctx ? rc : bls_fail(ctx, rc, "communication_round: worker %d: %s", i, lane->error.c_str());
            if (lane != ctx) BLS_HIP(ctx, hipEventRecord(ctx->lane_events[t], lane->stream));
            ++t;
        }
    }
    if (n_lanes > 0)
        for (int t = 0; t < n_trained; ++t) BLS_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->lane_events[t], 0));
    if (loss_table) {
        // in worker order on the one stream, so that of two workers that processed the same sample the later one wins
        int t = 0;
        for (int i = 0; i < P; ++i) {
            const bls_worker& w = workers[i];
            if (w.tau == 0) continue;
            const int64_t n = w.tau * batch, live = n < w.n_idx ? n : w.n_idx;
            hipLaunchKernelGGL(record_losses_kernel, dim3((unsigned)((live + 255) / 256)), dim3(256), 0, ctx->stream, w.idx, w.n_idx, n,
                               ctx->round_losses + loss_off[t], loss_table);
            ++t;
        }
    }
    int rc = weighted_aggregate(ctx, trained, weights, n_trained, d, global_params, 0);
    if (rc != BLS_OK) return rc;
    if (nb > 0) rc = weighted_aggregate(ctx, trained_buffers, weights, n_trained, nb, global_buffers, 0);
    if (rc != BLS_OK) return rc;
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

int train_epochs(bls_ctx* ctx, const bls_model* model, const bls_epoch_plan* plan, float* global_params, float* global_buffers,
                 float* worker_params, float* worker_buffers, float* worker_momentum, const void* x_pool, const int32_t* y_pool, int64_t N,
                 const float* u_fast, const float* u_slow, float* loss_table, int32_t* idx_work, int64_t* rounds_out) {
    if (!ctx) return BLS_EINVAL;
    if (rounds_out) *rounds_out = 0;
    if (!model || !plan) return bls_fail(ctx, BLS_EINVAL, "train_epochs: model or plan is NULL");
    const int P = plan->P_f + plan->P_s;
    if (plan->epochs < 0 || plan->P_f < 1 || plan->P_s < 0 || P > 64 || plan->batch < 1 || plan->n_milestones < 0 ||
        (plan->n_milestones > 0 && !plan->milestones) || !isfinite(plan->lr_gamma) || !isfinite(plan->opt.lr))
        return bls_fail(ctx, BLS_EINVAL, "train_epochs: need epochs >= 0, 1 <= P_f, 0 <= P_s, P_f + P_s <= 64, batch >= 1 and a finite schedule");
    int64_t nf = 0, k = 0, ns = 0;
    if (bls_epoch_allocation(N, plan->tau_f, plan->P_f, plan->tau_s, plan->P_s, plan->lambda, &nf, &k, &ns) != BLS_OK)
        return bls_fail(ctx, BLS_EINVAL, "train_epochs: allocation arguments out of range (see bls_epoch_allocation)");
    if (plan->epochs == 0 || N == 0) return BLS_OK;
    if (!global_params || !worker_params || !worker_momentum || !x_pool || !y_pool || !loss_table || !idx_work ||
        (model->num_buffers > 0 && (!global_buffers || !worker_buffers)))
        return bls_fail(ctx, BLS_EINVAL, "train_epochs: NULL pointer");
    const int64_t d = model->num_params, nb = model->num_buffers;
    // worker p's share of its group's list and the rounds needed to consume it at tau * batch samples per round
    int64_t share_off[64], share_len[64], tau[64], rounds = 0;
    for (int p = 0; p < P; ++p) {
        const bool fast = p < plan->P_f;
        int64_t off = 0, cnt = 0;
        bls_worker_share(fast ? nf : ns, fast ? plan->P_f : plan->P_s, fast ? p : p - plan->P_f, &off, &cnt);
        share_off[p] = (fast ? 0 : nf) + off;
        share_len[p] = cnt;
        tau[p] = fast ? plan->tau_f : plan->tau_s;
        if (tau[p] > 0 && cnt > 0) {
            const int64_t per_round = tau[p] * plan->batch, need = (cnt + per_round - 1) / per_round;
            if (need > rounds) rounds = need;
        }
    }
    int64_t rounds_run = 0;
    for (int64_t e = 0; e < plan->epochs; ++e) {
        int reached = 0;
        for (int m = 0; m < plan->n_milestones; ++m)
            if (plan->milestones[m] <= e) ++reached;
        bls_sgd opt = plan->opt;
        opt.lr = (float)((double)plan->opt.lr * pow((double)plan->lr_gamma, (double)reached));
        int rc = sample_epoch_variant(ctx, loss_table, u_fast ? u_fast + e * N : nullptr, u_slow ? u_slow + e * N : nullptr, N, plan->tau_f, plan->P_f,
                                      plan->tau_s, plan->P_s, plan->lambda, plan->scheme, plan->high_loss_to, idx_work, idx_work + nf);
        if (rc != BLS_OK) return rc;
        for (int64_t r = 0; r < rounds; ++r) {
            bls_worker ws[64];
            for (int p = 0; p < P; ++p) {
                const int64_t per_round = tau[p] * plan->batch, start = r * per_round;
                const int64_t hand = tau[p] > 0 && start < share_len[p] ? (share_len[p] - start < per_round ? share_len[p] - start : per_round) : 0;
                ws[p].tau = hand > 0 ? tau[p] : 0;
                ws[p].idx = idx_work + share_off[p] + start;
                ws[p].n_idx = hand;
                ws[p].params = worker_params + (int64_t)p * d;
                ws[p].buffers = nb > 0 ? worker_buffers + (int64_t)p * nb : nullptr;
                ws[p].momentum = worker_momentum + (int64_t)p * d;
            }
            rc = communication_round(ctx, model, global_params, global_buffers, ws, P, x_pool, y_pool, N, plan->batch, &opt, loss_table,
                                     plan->round_flags);
            if (rc != BLS_OK) return rc;
            ++rounds_run;
        }
    }
    if (rounds_out) *rounds_out = rounds_run;
    return BLS_OK;
}

int bls_sum_limits(double* forward_partial, double* backward_partial, double* weight_gradient_partial) {
    if (forward_partial) *forward_partial = 2.0 * FIX_PARTIAL_LIMIT / FIX_FWD_SCALE;   // the convolution's epilogue (half as many workgroups per word)
    if (backward_partial) *backward_partial = FIX_PARTIAL_LIMIT / FIX_BWD_SCALE;
    if (weight_gradient_partial) *weight_gradient_partial = FIX_PARTIAL_LIMIT / 1099511627776.0;   // the weight-gradient kernels' 2^40
    return BLS_OK;
}

int bls_weights_from_tau(const int64_t* tau, int P, float* weights_out) {
    if (!tau || !weights_out || P < 1) return BLS_EINVAL;
    double sum = 0.0;
    for (int i = 0; i < P; ++i) {
        if (tau[i] < 0) return BLS_EINVAL;
        sum += (double)tau[i];
    }
    if (!(sum > 0.0)) return BLS_EINVAL;
    for (int i = 0; i < P; ++i) weights_out[i] = (float)((double)tau[i] / sum);
    return BLS_OK;
}

}  // extern "C"
#pragma GCC visibility pop
