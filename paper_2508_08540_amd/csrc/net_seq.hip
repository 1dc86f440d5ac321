// Transformer encoder language model: scoring and local SGD steps.  Every matrix product (linear layers, attention
// scores, attention-weighted values, their gradients and the weight gradients) is one launch of the tiled MFMA GEMM;
// the kernels of seq.hip do the rest.  Activations are fp32 [tokens][width], heads are column slices of width D/H.
#include "kernels.h"
#include "net.h"

#define PROF(ctx, cls, call) \
    do {                     \
        ProfScope prof_(ctx, cls); \
        call;                \
    } while (0)

namespace {

constexpr int SCORE_SEQS = 128;  // sequences scored together: 16384 tokens fill the chip in every product (logits: 2 GiB at a 32000-word vocabulary)

struct LayerAct {
    float *q, *k, *v, *p, *ctx, *r1, *st1, *h1, *u, *g, *r2, *st2;
};

struct SeqScratch {
    int32_t *tok, *tgt;
    std::vector<float*> x;          // x[l] is the input of layer l, x[layers] the encoder output
    std::vector<LayerAct> act;      // one per layer when training, one shared set when scoring
    float *logits, *tok_loss, *loss;
    // training only
    float *grad, *da, *db, *dc, *dq, *dk, *dv, *df, *ds, *part, *cpart;
    fixsum_t* acc;
    int64_t acc_count;
    size_t part_floats;
};

// Splits of the token contraction of a weight gradient so that about two waves of workgroups are in flight.
int wgrad_splits(int M, int N, int64_t K) {
    const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 128);
    int64_t s = ceil_div(512, tiles);
    const int64_t max_s = K / 256 > 1 ? K / 256 : 1;
    if (s > max_s) s = max_s;
    if (s > 64) s = 64;
    return (int)s;
}

SeqScratch carve(Carver& c, const bls_model* m, int B, bool train) {
    const int L = m->enc_L, D = m->enc_D, H = m->enc_H, F = m->enc_F, V = m->enc_V, layers = (int)m->enc_layers.size();
    const int64_t T = (int64_t)B * L;
    SeqScratch s{};
    s.tok = c.take<int32_t>(T);
    s.tgt = c.take<int32_t>(T);
    const int sets = train ? layers : 1;
    s.x.resize(layers + 1);
    for (int l = 0; l <= layers; ++l) s.x[l] = (train || l < 2) ? c.take<float>(T * D) : s.x[l - 2];
    s.act.resize(layers);
    for (int l = 0; l < layers; ++l) {
        if (l >= sets) {
            s.act[l] = s.act[0];
            continue;
        }
        LayerAct& a = s.act[l];
        a.q = c.take<float>(T * D);
        a.k = c.take<float>(T * D);
        a.v = c.take<float>(T * D);
        a.p = c.take<float>((int64_t)B * H * L * L);
        a.ctx = c.take<float>(T * D);
        a.r1 = c.take<float>(T * D);
        a.st1 = c.take<float>(2 * T);
        a.h1 = c.take<float>(T * D);
        a.u = c.take<float>(T * F);
        a.g = c.take<float>(T * F);
        a.r2 = c.take<float>(T * D);
        a.st2 = c.take<float>(2 * T);
    }
    s.logits = c.take<float>(T * V);
    s.tok_loss = c.take<float>(T);
    s.loss = c.take<float>(B);
    if (!train) return s;
    s.grad = c.take<float>(m->num_params);
    s.da = c.take<float>(T * D);
    s.db = c.take<float>(T * D);
    s.dc = c.take<float>(T * D);
    s.dq = c.take<float>(T * D);
    s.dk = c.take<float>(T * D);
    s.dv = c.take<float>(T * D);
    s.df = c.take<float>(T * F);
    s.ds = c.take<float>((int64_t)B * H * L * L);
    size_t part = 0;
    auto need = [&](int M, int N) {
        const size_t f = gemm_tiled_partial_floats(M, N, wgrad_splits(M, N, T));
        part = f > part ? f : part;
    };
    need(D, D);
    need(F, D);
    need(D, F);
    need(V, D);
    s.part_floats = part;
    s.part = c.take<float>(part ? part : 1);
    size_t cs = colsum_partial_floats(T, F > D ? F : D);
    const size_t ln = layernorm_bwd_partial_floats(T, D), pos = colsum_partial_floats(B, L * D);
    cs = cs > ln ? cs : ln;
    s.cpart = c.take<float>(cs > pos ? cs : pos);
    s.acc_count = (int64_t)V * D;   // fixed-point accumulators of the token-embedding gradient
    s.acc = c.take<fixsum_t>(s.acc_count);
    return s;
}

size_t scratch_bytes(const bls_model* m, int B, bool train) {
    Carver c(nullptr);
    carve(c, m, B, train);
    return c.off;
}

// y[T][n_out] = x[T][n_in] W^T + b (+ R)
void linear(bls_ctx* ctx, hipStream_t st, int bf16, const float* x, int64_t T, int n_in, const float* W, const float* b, int n_out, float* y,
            const float* R = nullptr, float* gelu_out = nullptr) {
    GemmDesc d{};
    d.A = x; d.lda = n_in;
    d.B = W; d.ldb = n_in;
    d.C = y; d.ldc = n_out;
    d.bias = b; d.R = R; d.G = gelu_out;
    d.M = (int)T; d.N = n_out; d.K = n_in;
    d.alpha = 1.f;
    d.bf16 = bf16;
    PROF(ctx, PROF_GEMM, launch_gemm_tiled(st, d));
}

// dx[T][n_in] = dy[T][n_out] W (+ R)
void linear_dgrad(bls_ctx* ctx, hipStream_t st, int bf16, const float* dy, int64_t T, int n_out, const float* W, int n_in, float* dx,
                  const float* R = nullptr) {
    GemmDesc d{};
    d.A = dy; d.lda = n_out;
    d.B = W; d.ldb = n_in; d.b_kmajor = 1;
    d.C = dx; d.ldc = n_in;
    d.R = R;
    d.M = (int)T; d.N = n_in; d.K = n_out;
    d.alpha = 1.f;
    d.bf16 = bf16;
    PROF(ctx, PROF_GEMM, launch_gemm_tiled(st, d));
}

// dW[n_out][n_in] = dy^T x, contraction over the T tokens
void linear_wgrad(bls_ctx* ctx, hipStream_t st, int bf16, const float* dy, const float* x, int64_t T, int n_out, int n_in, float* dW, float* part) {
    GemmDesc d{};
    d.A = dy; d.lda = n_out; d.a_kmajor = 1;
    d.B = x; d.ldb = n_in; d.b_kmajor = 1;
    d.C = dW; d.ldc = n_in;
    d.M = n_out; d.N = n_in; d.K = (int)T;
    d.alpha = 1.f;
    d.bf16 = bf16;
    d.splits = wgrad_splits(n_out, n_in, T);
    d.part = part;
    PROF(ctx, PROF_CONV_WGRAD, launch_gemm_tiled(st, d));
}

// Batched product over (sample, head): matrices are slices of [T][D] activations (row pitch D, head offset D/H) or of
// the [B][H][L][L] probability tensor.
struct Slice {
    const float* p;
    bool probs;    // [B][H][L][L] tensor, otherwise [T][D] activation
    bool kmajor;
};
void attention_gemm(bls_ctx* ctx, hipStream_t st, const bls_model* m, int B, Slice a, Slice b, float* c, bool c_probs, int N, int K,
                    float alpha) {
    const int L = m->enc_L, D = m->enc_D, H = m->enc_H, dh = D / H;
    GemmDesc d{};
    auto strides = [&](bool probs, int& ld, int64_t& s1, int64_t& s2) {
        ld = probs ? L : D;
        s1 = probs ? (int64_t)H * L * L : (int64_t)L * D;
        s2 = probs ? (int64_t)L * L : dh;
    };
    d.A = a.p; d.a_kmajor = a.kmajor ? 1 : 0; strides(a.probs, d.lda, d.sa1, d.sa2);
    d.B = b.p; d.b_kmajor = b.kmajor ? 1 : 0; strides(b.probs, d.ldb, d.sb1, d.sb2);
    d.C = c; strides(c_probs, d.ldc, d.sc1, d.sc2);
    d.M = L; d.N = N; d.K = K;
    d.batch = B * H; d.inner = H;
    d.alpha = alpha;
    d.bf16 = m->desc.act_dtype == BLS_ACT_BF16 ? 1 : 0;
    PROF(ctx, PROF_GEMM, launch_gemm_tiled(st, d));
}

__global__ __launch_bounds__(256) void gather_sequences_kernel(const int32_t* __restrict__ x, const int32_t* __restrict__ y,
                                                               const int32_t* __restrict__ sel, int64_t k, int64_t start, int L,
                                                               int32_t* __restrict__ tok, int32_t* __restrict__ tgt) {
    const int b = blockIdx.x;
    const int64_t src = sel[(start + b) % k];
    for (int l = threadIdx.x; l < L; l += 256) {
        tok[(int64_t)b * L + l] = x[src * L + l];
        tgt[(int64_t)b * L + l] = y[src * L + l];
    }
}

// Encoder output for the tokens in `tok`; with keep the per-layer activations stay for the backward pass.
void forward(bls_ctx* ctx, hipStream_t st, const bls_model* m, const float* params, const int32_t* tok, int B, SeqScratch& s, bool keep) {
    const int L = m->enc_L, D = m->enc_D, H = m->enc_H, F = m->enc_F, dh = D / H;
    const int bf = m->desc.act_dtype == BLS_ACT_BF16 ? 1 : 0;
    const int64_t T = (int64_t)B * L;
    PROF(ctx, PROF_GATHER, launch_embed(st, tok, T, L, D, params + m->enc_tok, params + m->enc_pos, s.x[0]));
    for (size_t l = 0; l < m->enc_layers.size(); ++l) {
        const EncLayer& e = m->enc_layers[l];
        const LayerAct& a = s.act[l];
        const float* x = s.x[l];
        linear(ctx, st, bf, x, T, D, params + e.wq, params + e.bq, D, a.q);
        linear(ctx, st, bf, x, T, D, params + e.wk, params + e.bk, D, a.k);
        linear(ctx, st, bf, x, T, D, params + e.wv, params + e.bv, D, a.v);
        attention_gemm(ctx, st, m, B, {a.q, false, false}, {a.k, false, false}, a.p, true, L, dh, 1.f / sqrtf((float)dh));
        PROF(ctx, PROF_NORM, launch_softmax_rows(st, a.p, (int64_t)B * H * L, L));
        attention_gemm(ctx, st, m, B, {a.p, true, false}, {a.v, false, true}, a.ctx, false, dh, L, 1.f);
        linear(ctx, st, bf, a.ctx, T, D, params + e.wo, params + e.bo, D, a.r1, x);
        PROF(ctx, PROF_NORM, launch_layernorm(st, a.r1, T, D, params + e.ln1_g, params + e.ln1_b, a.h1, keep ? a.st1 : nullptr));
        // u = h1 W1^T + b1 and g = gelu(u) from one epilogue; scoring does not keep u
        linear(ctx, st, bf, a.h1, T, D, params + e.w1, params + e.b1, F, keep ? a.u : nullptr, nullptr, a.g);
        linear(ctx, st, bf, a.g, T, F, params + e.w2, params + e.b2, D, a.r2, a.h1);
        PROF(ctx, PROF_NORM, launch_layernorm(st, a.r2, T, D, params + e.ln2_g, params + e.ln2_b, s.x[l + 1], keep ? a.st2 : nullptr));
    }
}

}  // namespace

int seq_score(bls_ctx* ctx, const bls_model* m, const float* params, const int32_t* x, const int32_t* y, int64_t N, float* losses_out) {
    const int chunk = (int)(N < SCORE_SEQS ? N : SCORE_SEQS);
    int rc = bls_arena_reserve(ctx, scratch_bytes(m, chunk, false));
    if (rc != BLS_OK) return rc;
    hipStream_t st = ctx->stream;
    Carver c(ctx->arena);
    SeqScratch s = carve(c, m, chunk, false);
    const int L = m->enc_L, D = m->enc_D, V = m->enc_V, layers = (int)m->enc_layers.size();
    const int bf = m->desc.act_dtype == BLS_ACT_BF16 ? 1 : 0;
    for (int64_t first = 0; first < N; first += chunk) {
        const int B = (int)(N - first < chunk ? N - first : chunk);
        const int64_t T = (int64_t)B * L;
        forward(ctx, st, m, params, x + first * L, B, s, false);
        linear(ctx, st, bf, s.x[layers], T, D, params + m->enc_head, nullptr, V, s.logits);
        PROF(ctx, PROF_HEAD, launch_token_ce(st, s.logits, y + first * L, T, V, s.tok_loss, 0.f));
        PROF(ctx, PROF_HEAD, launch_sample_mean(st, s.tok_loss, B, L, losses_out + first));
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

int seq_local_step(bls_ctx* ctx, const bls_model* m, float* params, float* momentum, const int32_t* x_pool, const int32_t* y_pool, int64_t N,
                   const int32_t* sel, int64_t k, int64_t batch, int64_t tau, const bls_sgd& opt, float* step_losses_out) {
    (void)N;
    const int B = (int)batch;
    const int L = m->enc_L, D = m->enc_D, H = m->enc_H, F = m->enc_F, V = m->enc_V, dh = D / H, layers = (int)m->enc_layers.size();
    if (m->enc_layers[0].ln1_b != m->enc_layers[0].ln1_g + D || m->enc_layers[0].ln2_b != m->enc_layers[0].ln2_g + D)
        return bls_fail(ctx, BLS_EUNSUPPORTED, "local_step: layer-norm scale and shift must be adjacent");
    const int bf = m->desc.act_dtype == BLS_ACT_BF16 ? 1 : 0;
    const int64_t T = (int64_t)B * L;
    if (T >= (int64_t(1) << 31) / 2 || T * (int64_t)V >= (int64_t(1) << 40))
        return bls_fail(ctx, BLS_EINVAL, "local_step: batch * sequence length too large");
    int rc = bls_arena_reserve(ctx, scratch_bytes(m, B, true));
    if (rc != BLS_OK) return rc;
    hipStream_t st = ctx->stream;
    Carver c(ctx->arena);
    SeqScratch s = carve(c, m, B, true);

    FixRangeTable emb_tab{};
    emb_tab.n = 1;
    emb_tab.r[0] = {0, m->enc_tok, (int64_t)V * D};
    PROF(ctx, PROF_UPDATE, launch_fill_zero(st, reinterpret_cast<float*>(s.acc), s.acc_count * 2));
    const float gscale = 1.f / (float)T;   // mean over the batch of per-sample means over positions
    const float att = 1.f / sqrtf((float)dh);

    for (int64_t j = 0; j < tau; ++j) {
        {
            ProfScope prof(ctx, PROF_GATHER);
            hipLaunchKernelGGL(gather_sequences_kernel, dim3(B), dim3(256), 0, st, x_pool, y_pool, sel, k, j * B, L, s.tok, s.tgt);
        }
        forward(ctx, st, m, params, s.tok, B, s, true);
        const float* hf = s.x[layers];
        linear(ctx, st, bf, hf, T, D, params + m->enc_head, nullptr, V, s.logits);
        PROF(ctx, PROF_HEAD, launch_token_ce(st, s.logits, s.tgt, T, V, s.tok_loss, gscale));
        PROF(ctx, PROF_HEAD, launch_sample_mean(st, s.tok_loss, B, L, step_losses_out ? step_losses_out + j * B : s.loss));
        // head
        linear_wgrad(ctx, st, bf, s.logits, hf, T, V, D, s.grad + m->enc_head, s.part);
        linear_dgrad(ctx, st, bf, s.logits, T, V, params + m->enc_head, D, s.da);
        for (int l = layers - 1; l >= 0; --l) {
            const EncLayer& e = m->enc_layers[l];
            const LayerAct& a = s.act[l];
            const float* x = s.x[l];
            // h = LN2(r2): da holds dh, db receives dr2
            PROF(ctx, PROF_NORM, launch_layernorm_bwd(st, s.da, a.r2, a.st2, T, D, params + e.ln2_g, s.db, s.cpart, s.grad + e.ln2_g));
            // r2 = h1 + g W2^T + b2
            linear_wgrad(ctx, st, bf, s.db, a.g, T, D, F, s.grad + e.w2, s.part);
            PROF(ctx, PROF_NORM, launch_colsum_tokens(st, s.db, T, D, s.cpart, s.grad + e.b2));
            linear_dgrad(ctx, st, bf, s.db, T, D, params + e.w2, F, s.df);
            PROF(ctx, PROF_NORM, launch_gelu_bwd(st, s.df, a.u, T * F));
            // u = h1 W1^T + b1
            linear_wgrad(ctx, st, bf, s.df, a.h1, T, F, D, s.grad + e.w1, s.part);
            PROF(ctx, PROF_NORM, launch_colsum_tokens(st, s.df, T, F, s.cpart, s.grad + e.b1));
            linear_dgrad(ctx, st, bf, s.df, T, F, params + e.w1, D, s.da, s.db);   // da = dh1 (both uses of h1)
            // h1 = LN1(r1): db receives dr1
            PROF(ctx, PROF_NORM, launch_layernorm_bwd(st, s.da, a.r1, a.st1, T, D, params + e.ln1_g, s.db, s.cpart, s.grad + e.ln1_g));
            // r1 = x + ctx Wo^T + bo
            linear_wgrad(ctx, st, bf, s.db, a.ctx, T, D, D, s.grad + e.wo, s.part);
            PROF(ctx, PROF_NORM, launch_colsum_tokens(st, s.db, T, D, s.cpart, s.grad + e.bo));
            linear_dgrad(ctx, st, bf, s.db, T, D, params + e.wo, D, s.dc);          // dc = dctx
            // ctx = P v;  P = softmax(att * q k^T)
            attention_gemm(ctx, st, m, B, {a.p, true, true}, {s.dc, false, true}, s.dv, false, dh, L, 1.f);      // dv = P^T dctx
            attention_gemm(ctx, st, m, B, {s.dc, false, false}, {a.v, false, false}, s.ds, true, L, dh, 1.f);    // dP = dctx v^T
            PROF(ctx, PROF_NORM, launch_softmax_bwd_rows(st, s.ds, a.p, (int64_t)B * H * L, L, att));
            attention_gemm(ctx, st, m, B, {s.ds, true, false}, {a.k, false, true}, s.dq, false, dh, L, 1.f);     // dq = dS k
            attention_gemm(ctx, st, m, B, {s.ds, true, true}, {a.q, false, true}, s.dk, false, dh, L, 1.f);      // dk = dS^T q
            // q, k, v projections of x
            linear_wgrad(ctx, st, bf, s.dq, x, T, D, D, s.grad + e.wq, s.part);
            linear_wgrad(ctx, st, bf, s.dk, x, T, D, D, s.grad + e.wk, s.part);
            linear_wgrad(ctx, st, bf, s.dv, x, T, D, D, s.grad + e.wv, s.part);
            PROF(ctx, PROF_NORM, launch_colsum_tokens(st, s.dq, T, D, s.cpart, s.grad + e.bq));
            PROF(ctx, PROF_NORM, launch_colsum_tokens(st, s.dk, T, D, s.cpart, s.grad + e.bk));
            PROF(ctx, PROF_NORM, launch_colsum_tokens(st, s.dv, T, D, s.cpart, s.grad + e.bv));
            linear_dgrad(ctx, st, bf, s.dq, T, D, params + e.wq, D, s.da, s.db);    // da = dx, starting from the residual path
            linear_dgrad(ctx, st, bf, s.dk, T, D, params + e.wk, D, s.da, s.da);
            linear_dgrad(ctx, st, bf, s.dv, T, D, params + e.wv, D, s.da, s.da);
        }
        // embeddings: position gradient = sum over samples, token gradient = scatter by id
        PROF(ctx, PROF_NORM, launch_colsum_tokens(st, s.da, B, L * D, s.cpart, s.grad + m->enc_pos));
        PROF(ctx, PROF_NORM, launch_embed_grad(st, s.tok, T, D, s.da, s.acc));
        PROF(ctx, PROF_UPDATE, launch_fix_finalize(st, emb_tab, s.acc, s.grad));
        PROF(ctx, PROF_UPDATE, launch_sgd(st, params, momentum, s.grad, m->num_params, opt.lr, opt.momentum, opt.weight_decay));
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
