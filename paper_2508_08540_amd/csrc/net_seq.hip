// Transformer encoder language model: scoring and local SGD steps.  Every matrix product (linear layers, attention
// scores, attention-weighted values, their gradients and the weight gradients) is one launch of a tiled MFMA GEMM;
// the kernels of seq.hip do the rest.  Activations are [tokens][width], heads are column slices of width D/H.
//
// Two modes.  fp32: every tensor is fp32 and the products run on the fp32 matrix instruction.  bf16 factors: every
// tensor that is a factor of some product also (or only) exists as a bf16 copy, written by the kernel that produces
// it, and the products read those copies (bf16 matrix instruction, fp32 sums); everything that is not a product -
// residual sums, layer norm, softmax, GELU derivative, bias and layer-norm gradients, the loss, the parameters and
// their update - reads and writes fp32.  Tensors that are only ever factors (q, k, v, the attention output, GELU
// output, the gradients of the attention output, of the scores and of the logits) exist in bf16 alone.
#include "kernels.h"
#include "net.h"

#define PROF(ctx, cls, call) \
    do {                     \
        ProfScope prof_(ctx, cls); \
        call;                \
    } while (0)

namespace {

// Tokens scored together.  65536 give every product of the bf16 mode at least two rounds of workgroups, so that the first
// loads and the epilogue of one tile overlap the K loop of another; the fp32 mode stores the logits of a chunk
// (4 GiB at 32768 tokens and a 32000-word vocabulary) and keeps their element offsets below 2^31.
constexpr int64_t SCORE_TOKENS_BF16 = 65536, SCORE_TOKENS_F32 = 32768;
int score_chunk(const bls_model* m, int64_t N) {
    const bool bf = m->desc.act_dtype == BLS_ACT_BF16;
    int64_t tokens = bf ? SCORE_TOKENS_BF16 : SCORE_TOKENS_F32;
    if (!bf && tokens * m->enc_V >= (int64_t(1) << 31)) tokens = ((int64_t(1) << 31) - 1) / m->enc_V;
    int64_t seqs = tokens / m->enc_L;
    if (seqs < 1) seqs = 1;
    return (int)(N < seqs ? N : seqs);
}

// A tensor as fp32 (f), as bf16 (h), or both; a NULL member does not exist in this mode.
struct Mat {
    float* f = nullptr;
    uint16_t* h = nullptr;
};

struct LayerAct {
    Mat q, k, v, p, ctx, h1, g;
    float *r1, *st1, *u, *r2, *st2;
};

struct SeqScratch {
    bool bf = false;
    int32_t *tok, *tgt;
    uint16_t* w16;                  // bf16 copy of the parameter vector (bf16 mode)
    std::vector<Mat> x;             // x[l] is the input of layer l, x[layers] the encoder output
    std::vector<LayerAct> act;      // one per layer when training, one shared set when scoring
    float *logits, *tok_loss, *loss;
    float *ce_part, *ce_tlogit, *ce_rows;   // bf16 mode: softmax statistics left by the vocabulary projection
    int ce_parts;
    // training only
    Mat dlogits;                    // fp32 mode: the logits buffer itself
    Mat dc, ds;                     // gradient of the attention output, of the scores (unfused attention only)
    // gradients that weight-gradient products read on the side stream: one buffer per layer, so that nothing they read is
    // overwritten before the streams join.  db2 / db1 = gradient of the input of the second / first layer norm
    std::vector<Mat> db2, db1, df, dq, dk, dv;
    float *grad, *da, *part, *part_main, *cpart;   // part: split-K partial sums of the side stream, part_main: of the main stream
    size_t cpart_floats;
    fixsum_t* acc;
    int64_t acc_count;
};

// Splits of the token contraction of a weight gradient so that about two waves of workgroups are in flight.
int wgrad_splits(int M, int N, int64_t K, int batch = 1) {
    const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 128) * batch;
    int64_t s = ceil_div(512, tiles);
    const int64_t max_s = K / 256 > 1 ? K / 256 : 1;
    if (s > max_s) s = max_s;
    if (s > 64) s = 64;
    return (int)s;
}

// Splits of a long contraction whose output has too few tiles to keep three workgroups on every compute unit (what
// hides the load latency of the K loop); only for fp32 outputs, since the partial sums are added by a second kernel.
#define DGRAD_SPLIT_MIN_K 4096
int dgrad_splits(int64_t M, int N, int K) {
    const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 128);
    if (K < DGRAD_SPLIT_MIN_K || tiles >= 512) return 1;
    int64_t s = ceil_div(768, tiles);
    if (s > K / 1024) s = K / 1024;
    return (int)(s > 1 ? s : 1);
}

enum Kind { F32_ONLY, BOTH, FACTOR_ONLY };   // FACTOR_ONLY: fp32 in fp32 mode, bf16 alone in bf16 mode

Mat take(Carver& c, bool bf, Kind kind, int64_t n) {
    Mat m;
    if (!bf || kind != FACTOR_ONLY) m.f = c.take<float>(n);
    if (bf && kind != F32_ONLY) m.h = c.take<uint16_t>(n);
    return m;
}

// Three tensors of n elements each, exactly n apart (one product can then run over all three as a batch)
void take3(Carver& c, bool bf, Kind kind, int64_t n, Mat& a, Mat& b, Mat& d) {
    const Mat all = take(c, bf, kind, 3 * n);
    a = all;
    b = Mat{all.f ? all.f + n : nullptr, all.h ? all.h + n : nullptr};
    d = Mat{all.f ? all.f + 2 * n : nullptr, all.h ? all.h + 2 * n : nullptr};
}

SeqScratch carve(Carver& c, const bls_model* m, int B, bool train) {
    const int L = m->enc_L, D = m->enc_D, H = m->enc_H, F = m->enc_F, V = m->enc_V, layers = (int)m->enc_layers.size();
    const int64_t T = (int64_t)B * L, PP = (int64_t)B * H * L * L;
    SeqScratch s{};
    const bool bf = s.bf = m->desc.act_dtype == BLS_ACT_BF16;
    s.tok = c.take<int32_t>(T);
    s.tgt = c.take<int32_t>(T);
    s.w16 = bf ? c.take<uint16_t>(m->num_params) : nullptr;
    const int sets = train ? layers : 1;
    s.x.resize(layers + 1);
    for (int l = 0; l <= layers; ++l) s.x[l] = (train || l < 2) ? take(c, bf, BOTH, T * D) : s.x[l - 2];
    s.act.resize(layers);
    for (int l = 0; l < layers; ++l) {
        if (l >= sets) {
            s.act[l] = s.act[0];
            continue;
        }
        LayerAct& a = s.act[l];
        take3(c, bf, FACTOR_ONLY, T * D, a.q, a.k, a.v);
        a.p = take(c, bf, BOTH, PP);
        a.ctx = take(c, bf, FACTOR_ONLY, T * D);
        a.r1 = c.take<float>(T * D);
        a.st1 = c.take<float>(2 * T);
        a.h1 = take(c, bf, BOTH, T * D);
        a.u = c.take<float>(T * F);
        a.g = take(c, bf, FACTOR_ONLY, T * F);
        a.r2 = c.take<float>(T * D);
        a.st2 = c.take<float>(2 * T);
    }
    // bf16 mode: the vocabulary projection leaves row statistics behind and scoring never stores the logits
    s.logits = (bf && !train) ? nullptr : c.take<float>(T * V);
    s.ce_parts = 2 * (int)ceil_div(V, 128);
    s.ce_part = bf ? c.take<float>(T * s.ce_parts * 2) : nullptr;
    s.ce_tlogit = bf ? c.take<float>(T) : nullptr;
    s.ce_rows = bf ? c.take<float>(2 * T) : nullptr;
    s.tok_loss = c.take<float>(T);
    s.loss = c.take<float>(B);
    if (!train) return s;
    if (bf) s.dlogits.h = c.take<uint16_t>(T * V);
    else s.dlogits.f = s.logits;
    s.grad = c.take<float>(m->num_params);
    s.da = c.take<float>(T * D);
    s.dc = take(c, bf, FACTOR_ONLY, T * D);
    s.ds = take(c, bf, BOTH, PP);
    s.db2.resize(layers); s.db1.resize(layers); s.df.resize(layers); s.dq.resize(layers); s.dk.resize(layers); s.dv.resize(layers);
    for (int l = 0; l < layers; ++l) {
        s.db2[l] = take(c, bf, BOTH, T * D);
        s.db1[l] = take(c, bf, BOTH, T * D);
        s.df[l] = take(c, bf, BOTH, T * F);
        take3(c, bf, BOTH, T * D, s.dq[l], s.dk[l], s.dv[l]);
    }
    size_t part = 0;
    auto need = [&](int M, int N) {
        const size_t f = gemm_tiled_partial_floats(M, N, wgrad_splits(M, N, T));
        part = f > part ? f : part;
    };
    need(D, D);
    {
        const size_t f = 3 * gemm_tiled_partial_floats(D, D, wgrad_splits(D, D, T, 3));
        part = f > part ? f : part;
    }
    need(F, D);
    need(D, F);
    need(V, D);
    s.part = c.take<float>(part ? part : 1);
    part = 0;
    for (int n_out : {D, F, V})
        for (int n_in : {D, F}) {
            const size_t f = gemm_tiled_partial_floats((int)T, n_in, dgrad_splits(T, n_in, n_out));
            part = f > part ? f : part;
        }
    s.part_main = c.take<float>(part ? part : 1);
    // partial column sums of one backward pass: per layer five D-wide and one F-wide bias gradient and two layer norms
    const size_t per_layer = 3 * colsum_partial_floats(T, D) + colsum_partial_floats(T, F) + gelu_bwd_colsum_floats(T, F) + 2 * layernorm_bwd_partial_floats(T, D) + (size_t)12 * B * D;
    const size_t pos = colsum_partial_floats(B, L * D);
    s.cpart_floats = per_layer * layers > pos ? per_layer * layers : pos;
    s.cpart = c.take<float>(s.cpart_floats);
    s.acc_count = (int64_t)V * D;   // fixed-point accumulators of the token-embedding gradient
    s.acc = c.take<fixsum_t>(s.acc_count);
    return s;
}

size_t scratch_bytes(const bls_model* m, int B, bool train) {
    Carver c(nullptr);
    carve(c, m, B, train);
    return c.off;
}

// One product C = alpha * A B^T (+ bias) (+ R) in the mode of the scratch: fp32 members and the fp32 GEMM, or bf16
// members and the bf16 GEMM.  out takes the result in every form it has; gelu (optional) takes gelu(result).
struct Product {
    Mat A, B, out, gelu;
    const float *bias = nullptr, *R = nullptr;
    float* part = nullptr;
    int M = 0, N = 0, K = 0, lda = 0, ldb = 0, ldc = 0;
    bool a_kmajor = false, b_kmajor = false;
    int batch = 1, inner = 1, splits = 1;
    int64_t sa1 = 0, sa2 = 0, sb1 = 0, sb2 = 0, sc1 = 0, sc2 = 0, sbias1 = 0;
    float alpha = 1.f;
    const int32_t* ce_targets = nullptr;   // bf16 mode only: leave softmax statistics of the rows behind
    float *ce_part = nullptr, *ce_tlogit = nullptr;
};

void multiply(bls_ctx* ctx, hipStream_t st, bool bf, const Product& p, int prof_class) {
    ProfScope prof(ctx, prof_class, st);
    if (bf) {
        Gemm16Desc d{};
        d.A = p.A.h; d.B = p.B.h; d.C = p.out.f; d.C16 = p.out.h; d.G16 = p.gelu.h;
        d.bias = p.bias; d.R = p.R; d.part = p.part;
        d.M = p.M; d.N = p.N; d.K = p.K; d.lda = p.lda; d.ldb = p.ldb; d.ldc = p.ldc;
        d.a_kmajor = p.a_kmajor; d.b_kmajor = p.b_kmajor;
        d.batch = p.batch; d.inner = p.inner; d.splits = p.splits;
        d.sa1 = p.sa1; d.sa2 = p.sa2; d.sb1 = p.sb1; d.sb2 = p.sb2; d.sc1 = p.sc1; d.sc2 = p.sc2;
        d.sbias1 = p.sbias1;
        d.alpha = p.alpha;
        d.ce_part = p.ce_part; d.ce_targets = p.ce_targets; d.ce_tlogit = p.ce_tlogit;
        launch_gemm16(st, d);
    } else {
        GemmDesc d{};
        d.A = p.A.f; d.B = p.B.f; d.C = p.out.f; d.G = p.gelu.f;
        d.bias = p.bias; d.R = p.R; d.part = p.part;
        d.M = p.M; d.N = p.N; d.K = p.K; d.lda = p.lda; d.ldb = p.ldb; d.ldc = p.ldc;
        d.a_kmajor = p.a_kmajor; d.b_kmajor = p.b_kmajor;
        d.batch = p.batch; d.inner = p.inner; d.splits = p.splits;
        d.sa1 = p.sa1; d.sa2 = p.sa2; d.sb1 = p.sb1; d.sb2 = p.sb2; d.sc1 = p.sc1; d.sc2 = p.sc2;
        d.alpha = p.alpha;
        launch_gemm_tiled(st, d);
    }
}

struct Net {
    bls_ctx* ctx;
    hipStream_t st;
    const bls_model* m;
    const float* params;
    SeqScratch* s;
    int B;

    Mat weight(int64_t off) const { return Mat{const_cast<float*>(params) + off, s->bf ? s->w16 + off : nullptr}; }

    // y[T][n_out] = x[T][n_in] W^T + b (+ R); gelu (optional) takes gelu(y)
    void linear(Mat x, int64_t T, int n_in, int64_t w_off, int64_t b_off, int n_out, Mat y, const float* R = nullptr, Mat gelu = Mat{}) const {
        Product p;
        p.A = x; p.lda = n_in;
        p.B = weight(w_off); p.ldb = n_in;
        p.out = y; p.gelu = gelu; p.ldc = n_out;
        p.bias = b_off >= 0 ? params + b_off : nullptr;
        p.R = R;
        p.M = (int)T; p.N = n_out; p.K = n_in;
        multiply(ctx, st, s->bf, p, PROF_GEMM);
    }
    // Per-token losses of the encoder output hf against `targets`; with keep_logits the logits stay in s->logits (and,
    // in bf16 mode, the row statistics in s->ce_rows) for the gradient.
    void token_losses(Mat hf, const int32_t* targets, int64_t T, bool keep_logits) const {
        const int D = m->enc_D, V = m->enc_V;
        Product p;
        p.A = hf; p.lda = D;
        p.B = weight(m->enc_head); p.ldb = D;
        p.ldc = V;
        p.M = (int)T; p.N = V; p.K = D;
        if (s->bf) {
            p.out.f = keep_logits ? s->logits : nullptr;
            p.ce_part = s->ce_part; p.ce_targets = targets; p.ce_tlogit = s->ce_tlogit;
            multiply(ctx, st, true, p, PROF_GEMM);
            PROF(ctx, PROF_HEAD, launch_ce_combine(st, s->ce_part, s->ce_parts, s->ce_tlogit, T, s->tok_loss, keep_logits ? s->ce_rows : nullptr));
        } else {
            p.out.f = s->logits;
            multiply(ctx, st, false, p, PROF_GEMM);
        }
    }
    // dx[T][n_in] = dy[T][n_out] W (+ R)
    void linear_dgrad(Mat dy, int64_t T, int n_out, int64_t w_off, int n_in, Mat dx, const float* R = nullptr) const {
        Product p;
        p.A = dy; p.lda = n_out;
        p.B = weight(w_off); p.ldb = n_in; p.b_kmajor = true;
        p.out = dx; p.ldc = n_in;
        p.R = R;
        p.M = (int)T; p.N = n_in; p.K = n_out;
        if (s->bf && !dx.h) {
            p.splits = dgrad_splits(T, n_in, n_out);
            p.part = s->part_main;
        }
        multiply(ctx, st, s->bf, p, PROF_GEMM);
    }
    // dW[n_out][n_in] = dy^T x, contraction over the T tokens
    void linear_wgrad(Mat dy, Mat x, int64_t T, int n_out, int n_in, int64_t w_off) const {
        Product p;
        p.A = dy; p.lda = n_out; p.a_kmajor = true;
        p.B = x; p.ldb = n_in; p.b_kmajor = true;
        p.out.f = s->grad + w_off; p.ldc = n_in;
        p.M = n_out; p.N = n_in; p.K = (int)T;
        p.splits = wgrad_splits(n_out, n_in, T);
        p.part = s->part;
        multiply(ctx, st, s->bf, p, PROF_CONV_WGRAD);
    }
    // q, k, v = x Wq^T + bq, ... as one batch of three products where the three weights (and biases, and outputs) are
    // equally spaced; three products otherwise
    void qkv(Mat x, int64_t T, const EncLayer& e, const LayerAct& a) const {
        const int D = m->enc_D;
        const int64_t sw = e.wk - e.wq, so = a.k.h - a.q.h;
        if (s->bf && e.wv - e.wk == sw && e.bk - e.bq == sw && e.bv - e.bk == sw && a.v.h - a.k.h == so) {
            Product p;
            p.A = x; p.lda = D;
            p.B = weight(e.wq); p.ldb = D; p.sb1 = sw;
            p.out = a.q; p.ldc = D; p.sc1 = so;
            p.bias = params + e.bq; p.sbias1 = sw;
            p.M = (int)T; p.N = D; p.K = D;
            p.batch = 3;
            multiply(ctx, st, true, p, PROF_GEMM);
            return;
        }
        linear(x, T, D, e.wq, e.bq, D, a.q);
        linear(x, T, D, e.wk, e.bk, D, a.k);
        linear(x, T, D, e.wv, e.bv, D, a.v);
    }
    // Weight gradients of the same three projections from dq, dk, dv
    void qkv_wgrad(Mat dq, Mat dk, Mat dv, Mat x, int64_t T, const EncLayer& e) const {
        const int D = m->enc_D;
        const int64_t sw = e.wk - e.wq, sd = dk.h - dq.h;
        if (s->bf && e.wv - e.wk == sw && dv.h - dk.h == sd) {
            Product p;
            p.A = dq; p.lda = D; p.a_kmajor = true; p.sa1 = sd;
            p.B = x; p.ldb = D; p.b_kmajor = true;
            p.out.f = s->grad + e.wq; p.ldc = D; p.sc1 = sw;
            p.M = D; p.N = D; p.K = (int)T;
            p.batch = 3;
            p.splits = wgrad_splits(D, D, T, 3);
            p.part = s->part;
            multiply(ctx, st, true, p, PROF_CONV_WGRAD);
            return;
        }
        linear_wgrad(dq, x, T, D, D, e.wq);
        linear_wgrad(dk, x, T, D, D, e.wk);
        linear_wgrad(dv, x, T, D, D, e.wv);
    }
    // Batched product over (sample, head): factors and result are slices of [T][D] activations (row pitch D, head
    // offset D/H) or of a [B][H][L][L] tensor (probs).
    void attention(Mat a, bool a_probs, bool a_kmajor, Mat b, bool b_probs, bool b_kmajor, Mat c, bool c_probs, int N, int K, float alpha) const {
        const int L = m->enc_L, D = m->enc_D, H = m->enc_H, dh = D / H;
        Product p;
        auto strides = [&](bool probs, int& ld, int64_t& s1, int64_t& s2) {
            ld = probs ? L : D;
            s1 = probs ? (int64_t)H * L * L : (int64_t)L * D;
            s2 = probs ? (int64_t)L * L : dh;
        };
        p.A = a; p.a_kmajor = a_kmajor; strides(a_probs, p.lda, p.sa1, p.sa2);
        p.B = b; p.b_kmajor = b_kmajor; strides(b_probs, p.ldb, p.sb1, p.sb2);
        p.out = c; strides(c_probs, p.ldc, p.sc1, p.sc2);
        p.M = L; p.N = N; p.K = K;
        p.batch = B * H; p.inner = H;
        p.alpha = alpha;
        multiply(ctx, st, s->bf, p, PROF_GEMM);
    }

    // Encoder output for the tokens in `tok`; with keep the per-layer activations stay for the backward pass.
    void forward(const int32_t* tok, bool keep) const {
        const int L = m->enc_L, D = m->enc_D, H = m->enc_H, F = m->enc_F, dh = D / H;
        const int64_t T = (int64_t)B * L;
        PROF(ctx, PROF_GATHER, launch_embed(st, tok, T, L, D, params + m->enc_tok, params + m->enc_pos, s->x[0].f, s->x[0].h));
        for (size_t l = 0; l < m->enc_layers.size(); ++l) {
            const EncLayer& e = m->enc_layers[l];
            const LayerAct& a = s->act[l];
            const Mat x = s->x[l];
            qkv(x, T, e, a);
            const float att = 1.f / sqrtf((float)dh);
            bool fused = false;
            if (s->bf) {
                // short sequences: scores, softmax and weighted values of a (sample, head) in one workgroup
                ProfScope prof_(ctx, PROF_GEMM);
                fused = launch_attention16(st, a.q.h, a.k.h, a.v.h, D, B, H, L, dh, att, a.ctx.h, D, keep ? a.p.f : nullptr, keep ? a.p.h : nullptr);
            }
            if (!fused) {
                // scores into the fp32 probability buffer, softmax in place (kept in fp32 only where something reads it)
                attention(a.q, false, false, a.k, false, false, Mat{a.p.f, nullptr}, true, L, dh, att);
                PROF(ctx, PROF_NORM, launch_softmax_rows(st, a.p.f, a.p.h, keep || !s->bf, (int64_t)B * H * L, L));
                attention(a.p, true, false, a.v, false, true, a.ctx, false, dh, L, 1.f);
            }
            linear(a.ctx, T, D, e.wo, e.bo, D, Mat{a.r1, nullptr}, x.f);
            PROF(ctx, PROF_NORM, launch_layernorm(st, a.r1, T, D, params + e.ln1_g, params + e.ln1_b, a.h1.f, a.h1.h, keep ? a.st1 : nullptr));
            // u = h1 W1^T + b1 and g = gelu(u) from one epilogue; scoring does not keep u
            linear(a.h1, T, D, e.w1, e.b1, F, Mat{keep ? a.u : nullptr, nullptr}, nullptr, a.g);
            linear(a.g, T, F, e.w2, e.b2, D, Mat{a.r2, nullptr}, a.h1.f);
            PROF(ctx, PROF_NORM, launch_layernorm(st, a.r2, T, D, params + e.ln2_g, params + e.ln2_b, s->x[l + 1].f, s->x[l + 1].h, keep ? a.st2 : nullptr));
        }
    }

    // bf16 copies of everything after the embeddings (the embeddings are only ever looked up)
    void refresh_weight_copies() const {
        if (!s->bf) return;
        const int64_t first = m->enc_layers[0].wq;
        PROF(ctx, PROF_UPDATE, launch_to_bf16(st, params + first, s->w16 + first, m->num_params - first));
    }
};

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

}  // namespace

size_t seq_workspace_bytes(const bls_model* m, int64_t n, bool train) { return scratch_bytes(m, train ? (int)n : score_chunk(m, n), train); }

int seq_score(bls_ctx* ctx, const bls_model* m, const float* params, const int32_t* x, const int32_t* y, int64_t N, float* losses_out) {
    const int chunk = score_chunk(m, N);
    int rc = bls_arena_reserve(ctx, scratch_bytes(m, chunk, false));
    if (rc != BLS_OK) return rc;
    hipStream_t st = ctx->stream;
    Carver c(ctx->arena);
    SeqScratch s = carve(c, m, chunk, false);
    const int L = m->enc_L, V = m->enc_V, layers = (int)m->enc_layers.size();
    Net net{ctx, st, m, params, &s, chunk};
    net.refresh_weight_copies();
    for (int64_t first = 0; first < N; first += chunk) {
        net.B = (int)(N - first < chunk ? N - first : chunk);
        const int64_t T = (int64_t)net.B * L;
        net.forward(x + first * L, false);
        net.token_losses(s.x[layers], y + first * L, T, false);
        if (!s.bf) PROF(ctx, PROF_HEAD, launch_token_ce(st, s.logits, y + first * L, T, V, s.tok_loss, 0.f, nullptr));
        PROF(ctx, PROF_HEAD, launch_sample_mean(st, s.tok_loss, net.B, L, losses_out + first));
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
    const int64_t T = (int64_t)B * L;
    if (T >= (int64_t(1) << 31) / 2 || T * (int64_t)V >= (int64_t(1) << 40))
        return bls_fail(ctx, BLS_EINVAL, "local_step: batch * sequence length too large");
    int rc = bls_arena_reserve(ctx, scratch_bytes(m, B, true));
    if (rc != BLS_OK) return rc;
    hipStream_t st = ctx->stream;
    Carver c(ctx->arena);
    SeqScratch s = carve(c, m, B, true);
    Net net{ctx, st, m, params, &s, B};
    Net side = net;   // the same products on the side stream
    side.st = ctx->aux;

    FixRangeTable emb_tab{};
    emb_tab.n = 1;
    emb_tab.r[0] = {0, m->enc_tok, (int64_t)V * D};
    PROF(ctx, PROF_UPDATE, launch_fill_zero(st, reinterpret_cast<float*>(s.acc), s.acc_count * 2));
    // Column sums (bias and layer-norm gradients) leave their partial sums in s.cpart; one launch at the end of the
    // backward pass, or when the table or the buffer is full, folds them all into the gradient.
    ColsumTable sums{};
    size_t sums_used = 0;
    auto flush_sums = [&]() {
        if (sums.n > 0) PROF(ctx, PROF_NORM, launch_colsum_table(st, sums, s.cpart, s.grad));
        sums.n = 0;
        sums_used = 0;
    };
    auto reserve_sums = [&](size_t floats) {
        if (sums.n + 3 > COLSUM_TABLE_MAX || sums_used + floats > s.cpart_floats) flush_sums();
        float* part = s.cpart + sums_used;
        sums_used += floats;
        return part;
    };
    auto push_sums = [&](size_t part_off, int rows, int N, int pitch, int64_t out_off) {
        if (sums.n == COLSUM_TABLE_MAX) return false;   // callers reserve first, which leaves room for three jobs
        sums.j[sums.n++] = ColsumJob{(int64_t)part_off, out_off, rows, N, pitch};
        return true;
    };
    auto bias_grad = [&](const float* dy, int N, int64_t out_off) {
        if (T <= 64) {
            PROF(ctx, PROF_NORM, launch_colsum_tokens(st, dy, T, N, nullptr, s.grad + out_off));
            return;
        }
        float* part = reserve_sums(colsum_partial_floats(T, N));
        int rows = 0;
        PROF(ctx, PROF_NORM, rows = launch_colsum_partial(st, dy, T, N, part));
        push_sums(part - s.cpart, rows, N, N, out_off);
    };
    // layer norm backward; the column sums of its result are the gradient of the bias at bias_off
    auto layernorm_bwd = [&](const float* dy, const float* xin, const float* stats, int64_t g_off, float* dx, uint16_t* dx16, int64_t bias_off) {
        float* part = reserve_sums(layernorm_bwd_partial_floats(T, D));
        int rows = 0;
        PROF(ctx, PROF_NORM, rows = launch_layernorm_bwd_partial(st, dy, xin, stats, T, D, params + g_off, dx, dx16, part));
        push_sums(part - s.cpart, rows, 2 * D, 3 * D, g_off);
        push_sums(part - s.cpart + 2 * D, rows, D, 3 * D, bias_off);
    };
    const float gscale = 1.f / (float)T;   // mean over the batch of per-sample means over positions
    const float att = 1.f / sqrtf((float)dh);
    const Mat da{s.da, nullptr};

    for (int64_t j = 0; j < tau; ++j) {
        net.refresh_weight_copies();
        {
            ProfScope prof(ctx, PROF_GATHER);
            hipLaunchKernelGGL(gather_sequences_kernel, dim3(B), dim3(256), 0, st, x_pool, y_pool, sel, k, j * B, L, s.tok, s.tgt);
        }
        net.forward(s.tok, true);
        const Mat hf = s.x[layers];
        net.token_losses(hf, s.tgt, T, true);
        if (s.bf) PROF(ctx, PROF_HEAD, launch_ce_grad(st, s.logits, s.tgt, s.ce_rows, T, V, gscale, s.dlogits.h));
        else PROF(ctx, PROF_HEAD, launch_token_ce(st, s.logits, s.tgt, T, V, s.tok_loss, gscale, nullptr));
        PROF(ctx, PROF_HEAD, launch_sample_mean(st, s.tok_loss, B, L, step_losses_out ? step_losses_out + j * B : s.loss));
        // Weight gradients are off the critical path (only the update needs them): each product runs on the side stream
        // after an event that marks its gradient factor as written.
        size_t n_forks = 0;
        auto aside = [&]() -> int {
            if (n_forks == ctx->fork_events.size()) {
                hipEvent_t ev;
                BLS_HIP(ctx, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
                ctx->fork_events.push_back(ev);
            }
            hipEvent_t ev = ctx->fork_events[n_forks++];
            BLS_HIP(ctx, hipEventRecord(ev, st));
            BLS_HIP(ctx, hipStreamWaitEvent(ctx->aux, ev, 0));
            return BLS_OK;
        };
        int rc2;
        // head
        if ((rc2 = aside()) != BLS_OK) return rc2;
        side.linear_wgrad(s.dlogits, hf, T, V, D, m->enc_head);
        net.linear_dgrad(s.dlogits, T, V, m->enc_head, D, da);
        for (int l = layers - 1; l >= 0; --l) {
            const EncLayer& e = m->enc_layers[l];
            const LayerAct& a = s.act[l];
            const Mat x = s.x[l];
            const Mat db2 = s.db2[l], db1 = s.db1[l], df = s.df[l], dq = s.dq[l], dk = s.dk[l], dv = s.dv[l];
            // h = LN2(r2): da holds dh, db2 receives dr2
            layernorm_bwd(s.da, a.r2, a.st2, e.ln2_g, db2.f, db2.h, e.b2);
            // r2 = h1 + g W2^T + b2
            if ((rc2 = aside()) != BLS_OK) return rc2;
            side.linear_wgrad(db2, a.g, T, D, F, e.w2);
            net.linear_dgrad(db2, T, D, e.w2, F, Mat{df.f, nullptr});
            {
                // du = dg * gelu'(u) with the partial sums of the bias gradient
                float* part = reserve_sums(gelu_bwd_colsum_floats(T, F));
                int rows = 0;
                PROF(ctx, PROF_NORM, rows = launch_gelu_bwd_colsum(st, df.f, a.u, df.h, T, F, part));
                if (rows > 0) {
                    push_sums(part - s.cpart, rows, F, F, e.b1);
                } else {
                    PROF(ctx, PROF_NORM, launch_gelu_bwd(st, df.f, a.u, df.h, T * F));
                    bias_grad(df.f, F, e.b1);
                }
            }
            // u = h1 W1^T + b1
            if ((rc2 = aside()) != BLS_OK) return rc2;
            side.linear_wgrad(df, a.h1, T, F, D, e.w1);
            net.linear_dgrad(df, T, F, e.w1, D, da, db2.f);   // da = dh1 (both uses of h1)
            // h1 = LN1(r1): db1 receives dr1
            layernorm_bwd(s.da, a.r1, a.st1, e.ln1_g, db1.f, db1.h, e.bo);
            // r1 = x + ctx Wo^T + bo
            if ((rc2 = aside()) != BLS_OK) return rc2;
            side.linear_wgrad(db1, a.ctx, T, D, D, e.wo);
            net.linear_dgrad(db1, T, D, e.wo, D, s.dc);          // dc = dctx
            // ctx = P v;  P = softmax(att * q k^T)
            bool fused = false;
            if (s.bf) {
                float* part = reserve_sums((size_t)3 * 4 * B * D);
                ProfScope prof_(ctx, PROF_GEMM);
                fused = launch_attention16_bwd(st, a.q.h, a.k.h, a.v.h, s.dc.h, a.p.f, D, B, H, L, dh, att, dq.f, dk.f, dv.f, dq.h, dk.h, dv.h, part);
                const int64_t offs[3] = {e.bq, e.bk, e.bv};
                for (int i = 0; fused && i < 3; ++i) push_sums(part - s.cpart + (size_t)i * 4 * B * D, 4 * B, D, D, offs[i]);
            }
            if (!fused) {
                net.attention(a.p, true, true, s.dc, false, true, dv, false, dh, L, 1.f);                      // dv = P^T dctx
                net.attention(s.dc, false, false, a.v, false, false, Mat{s.ds.f, nullptr}, true, L, dh, 1.f);  // dP = dctx v^T
                PROF(ctx, PROF_NORM, launch_softmax_bwd_rows(st, s.ds.f, a.p.f, s.ds.h, (int64_t)B * H * L, L, att));
                net.attention(s.ds, true, false, a.k, false, true, dq, false, dh, L, 1.f);                     // dq = dS k
                net.attention(s.ds, true, true, a.q, false, true, dk, false, dh, L, 1.f);                      // dk = dS^T q
            }
            // q, k, v projections of x
            if ((rc2 = aside()) != BLS_OK) return rc2;
            side.qkv_wgrad(dq, dk, dv, x, T, e);
            if (!fused) {
                bias_grad(dq.f, D, e.bq);
                bias_grad(dk.f, D, e.bk);
                bias_grad(dv.f, D, e.bv);
            }
            net.linear_dgrad(dq, T, D, e.wq, D, da, db1.f);    // da = dx, starting from the residual path
            net.linear_dgrad(dk, T, D, e.wk, D, da, s.da);
            net.linear_dgrad(dv, T, D, e.wv, D, da, s.da);
        }
        // embeddings: position gradient = sum over samples, token gradient = scatter by id
        flush_sums();
        PROF(ctx, PROF_NORM, launch_colsum_tokens(st, s.da, B, L * D, s.cpart, s.grad + m->enc_pos));
        PROF(ctx, PROF_NORM, launch_embed_grad(st, s.tok, T, D, s.da, s.acc));
        PROF(ctx, PROF_UPDATE, launch_fix_finalize(st, emb_tab, s.acc, s.grad));
        BLS_HIP(ctx, hipEventRecord(ctx->join_event, ctx->aux));   // every weight gradient is in
        BLS_HIP(ctx, hipStreamWaitEvent(st, ctx->join_event, 0));
        PROF(ctx, PROF_UPDATE, launch_sgd(st, params, momentum, s.grad, m->num_params, opt.lr, opt.momentum, opt.weight_decay));
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
