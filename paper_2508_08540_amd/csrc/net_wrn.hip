// Passes of the pre-activation wide residual network: scoring (inference-mode forward + per-sample loss)
// and the local SGD steps (train-mode forward, backward, update).  All convolutions run on the wide-layer
// kernel; batch norm, head, weight gradient and update kernels are shared with the other networks.
#include "net.h"

#include "kernels.h"

#define PROF(ctx, cls, call) \
    do {                     \
        ProfScope prof_(ctx, cls); \
        call;                \
    } while (0)

namespace {

constexpr int PAD_C = 16;        // the stem's input is zero-padded to 16 channels
constexpr int SCORE_CHUNK = 1024;   // images scored together
typedef uint8_t act_t;

int padded(int c) { return c < PAD_C ? PAD_C : c; }

struct ConvRef {
    const ConvSlot* slot;
    int64_t fwd_off, dgrad_off;  // byte offsets of the packed copies (dgrad_off < 0: none)
    int64_t acc_off;             // accumulators of this layer
};

struct BnRef {
    const BnSlot* slot;
    float *mean, *invstd;
    fixsum_t *fsums, *bsums;     // forward (sum, sum of squares) and backward (sum g, sum g*xhat) accumulators
};

struct WrnScratch {
    int act;
    size_t esz;
    act_t* wpack;
    PackTable tab;
    UpdateTable utab;
    std::vector<ConvRef> convs;  // 0: stem; then per block conv1, conv2, [shortcut]
    std::vector<BnRef> bns;      // per block bn1, bn2; last: final
    act_t *xpad, *y0, *a_final;
    std::vector<act_t*> o1, y1, o2, sc, out;  // per block
    act_t *g1, *g2, *g3, *g4;    // backward temporaries; in inference g1..g4 rotate as activations
    // gradients that the weight-gradient kernels of the side stream read: they keep a buffer of their own for the whole
    // backward pass.  dblk[i] = gradient of the input of block i (dblk[blocks] = of the last block's output),
    // dy1[i] = gradient of the first convolution's output in block i
    std::vector<act_t*> dblk, dy1;
    fixsum_t *sums, *wacc;
    int64_t n_sums, wacc_count;
    float *grad, *loss, *feat, *dlogits, *dfeat;
    int32_t* yb;
    // bf16: weight gradients of the 1x1 shortcuts as one GEMM dW = dy^T x over the pixels
    uint16_t* xs16;     // the shortcut's input sampled at its stride, [pixels_out][c_in]
    float* gpart;       // partial sums of the split contraction
};

// The 1x1 shortcut's weight gradient is a plain matrix product over the output pixels; in bf16 it runs on the bf16 GEMM
// (split over the pixels, partial sums added in order) instead of the convolution weight-gradient kernel.
// The same holds tap by tap for a 3x3 layer (one product per tap over inputs gathered at that tap's offset, zero outside
// the map); the layers the bf16 weight-gradient kernel does not cover (stride 2, fewer than 64 input channels) go this way.
bool shortcut_wgrad_by_gemm(int act, const ConvSlot& c, int B = 2) {
    if (act != ACT_BF16 || c.c_in < 16 || c.c_in % 8 != 0 || c.c_out % 8 != 0) return false;
    if (c.taps == 1) return true;
    ConvShape cs;
    cs.B = B; cs.h_in = c.h_in; cs.c_in = c.c_in; cs.c_out = c.c_out; cs.stride = c.stride; cs.c_in_real = c.c_in; cs.taps = c.taps;
    return !wgrad16_covers(act, cs);
}
int shortcut_splits(const ConvSlot& c, int B) {
    const int64_t tiles = ceil_div(c.c_out, 128) * ceil_div(c.c_in, 128) * c.taps, K = (int64_t)B * c.h_out * c.h_out;
    int64_t sp = ceil_div(512, tiles);
    const int64_t most = K / 256 > 1 ? K / 256 : 1;
    sp = sp > most ? most : sp;
    return (int)(sp > 64 ? 64 : sp);
}

ConvShape shape_of(const ConvSlot& c, int B) {
    ConvShape cs;
    cs.B = B; cs.h_in = c.h_in; cs.c_in = padded(c.c_in); cs.c_out = c.c_out; cs.stride = c.stride; cs.c_in_real = c.c_in;
    cs.taps = c.taps;
    return cs;
}

WrnScratch carve(Carver& c, const bls_model* m, int B, bool train) {
    WrnScratch s{};
    s.act = m->desc.act_dtype == BLS_ACT_BF16 ? ACT_BF16 : ACT_F32;
    s.esz = act_bytes(s.act);
    const size_t esz = s.esz;
    const int hw = m->desc.image_hw;
    // convolutions in parameter order
    std::vector<const ConvSlot*> slots{&m->wrn_stem};
    for (const WrnBlock& b : m->wrn_blocks) {
        slots.push_back(&b.conv1);
        slots.push_back(&b.conv2);
        if (b.proj) slots.push_back(&b.shortcut);
    }
    s.tab.n = 0;
    s.utab.n = 0;
    int64_t quads = 0, acc = 0;
    s.convs.resize(slots.size());
    for (int pass = 0; pass < (train ? 2 : 1); ++pass)
        for (size_t i = (pass == 0 ? 0 : 1); i < slots.size(); ++i) {
            const ConvSlot& cv = *slots[i];
            PackEntry& e = s.tab.e[s.tab.n++];
            e.w_off = cv.w_off; e.pack_off = quads;
            e.c_in = padded(cv.c_in); e.c_out = cv.c_out; e.c_in_real = cv.c_in; e.dgrad = pass; e.taps = cv.taps; e.pad_ = 0;
            if (pass == 0) {
                s.convs[i].slot = &cv;
                s.convs[i].fwd_off = quads * 4 * (int64_t)esz;
                s.convs[i].dgrad_off = -1;
            } else {
                s.convs[i].dgrad_off = quads * 4 * (int64_t)esz;
            }
            quads += (int64_t)e.c_in * e.c_out * cv.taps / 4;
        }
    s.tab.total_vec4 = quads;
    s.wpack = c.take<act_t>(quads * 4 * esz);
    for (size_t i = 0; i < slots.size(); ++i) {
        const ConvSlot& cv = *slots[i];
        ConvShape cs = shape_of(cv, B);
        s.convs[i].acc_off = acc;
        UpdateEntry& ue = s.utab.e[s.utab.n++];
        ue.w_off = cv.w_off; ue.n = (int64_t)cv.c_out * cv.taps * cv.c_in; ue.acc_off = acc;
        ue.fwd_quad = s.convs[i].fwd_off / (4 * (int64_t)esz);
        ue.dgrad_quad = s.convs[i].dgrad_off >= 0 ? s.convs[i].dgrad_off / (4 * (int64_t)esz) : -1;
        ue.c_in = cs.c_in; ue.c_out = cs.c_out; ue.c_in_real = cs.c_in_real; ue.taps = cv.taps;
        if (shortcut_wgrad_by_gemm(s.act, cv)) {
            ue.replicas = 0; ue.pad_ = 0;   // gradient arrives as floats in grad[]
        } else {
            ue.replicas = conv_wgrad_replicas(s.act, cs); ue.pad_ = 0;
            acc += conv_wgrad_accumulators(s.act, cs);
        }
    }
    // batch norms
    std::vector<const BnSlot*> bslots;
    for (const WrnBlock& b : m->wrn_blocks) {
        bslots.push_back(&b.bn1);
        bslots.push_back(&b.bn2);
    }
    bslots.push_back(&m->wrn_final_bn);
    s.bns.resize(bslots.size());
    int64_t n_sums = 0;
    for (size_t i = 0; i < bslots.size(); ++i) n_sums += 2 * (int64_t)FIX_REPLICAS * 2 * bslots[i]->c;
    s.n_sums = n_sums;
    s.sums = train ? c.take<fixsum_t>(n_sums) : nullptr;
    int64_t so = 0;
    for (size_t i = 0; i < bslots.size(); ++i) {
        BnRef& r = s.bns[i];
        r.slot = bslots[i];
        r.mean = c.take<float>(r.slot->c);
        r.invstd = c.take<float>(r.slot->c);
        const int64_t set = (int64_t)FIX_REPLICAS * 2 * r.slot->c;
        r.fsums = train ? s.sums + so : nullptr;
        r.bsums = train ? s.sums + so + set : nullptr;
        so += 2 * set;
    }
    // activations
    s.xpad = c.take<act_t>((size_t)B * hw * hw * PAD_C * esz);
    s.yb = c.take<int32_t>(B);
    s.loss = c.take<float>(B);
    int64_t max_act = (int64_t)B * hw * hw * padded(m->wrn_stem.c_out);
    for (const WrnBlock& b : m->wrn_blocks) {
        max_act = std::max<int64_t>(max_act, (int64_t)B * b.conv1.h_in * b.conv1.h_in * b.conv1.c_in);
        max_act = std::max<int64_t>(max_act, (int64_t)B * b.conv1.h_out * b.conv1.h_out * b.conv1.c_out);
    }
    const size_t nb = m->wrn_blocks.size();
    s.o1.assign(nb, nullptr); s.y1.assign(nb, nullptr); s.o2.assign(nb, nullptr); s.sc.assign(nb, nullptr); s.out.assign(nb, nullptr);
    s.dblk.assign(nb + 1, nullptr); s.dy1.assign(nb, nullptr);
    s.g1 = c.take<act_t>(max_act * esz);
    s.g2 = c.take<act_t>(max_act * esz);
    s.g3 = c.take<act_t>(max_act * esz);
    s.g4 = c.take<act_t>(max_act * esz);
    if (train) {
        s.y0 = c.take<act_t>((size_t)B * hw * hw * m->wrn_stem.c_out * esz);
        for (size_t i = 0; i < nb; ++i) {
            const WrnBlock& b = m->wrn_blocks[i];
            const size_t in_elems = (size_t)B * b.conv1.h_in * b.conv1.h_in * b.conv1.c_in;
            const size_t out_elems = (size_t)B * b.conv1.h_out * b.conv1.h_out * b.conv1.c_out;
            s.o1[i] = c.take<act_t>(in_elems * esz);
            s.y1[i] = c.take<act_t>(out_elems * esz);
            s.dblk[i] = c.take<act_t>(in_elems * esz);
            s.dy1[i] = c.take<act_t>(out_elems * esz);
            if (i + 1 == nb) s.dblk[nb] = c.take<act_t>(out_elems * esz);
            s.o2[i] = c.take<act_t>(out_elems * esz);
            if (b.proj) s.sc[i] = c.take<act_t>(out_elems * esz);
            s.out[i] = c.take<act_t>(out_elems * esz);
        }
        s.a_final = c.take<act_t>((size_t)B * m->final_hw * m->final_hw * m->final_c * esz);
        s.wacc = c.take<fixsum_t>(acc);
        s.wacc_count = acc;
        s.grad = c.take<float>(m->num_params);
        s.feat = c.take<float>((size_t)B * m->final_c);
        s.dlogits = c.take<float>((size_t)B * m->desc.classes);
        s.dfeat = c.take<float>((size_t)B * m->final_c);
        size_t xs = 0, gp = 0;
        for (const WrnBlock& b : m->wrn_blocks)
            if (b.proj && shortcut_wgrad_by_gemm(s.act, b.shortcut)) {
                const ConvSlot& cv = b.shortcut;
                const size_t sampled = cv.stride != 1 ? (size_t)B * cv.h_out * cv.h_out * cv.c_in : 0;
                const size_t part = (size_t)cv.c_out * cv.c_in * shortcut_splits(cv, B);
                xs = sampled > xs ? sampled : xs;
                gp = part > gp ? part : gp;
            }
        for (const WrnBlock& b : m->wrn_blocks)
            for (const ConvSlot* cv : {&b.conv1, &b.conv2})
                if (shortcut_wgrad_by_gemm(s.act, *cv)) {
                    const size_t gathered = (size_t)9 * B * cv->h_out * cv->h_out * cv->c_in;
                    const size_t part = (size_t)9 * cv->c_out * cv->c_in * shortcut_splits(*cv, B);
                    xs = gathered > xs ? gathered : xs;
                    gp = part > gp ? part : gp;
                }
        s.xs16 = c.take<uint16_t>(xs ? xs : 1);
        s.gpart = c.take<float>(gp ? gp : 1);
    }
    return s;
}

size_t scratch_bytes(const bls_model* m, int B, bool train) {
    Carver c(nullptr);
    carve(c, m, B, train);
    return c.off;
}

// y = conv(x) [+ add], optional statistics of y into `stats` (forward accumulators of the batch norm that reads y)
int conv_fwd(bls_ctx* ctx, hipStream_t st, const WrnScratch& s, const ConvRef& cr, int B, const act_t* x, act_t* y, const act_t* add,
             fixsum_t* stats, const WconvBn* bn = nullptr) {
    const ConvSlot& c = *cr.slot;
    ProfScope prof_(ctx, PROF_CONV_FWD);
    if (launch_wconv(st, s.act, c.taps, B, c.h_in, c.h_out, padded(c.c_in), c.c_out, c.stride, 0, x, s.wpack + cr.fwd_off, y, add, stats,
                     FIX_FWD_SCALE, bn) != 0)
        return bls_fail(ctx, BLS_EUNSUPPORTED, "convolution %dx%d, %d -> %d channels, map %d is outside what the kernels cover",
                        c.taps == 9 ? 3 : 1, c.taps == 9 ? 3 : 1, c.c_in, c.c_out, c.h_in);
    return BLS_OK;
}

// dx = conv_transpose(dy) [+ add]: a stride-1 convolution of dy (read with zeros inserted for a stride-2 layer)
// with the transposed, flipped weights; channel roles swap
int conv_dgrad(bls_ctx* ctx, hipStream_t st, const WrnScratch& s, const ConvRef& cr, int B, const act_t* dy, act_t* dx, const act_t* add) {
    const ConvSlot& c = *cr.slot;
    ProfScope prof_(ctx, PROF_CONV_DGRAD);
    if (launch_wconv(st, s.act, c.taps, B, c.h_in, c.h_in, c.c_out, c.c_in, 1, c.stride == 2 ? 1 : 0, dy, s.wpack + cr.dgrad_off, dx, add,
                     nullptr, 0.0) != 0)
        return bls_fail(ctx, BLS_EUNSUPPORTED, "input gradient of a %d -> %d convolution on map %d is outside what the kernels cover",
                        c.c_in, c.c_out, c.h_in);
    return BLS_OK;
}

// xs[b][oy][ox][:] = x[b][stride * oy][stride * ox][:], 16 bytes per thread
__global__ __launch_bounds__(256) void sample_pixels_kernel(const uint16_t* __restrict__ x, int h_in, int h_out, int stride, int c8, int64_t n16,
                                                            uint16_t* __restrict__ xs) {
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += step) {
        const int64_t pix = i / c8;
        const int c = (int)(i - pix * c8);
        const int ox = (int)(pix % h_out);
        const int64_t t = pix / h_out;
        const int oy = (int)(t % h_out);
        const int64_t b = t / h_out;
        const int64_t src = ((b * h_in + (int64_t)stride * oy) * h_in + (int64_t)stride * ox) * c8 + c;
        reinterpret_cast<uint4*>(xs)[i] = reinterpret_cast<const uint4*>(x)[src];
    }
}

// xs[t][b][oy][ox][:] = x[b][stride * oy + ky - 1][stride * ox + kx - 1][:] for tap t = 3 ky + kx, zero outside the map
__global__ __launch_bounds__(256) void gather_taps_kernel(const uint16_t* __restrict__ x, int h_in, int h_out, int stride, int c8, int64_t n16,
                                                          uint16_t* __restrict__ xs) {
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < 9 * n16; i += step) {
        const int t = (int)(i / n16);
        const int64_t j = i - (int64_t)t * n16, pix = j / c8;
        const int c = (int)(j - pix * c8);
        const int ox = (int)(pix % h_out);
        const int64_t q = pix / h_out;
        const int oy = (int)(q % h_out);
        const int64_t b = q / h_out;
        const int iy = stride * oy + t / 3 - 1, ix = stride * ox + t % 3 - 1;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (iy >= 0 && iy < h_in && ix >= 0 && ix < h_in) v = reinterpret_cast<const uint4*>(x)[((b * h_in + iy) * h_in + ix) * c8 + c];
        reinterpret_cast<uint4*>(xs)[i] = v;
    }
}

void conv_wgrad(bls_ctx* ctx, hipStream_t st, const WrnScratch& s, const ConvRef& cr, int B, const act_t* x, const act_t* dy) {
    ProfScope prof_(ctx, PROF_CONV_WGRAD, st);
    const ConvSlot& c = *cr.slot;
    if (c.taps == 9 && shortcut_wgrad_by_gemm(s.act, c)) {
        const int64_t pixels = (int64_t)B * c.h_out * c.h_out, n16 = pixels * (c.c_in / 8);
        int64_t blocks = (9 * n16 + 255) / 256;
        hipLaunchKernelGGL(gather_taps_kernel, dim3((unsigned)(blocks > 8192 ? 8192 : blocks)), dim3(256), 0, st, reinterpret_cast<const uint16_t*>(x),
                           c.h_in, c.h_out, c.stride, c.c_in / 8, n16, s.xs16);
        Gemm16Desc d{};
        d.A = reinterpret_cast<const uint16_t*>(dy); d.lda = c.c_out; d.a_kmajor = 1;            // the same dy for every tap
        d.B = s.xs16; d.ldb = c.c_in; d.b_kmajor = 1; d.sb1 = pixels * c.c_in;
        d.C = s.grad + c.w_off; d.ldc = 9 * c.c_in; d.sc1 = c.c_in;                              // w[c_out][tap][c_in]
        d.M = c.c_out; d.N = c.c_in; d.K = (int)pixels;
        d.batch = 9; d.inner = 1;
        d.alpha = 1.f;
        d.splits = shortcut_splits(c, B);
        d.part = s.gpart;
        launch_gemm16(st, d);
        return;
    }
    if (c.taps == 1 && shortcut_wgrad_by_gemm(s.act, c)) {
        const int64_t pixels = (int64_t)B * c.h_out * c.h_out;
        const uint16_t* xs = reinterpret_cast<const uint16_t*>(x);
        if (c.stride != 1) {
            const int64_t n16 = pixels * (c.c_in / 8);
            int64_t blocks = (n16 + 255) / 256;
            hipLaunchKernelGGL(sample_pixels_kernel, dim3((unsigned)(blocks > 4096 ? 4096 : blocks)), dim3(256), 0, st, xs, c.h_in, c.h_out, c.stride,
                               c.c_in / 8, n16, s.xs16);
            xs = s.xs16;
        }
        Gemm16Desc d{};
        d.A = reinterpret_cast<const uint16_t*>(dy); d.lda = c.c_out; d.a_kmajor = 1;
        d.B = xs; d.ldb = c.c_in; d.b_kmajor = 1;
        d.C = s.grad + c.w_off; d.ldc = c.c_in;
        d.M = c.c_out; d.N = c.c_in; d.K = (int)pixels;
        d.alpha = 1.f;
        d.splits = shortcut_splits(c, B);
        d.part = s.gpart;
        launch_gemm16(st, d);
        return;
    }
    launch_conv_wgrad(st, s.act, shape_of(c, B), x, dy, s.wacc + cr.acc_off);
}

void bn_forward(bls_ctx* ctx, hipStream_t st, const WrnScratch& s, const BnRef& bn, const float* params, float* buffers, int64_t pixels,
                const act_t* y, act_t* out) {
    BnStats bs{};
    bs.sums = bn.fsums;
    bs.count = (double)pixels;
    bs.mean = bn.mean; bs.invstd = bn.invstd;
    bs.running_mean = buffers + bn.slot->rmean_off; bs.running_var = buffers + bn.slot->rvar_off;
    PROF(ctx, PROF_NORM, launch_bn_apply(st, s.act, y, pixels, bn.slot->c, bs, params + bn.slot->gamma_off, params + bn.slot->beta_off, nullptr,
                                         bn.slot->c, 1, 1, out));
}

// Backward of out = relu(bn(y)): dy = d/dy of <dout, out> [+ add]; the scale and shift gradients go to grad
void bn_backward(bls_ctx* ctx, hipStream_t st, const WrnScratch& s, const BnRef& bn, const float* params, int64_t pixels, const void* dout,
                 int shared, const act_t* out, const act_t* y, act_t* dy, const act_t* add) {
    ProfScope prof_(ctx, PROF_NORM);
    launch_bn_bwd_reduce(st, s.act, dout, shared, out, y, pixels, bn.slot->c, bn.mean, bn.invstd, bn.bsums);
    launch_bn_bwd_apply(st, s.act, dout, shared, out, y, pixels, bn.slot->c, bn.mean, bn.invstd, params + bn.slot->gamma_off, bn.bsums,
                        s.grad + bn.slot->gamma_off, s.grad + bn.slot->beta_off, dy, nullptr, add);
}

// Inference forward over a batch gathered into s.xpad.  Every batch norm uses running statistics, which are known before
// the convolution that produces its input runs: that convolution applies it (and the ReLU) in its epilogue and stores the
// activation the next layer reads; the raw sum of a block goes to memory as well only where the next block adds it back
// through an identity shortcut.  No batch-norm launches; four buffers rotate.
int forward_inference(bls_ctx* ctx, hipStream_t st, const bls_model* m, const float* params, const float* buffers, int B, WrnScratch& s,
                      bool prepare, const act_t** final_act) {
    if (prepare) {
        PROF(ctx, PROF_UPDATE, launch_pack_weights(st, s.act, params, s.wpack, s.tab));
        for (const BnRef& bn : s.bns)
            PROF(ctx, PROF_NORM, launch_bn_inference_stats(st, buffers + bn.slot->rmean_off, buffers + bn.slot->rvar_off, bn.slot->c, bn.mean, bn.invstd));
    }
    act_t* rot[4] = {s.g1, s.g2, s.g3, s.g4};
    int next = 0;
    auto take = [&](const act_t* k0, const act_t* k1, const act_t* k2) {
        for (;;) {
            act_t* p = rot[next];
            next = (next + 1) & 3;
            if (p != k0 && p != k1 && p != k2) return p;
        }
    };
    auto fused = [&](const BnRef& bn, act_t* raw) {
        return WconvBn{bn.mean, bn.invstd, params + bn.slot->gamma_off, params + bn.slot->beta_off, raw};
    };
    const size_t nb = m->wrn_blocks.size();
    int rc;
    size_t ci = 0, bi = 0;
    // the stem's output: normalised by the first block's first batch norm, raw as well when that block's shortcut is the identity
    act_t* cur = take(nullptr, nullptr, nullptr);                                   // relu(bn1(block input))
    act_t* cur_raw = (nb && !m->wrn_blocks[0].proj) ? take(cur, nullptr, nullptr) : nullptr;   // block input
    {
        const WconvBn f = fused(s.bns[0], cur_raw);
        rc = conv_fwd(ctx, st, s, s.convs[ci++], B, s.xpad, cur, nullptr, nullptr, &f);
        if (rc != BLS_OK) return rc;
    }
    for (size_t i = 0; i < nb; ++i) {
        const WrnBlock& b = m->wrn_blocks[i];
        ++bi;                                    // bn1 was applied by the producer of `cur`
        const BnRef& bn2 = s.bns[bi++];
        const BnRef& bn_next = s.bns[bi];        // the batch norm that reads this block's output
        act_t* o2 = take(cur, cur_raw, nullptr);
        {
            const WconvBn f = fused(bn2, nullptr);
            rc = conv_fwd(ctx, st, s, s.convs[ci++], B, cur, o2, nullptr, nullptr, &f);
            if (rc != BLS_OK) return rc;
        }
        const ConvRef& c2 = s.convs[ci++];
        const act_t* shortcut = cur_raw;
        if (b.proj) {
            act_t* sc = take(cur, o2, nullptr);
            rc = conv_fwd(ctx, st, s, s.convs[ci++], B, cur, sc, nullptr, nullptr);
            if (rc != BLS_OK) return rc;
            shortcut = sc;
        }
        const bool raw_needed = i + 1 < nb && !m->wrn_blocks[i + 1].proj;
        act_t* out = take(o2, shortcut, nullptr);
        act_t* out_raw = raw_needed ? take(o2, shortcut, out) : nullptr;
        {
            const WconvBn f = fused(bn_next, out_raw);
            rc = conv_fwd(ctx, st, s, c2, B, o2, out, shortcut, nullptr, &f);
            if (rc != BLS_OK) return rc;
        }
        cur = out;
        cur_raw = out_raw;
    }
    *final_act = cur;
    return BLS_OK;
}

// Training forward over a batch gathered into s.xpad: batch statistics, and everything the backward pass needs is kept.
int forward(bls_ctx* ctx, hipStream_t st, const bls_model* m, const float* params, float* buffers, int B, WrnScratch& s, bool prepare,
            const act_t** final_act) {
    if (prepare) {
        PROF(ctx, PROF_UPDATE, launch_pack_weights(st, s.act, params, s.wpack, s.tab));
        PROF(ctx, PROF_UPDATE, launch_fill_zero(st, reinterpret_cast<float*>(s.sums), s.n_sums * 2));
    }
    int rc;
    act_t* cur = s.y0;
    size_t ci = 0, bi = 0;
    rc = conv_fwd(ctx, st, s, s.convs[ci++], B, s.xpad, cur, nullptr, s.bns[0].fsums);
    if (rc != BLS_OK) return rc;
    for (size_t i = 0; i < m->wrn_blocks.size(); ++i) {
        const WrnBlock& b = m->wrn_blocks[i];
        const int64_t px_in = (int64_t)B * b.conv1.h_in * b.conv1.h_in, px_out = (int64_t)B * b.conv1.h_out * b.conv1.h_out;
        const BnRef& bn1 = s.bns[bi++];
        const BnRef& bn2 = s.bns[bi++];
        const BnRef& bn_next = s.bns[bi];  // the batch norm that reads this block's output
        bn_forward(ctx, st, s, bn1, params, buffers, px_in, cur, s.o1[i]);
        rc = conv_fwd(ctx, st, s, s.convs[ci++], B, s.o1[i], s.y1[i], nullptr, bn2.fsums);
        if (rc != BLS_OK) return rc;
        const ConvRef& c2 = s.convs[ci++];
        const act_t* shortcut = cur;
        if (b.proj) {
            rc = conv_fwd(ctx, st, s, s.convs[ci++], B, s.o1[i], s.sc[i], nullptr, nullptr);
            if (rc != BLS_OK) return rc;
            shortcut = s.sc[i];
        }
        bn_forward(ctx, st, s, bn2, params, buffers, px_out, s.y1[i], s.o2[i]);
        rc = conv_fwd(ctx, st, s, c2, B, s.o2[i], s.out[i], shortcut, bn_next.fsums);
        if (rc != BLS_OK) return rc;
        cur = s.out[i];
    }
    const int64_t px = (int64_t)B * m->final_hw * m->final_hw;
    bn_forward(ctx, st, s, s.bns[bi], params, buffers, px, cur, s.a_final);
    *final_act = s.a_final;
    return BLS_OK;
}

int backward(bls_ctx* ctx, hipStream_t st, const bls_model* m, const float* params, int B, WrnScratch& s) {
    const size_t nb = m->wrn_blocks.size();
    // convolution references per block
    std::vector<size_t> first(nb);
    size_t ci = 1;
    for (size_t i = 0; i < nb; ++i) {
        first[i] = ci;
        ci += m->wrn_blocks[i].proj ? 3 : 2;
    }
    const int64_t px_f = (int64_t)B * m->final_hw * m->final_hw;
    // The weight gradients are off the critical path (only the update needs them): each runs on the context's side
    // stream after an event that marks its dy as written; nothing they read is overwritten before the streams join at
    // the end of the pass (activations are per block, the gradients they read have buffers of their own).
    size_t n_forks = 0;
    auto wgrad_aside = [&](const ConvRef& cr, const act_t* x, const act_t* dy) -> int {
        if (n_forks == ctx->fork_events.size()) {
            hipEvent_t e;
            BLS_HIP(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
            ctx->fork_events.push_back(e);
        }
        hipEvent_t ev = ctx->fork_events[n_forks++];
        BLS_HIP(ctx, hipEventRecord(ev, st));
        BLS_HIP(ctx, hipStreamWaitEvent(ctx->aux, ev, 0));
        conv_wgrad(ctx, ctx->aux, s, cr, B, x, dy);
        return BLS_OK;
    };
    act_t* dnext = s.g2;   // main stream only
    act_t* g3 = s.g3;      // main stream only
    act_t* dcur = s.dblk[nb];
    bn_backward(ctx, st, s, s.bns[2 * nb], params, px_f, s.dfeat, m->final_hw * m->final_hw, s.a_final, s.out[nb - 1], dcur, nullptr);
    int rc;
    for (size_t ii = nb; ii-- > 0;) {
        const WrnBlock& b = m->wrn_blocks[ii];
        const int64_t px_in = (int64_t)B * b.conv1.h_in * b.conv1.h_in, px_out = (int64_t)B * b.conv1.h_out * b.conv1.h_out;
        const ConvRef& c1 = s.convs[first[ii]];
        const ConvRef& c2 = s.convs[first[ii] + 1];
        const act_t* block_in = ii == 0 ? s.y0 : s.out[ii - 1];
        act_t* dy1 = s.dy1[ii];
        if ((rc = wgrad_aside(c2, s.o2[ii], dcur)) != BLS_OK) return rc;
        rc = conv_dgrad(ctx, st, s, c2, B, dcur, g3, nullptr);                                   // g3 = d o2
        if (rc != BLS_OK) return rc;
        bn_backward(ctx, st, s, s.bns[2 * ii + 1], params, px_out, g3, 0, s.o2[ii], s.y1[ii], dy1, nullptr);
        if ((rc = wgrad_aside(c1, s.o1[ii], dy1)) != BLS_OK) return rc;
        const act_t* branch = nullptr;
        if (b.proj) {
            const ConvRef& cs = s.convs[first[ii] + 2];
            if ((rc = wgrad_aside(cs, s.o1[ii], dcur)) != BLS_OK) return rc;
            rc = conv_dgrad(ctx, st, s, cs, B, dcur, g3, nullptr);                               // g3 = gradient through the projection
            if (rc != BLS_OK) return rc;
            branch = g3;
        }
        rc = conv_dgrad(ctx, st, s, c1, B, dy1, dnext, branch);                                  // dnext = d o1
        if (rc != BLS_OK) return rc;
        // d block_in = bn1 backward of d o1, plus the gradient through an identity shortcut
        bn_backward(ctx, st, s, s.bns[2 * ii], params, px_in, dnext, 0, s.o1[ii], block_in, s.dblk[ii], b.proj ? nullptr : dcur);
        dcur = s.dblk[ii];
    }
    if ((rc = wgrad_aside(s.convs[0], s.xpad, dcur)) != BLS_OK) return rc;
    BLS_HIP(ctx, hipEventRecord(ctx->join_event, ctx->aux));
    BLS_HIP(ctx, hipStreamWaitEvent(st, ctx->join_event, 0));
    return BLS_OK;
}

}  // namespace

size_t wrn_workspace_bytes(const bls_model* m, int64_t n, bool train) {
    return scratch_bytes(m, (int)(train || n < SCORE_CHUNK ? n : SCORE_CHUNK), train);
}

int wrn_score(bls_ctx* ctx, const bls_model* m, const float* params, const float* buffers, const float* x, const int32_t* y, int64_t N,
              float* losses_out) {
    const int chunk = (int)(N < SCORE_CHUNK ? N : SCORE_CHUNK);
    int rc = bls_arena_reserve(ctx, scratch_bytes(m, chunk, false));
    if (rc != BLS_OK) return rc;
    hipStream_t st = ctx->stream;
    Carver c(ctx->arena);
    WrnScratch s = carve(c, m, chunk, false);
    const int hw = m->desc.image_hw;
    for (int64_t first = 0; first < N; first += chunk) {
        int B = (int)(N - first < chunk ? N - first : chunk);
        PROF(ctx, PROF_GATHER, launch_gather_images(st, x, y, nullptr, 1, 0, first, B, hw * hw, m->desc.in_channels, PAD_C, s.act, s.xpad, s.yb));
        const act_t* fin = nullptr;
        rc = forward_inference(ctx, st, m, params, buffers, B, s, first == 0, &fin);
        if (rc != BLS_OK) return rc;
        PROF(ctx, PROF_HEAD, launch_head_forward(st, s.act, fin, B, m->final_hw * m->final_hw, m->final_c, params + m->fc_w, params + m->fc_b,
                                                 m->desc.classes, s.yb, losses_out + first, nullptr, nullptr, nullptr, 0.f, false));
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}

int wrn_local_step(bls_ctx* ctx, const bls_model* m, float* params, float* buffers, float* momentum, const float* x_pool,
                   const int32_t* y_pool, int64_t N, const int32_t* sel, int64_t k, int64_t batch, int64_t tau, const bls_sgd& opt,
                   float* step_losses_out) {
    (void)N;
    const int B = (int)batch;
    int rc = bls_arena_reserve(ctx, scratch_bytes(m, B, true));
    if (rc != BLS_OK) return rc;
    hipStream_t st = ctx->stream;
    Carver c(ctx->arena);
    WrnScratch s = carve(c, m, B, true);
    const int hw = m->desc.image_hw, C = m->desc.classes;
    const float inv_b = 1.f / (float)B;
    PROF(ctx, PROF_UPDATE, launch_fill_zero(st, reinterpret_cast<float*>(s.wacc), s.wacc_count * 2));
    for (int64_t j = 0; j < tau; ++j) {
        float* loss = step_losses_out ? step_losses_out + j * B : s.loss;
        PROF(ctx, PROF_GATHER, launch_gather_images(st, x_pool, y_pool, sel, k, j * B, 0, B, hw * hw, m->desc.in_channels, PAD_C, s.act, s.xpad, s.yb));
        const act_t* fin = nullptr;
        rc = forward(ctx, st, m, params, buffers, B, s, j == 0, &fin);
        if (rc != BLS_OK) return rc;
        PROF(ctx, PROF_HEAD, launch_head_forward(st, s.act, fin, B, m->final_hw * m->final_hw, m->final_c, params + m->fc_w, params + m->fc_b, C,
                                                 s.yb, loss, s.feat, s.dlogits, s.dfeat, inv_b, false));
        // the head's weight gradient is only needed by the update: side stream, joined at the end of the backward pass
        BLS_HIP(ctx, hipEventRecord(ctx->head_event, st));
        BLS_HIP(ctx, hipStreamWaitEvent(ctx->aux, ctx->head_event, 0));
        {
            ProfScope prof_(ctx, PROF_HEAD, ctx->aux);
            launch_head_wgrad(ctx->aux, s.dlogits, s.feat, B, C, m->final_c, s.grad + m->fc_w, s.grad + m->fc_b);
        }
        rc = backward(ctx, st, m, params, B, s);
        if (rc != BLS_OK) return rc;
        PROF(ctx, PROF_UPDATE, launch_update(st, s.act, params, momentum, s.grad, m->num_params, opt.lr, opt.momentum, opt.weight_decay, s.wacc,
                                             s.wpack, s.utab, s.sums, s.n_sums));
    }
    BLS_HIP(ctx, hipGetLastError());
    return BLS_OK;
}
