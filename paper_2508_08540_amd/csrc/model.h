// Architecture description and flat-vector layout (host side).
#pragma once
#include "common.h"

struct TensorSlot {
    std::string name;
    int64_t offset;
    int ndim;
    int shape[4];
    bool is_buffer;
    int64_t count() const {
        int64_t n = 1;
        for (int i = 0; i < ndim; ++i) n *= shape[i];
        return n;
    }
};

// One batch-normalised 3x3 convolution of the residual network.
struct ConvBn {
    int c_in, c_out, stride;
    int h_in, h_out;          // square feature maps
    int64_t w_off;            // conv weight [c_out,3,3,c_in] in params
    int64_t gamma_off, beta_off;
    int64_t rmean_off, rvar_off;  // in buffers
};

// Pieces of the pre-activation wide residual network.
struct BnSlot {
    int c;
    int64_t gamma_off, beta_off;   // in params
    int64_t rmean_off, rvar_off;   // in buffers
};
struct ConvSlot {
    int c_in, c_out, stride, taps;  // taps 9: 3x3 with padding 1; 1: 1x1
    int h_in, h_out;
    int64_t w_off;                  // weight [c_out, k, k, c_in] in params
};
struct WrnBlock {
    BnSlot bn1, bn2;
    ConvSlot conv1, conv2, shortcut;  // shortcut is used only when proj
    bool proj;
};

// One layer of the transformer encoder: offsets into params.
struct EncLayer {
    int64_t wq, bq, wk, bk, wv, bv, wo, bo, ln1_g, ln1_b, w1, b1, w2, b2, ln2_g, ln2_b;
};

struct bls_model {
    bls_model_desc desc;
    int64_t num_params = 0;
    int64_t num_buffers = 0;
    std::vector<TensorSlot> tensors;
    // MLP
    int64_t fc1_w = 0, fc1_b = 0, fc2_w = 0, fc2_b = 0;
    int d_in = 0;
    // residual network: layers[0] is the stem, then conv1/conv2 of every block in order
    std::vector<ConvBn> layers;
    int64_t fc_w = 0, fc_b = 0;
    int final_c = 0, final_hw = 0;
    // wide residual network: stem convolution, blocks, batch norm before the classifier
    ConvSlot wrn_stem{};
    std::vector<WrnBlock> wrn_blocks;
    BnSlot wrn_final_bn{};
    // transformer encoder: vocabulary V, sequence length L, width D, heads H, feed-forward width F
    int enc_V = 0, enc_L = 0, enc_D = 0, enc_H = 0, enc_F = 0;
    int64_t enc_tok = 0, enc_pos = 0, enc_head = 0;
    std::vector<EncLayer> enc_layers;
};
