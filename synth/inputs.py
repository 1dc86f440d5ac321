"""Synthetic workloads shaped like the paper's (CIFAR-like 3x32x32 images, 10 classes).

Images are NHWC float32: x_i = mu_{y_i} + N(0, I) with class means mu_c = 0.5 * N(0, I)
and labels uniform over the classes.  They stand in for CIFAR-10, which the paper
trains ResNet20 on (Section 5, experimental settings).  Network weights are seed-drawn: He-normal convolutions
(std = sqrt(2 / fan_out)), BatchNorm scale 1 / shift 0, linear layers uniform
+-1/sqrt(fan_in).  Convolution weights are stored [C_out, 3, 3, C_in].
"""
import numpy as np

from . import rng

BASE_SEED = 250808540

# Sizes of the workloads this repository measures or tests.  'tau' is the number of local
# updates of the fast process per round, 'tau_workers' the per-worker step counts of a round (the
# aggregation weights follow from them on either side of a comparison: the oracle's weights_from_tau
# and the library's bls_weights_from_tau; this package computes none).
WORKLOADS = {
    "mlp": dict(id=0, model="mlp", pool=256, classes=10, k=64, batch=64, tau=4, lr=0.1, momentum=0.0,
                weight_decay=0.0, P=4, weights=(0.35, 0.35, 0.15, 0.15)),
    "resnet20_fp32": dict(id=1, model="resnet20", pool=512, classes=10, k=128, batch=128, tau=20, lr=0.1,
                          momentum=0.9, weight_decay=0.0, P=10, tau_workers=(32,) * 8 + (16,) * 2),
    # the same pool and selection with the batch size and local step count of the paper's own ResNet20 runs (batch 32,
    # tau_F = 32; hyper-parameter table of the appendix, Section 5.1): 1024 samples per pass, the selection walked cyclically
    "resnet20_b32": dict(id=1, model="resnet20", pool=512, classes=10, k=128, batch=32, tau=32, lr=0.1,
                         momentum=0.9, weight_decay=1e-4, P=10, tau_workers=(32,) * 8 + (16,) * 2),
    # the same network with bf16 activations and fp32 master weights, larger pool and selection
    "resnet20_bf16": dict(id=2, model="resnet20", act_dtype="bf16", pool=4096, classes=10, k=1024, batch=128, tau=50,
                          lr=0.1, momentum=0.9, weight_decay=0.0, P=10, tau_workers=(32,) * 8 + (16,) * 2),
    # wide residual network WRN-16-8, bf16 activations / fp32 master weights, 100 classes
    "wrn16_8_bf16": dict(id=3, model="wrn16_8", act_dtype="bf16", pool=2048, classes=100, k=512, batch=128, tau=4,
                         lr=0.1, momentum=0.9, weight_decay=0.0, P=10, tau_workers=(32,) * 8 + (16,) * 2),
    # encoder language model: 6 layers, d 512, 8 heads, FFN 2048, vocabulary 32000, sequences of 128 tokens
    # (bf16 factors in every matrix product, fp32 sums, storage and master weights; the _fp32 variant multiplies in fp32)
    "transformer": dict(id=4, model="transformer", act_dtype="bf16", pool=1024, classes=32000, seq_len=128, k=256, batch=64, tau=4,
                        lr=0.001, momentum=0.9, weight_decay=0.0, P=10, tau_workers=(32,) * 8 + (16,) * 2),
    "transformer_fp32": dict(id=4, model="transformer", pool=1024, classes=32000, seq_len=128, k=256, batch=64, tau=4,
                             lr=0.001, momentum=0.9, weight_decay=0.0, P=10, tau_workers=(32,) * 8 + (16,) * 2),
}


def workload(name):
    return dict(WORKLOADS[name])


def _seed(workload_id):
    return BASE_SEED + int(workload_id)


def image_pool(workload_id, n, classes, hw=32, channels=3, stream=0):
    """(x float32 [n, hw, hw, channels], y int32 [n])."""
    seed = _seed(workload_id)
    y = rng.randint(seed, 100 + stream, n, classes).astype(np.int32)
    per = hw * hw * channels
    mu = 0.5 * rng.normal(seed, 200 + stream, classes * per).reshape(classes, per)
    noise = rng.normal(seed, 300 + stream, n * per).reshape(n, per)
    x = (mu[y] + noise).astype(np.float32).reshape(n, hw, hw, channels)
    return x, y


def mlp_tensor_specs(d_in=3072, hidden=128, classes=10):
    """[(name, shape)] of the trainable tensors, in flat-vector order."""
    return [("fc1.weight", (hidden, d_in)), ("fc1.bias", (hidden,)),
            ("fc2.weight", (classes, hidden)), ("fc2.bias", (classes,))]


def _linear_init(seed, stream, out_f, in_f):
    bound = 1.0 / np.sqrt(in_f)
    w = (2.0 * rng.uniform01(seed, stream, out_f * in_f) - 1.0) * bound
    b = (2.0 * rng.uniform01(seed, stream + 1, out_f) - 1.0) * bound
    return w.reshape(out_f, in_f).astype(np.float32), b.astype(np.float32)


def mlp_init(workload_id, d_in=3072, hidden=128, classes=10):
    seed = _seed(workload_id)
    w1, b1 = _linear_init(seed, 1000, hidden, d_in)
    w2, b2 = _linear_init(seed, 1002, classes, hidden)
    return {"fc1.weight": w1, "fc1.bias": b1, "fc2.weight": w2, "fc2.bias": b2}


def resnet_tensor_specs(widths=(16, 32, 64), blocks=3, classes=10, in_channels=3):
    """(params, buffers): [(name, shape)] lists in flat-vector order.

    CIFAR-style residual network: a 3x3 stem convolution, len(widths) stages of `blocks`
    two-convolution residual blocks (the first block of every stage but the first has
    stride 2 and a parameter-free shortcut), global average pooling and a linear layer.
    """
    params, buffers = [], []

    def bn(prefix, c):
        params.append((prefix + ".weight", (c,)))
        params.append((prefix + ".bias", (c,)))
        buffers.append((prefix + ".running_mean", (c,)))
        buffers.append((prefix + ".running_var", (c,)))

    params.append(("stem.conv.weight", (widths[0], 3, 3, in_channels)))
    bn("stem.bn", widths[0])
    c_prev = widths[0]
    for s, c in enumerate(widths):
        for b in range(blocks):
            p = "s%d.b%d" % (s + 1, b)
            params.append((p + ".conv1.weight", (c, 3, 3, c_prev)))
            bn(p + ".bn1", c)
            params.append((p + ".conv2.weight", (c, 3, 3, c)))
            bn(p + ".bn2", c)
            c_prev = c
    params.append(("fc.weight", (classes, widths[-1])))
    params.append(("fc.bias", (classes,)))
    return params, buffers


def resnet_init(workload_id, widths=(16, 32, 64), blocks=3, classes=10, in_channels=3,
                perturb_bn=0.0):
    """(params dict, buffers dict) of float32 arrays.

    perturb_bn > 0 moves BatchNorm scale/shift and running statistics off their defaults
    (scale 1 +- perturb, shift +- perturb, mean +- perturb, var in [1, 1 + perturb]) so that
    tests exercise every term; 0 gives the standard initial state.
    """
    seed = _seed(workload_id)
    p_specs, b_specs = resnet_tensor_specs(widths, blocks, classes, in_channels)
    params, buffers = {}, {}
    for t, (name, shape) in enumerate(p_specs):
        n = int(np.prod(shape))
        stream = 2000 + 4 * t
        if name.endswith("conv.weight") or ".conv1." in name or ".conv2." in name:
            fan_out = shape[0] * 9
            params[name] = (rng.normal(seed, stream, n) * np.sqrt(2.0 / fan_out)).reshape(shape).astype(np.float32)
        elif name == "fc.weight":
            w, b = _linear_init(seed, stream, shape[0], shape[1])
            params["fc.weight"], params["fc.bias"] = w, b
        elif name == "fc.bias":
            pass
        elif name.endswith(".weight"):   # BatchNorm scale
            params[name] = (1.0 + perturb_bn * (2.0 * rng.uniform01(seed, stream, n) - 1.0)).astype(np.float32)
        else:                            # BatchNorm shift
            params[name] = (perturb_bn * (2.0 * rng.uniform01(seed, stream, n) - 1.0)).astype(np.float32)
    for t, (name, shape) in enumerate(b_specs):
        n = int(np.prod(shape))
        stream = 6000 + 4 * t
        if name.endswith("running_mean"):
            buffers[name] = (perturb_bn * (2.0 * rng.uniform01(seed, stream, n) - 1.0)).astype(np.float32)
        else:
            buffers[name] = (1.0 + perturb_bn * rng.uniform01(seed, stream, n)).astype(np.float32)
    return params, buffers


def wrn_tensor_specs(widths=(128, 256, 512), blocks=2, classes=100, stem=16, in_channels=3):
    """(params, buffers) of a pre-activation wide residual network, in flat-vector order.

    Per block: bn1, conv1, bn2, conv2 and, where the block changes the shape, a 1x1 shortcut
    convolution; after the last block a final batch norm and the linear classifier.
    """
    params, buffers = [], []

    def bn(prefix, c):
        params.append((prefix + ".weight", (c,)))
        params.append((prefix + ".bias", (c,)))
        buffers.append((prefix + ".running_mean", (c,)))
        buffers.append((prefix + ".running_var", (c,)))

    params.append(("stem.conv.weight", (stem, 3, 3, in_channels)))
    c_prev = stem
    for s, c in enumerate(widths):
        for b in range(blocks):
            p = "s%d.b%d" % (s + 1, b)
            stride = 2 if (b == 0 and s > 0) else 1
            bn(p + ".bn1", c_prev)
            params.append((p + ".conv1.weight", (c, 3, 3, c_prev)))
            bn(p + ".bn2", c)
            params.append((p + ".conv2.weight", (c, 3, 3, c)))
            if c_prev != c or stride != 1:
                params.append((p + ".shortcut.weight", (c, 1, 1, c_prev)))
            c_prev = c
    bn("final.bn", widths[-1])
    params.append(("fc.weight", (classes, widths[-1])))
    params.append(("fc.bias", (classes,)))
    return params, buffers


def wrn_init(workload_id, widths=(128, 256, 512), blocks=2, classes=100, stem=16, in_channels=3, perturb_bn=0.0):
    """(params dict, buffers dict) of float32 arrays for wrn_tensor_specs; same conventions as resnet_init."""
    seed = _seed(workload_id)
    p_specs, b_specs = wrn_tensor_specs(widths, blocks, classes, stem, in_channels)
    params, buffers = {}, {}
    for t, (name, shape) in enumerate(p_specs):
        n = int(np.prod(shape))
        stream = 12000 + 4 * t
        if len(shape) == 4:
            fan_out = shape[0] * shape[1] * shape[2]
            params[name] = (rng.normal(seed, stream, n) * np.sqrt(2.0 / fan_out)).reshape(shape).astype(np.float32)
        elif name == "fc.weight":
            w, b = _linear_init(seed, stream, shape[0], shape[1])
            params["fc.weight"], params["fc.bias"] = w, b
        elif name == "fc.bias":
            pass
        elif name.endswith(".weight"):
            params[name] = (1.0 + perturb_bn * (2.0 * rng.uniform01(seed, stream, n) - 1.0)).astype(np.float32)
        else:
            params[name] = (perturb_bn * (2.0 * rng.uniform01(seed, stream, n) - 1.0)).astype(np.float32)
    for t, (name, shape) in enumerate(b_specs):
        n = int(np.prod(shape))
        stream = 16000 + 4 * t
        if name.endswith("running_mean"):
            buffers[name] = (perturb_bn * (2.0 * rng.uniform01(seed, stream, n) - 1.0)).astype(np.float32)
        else:
            buffers[name] = (1.0 + perturb_bn * rng.uniform01(seed, stream, n)).astype(np.float32)
    return params, buffers


def transformer_tensor_specs(vocab=32000, seq_len=128, d_model=512, d_ff=2048, layers=6):
    """[(name, shape)] of the encoder language model's parameters, in flat-vector order (no buffers)."""
    specs = [("tok_emb.weight", (vocab, d_model)), ("pos_emb.weight", (seq_len, d_model))]
    for l in range(layers):
        n = "l%d." % l
        for a in ("q", "k", "v", "o"):
            specs += [(n + "attn.%s.weight" % a, (d_model, d_model)), (n + "attn.%s.bias" % a, (d_model,))]
        specs += [(n + "ln1.weight", (d_model,)), (n + "ln1.bias", (d_model,)),
                  (n + "ffn.fc1.weight", (d_ff, d_model)), (n + "ffn.fc1.bias", (d_ff,)),
                  (n + "ffn.fc2.weight", (d_model, d_ff)), (n + "ffn.fc2.bias", (d_model,)),
                  (n + "ln2.weight", (d_model,)), (n + "ln2.bias", (d_model,))]
    specs.append(("head.weight", (vocab, d_model)))
    return specs


def transformer_init(workload_id, vocab=32000, seq_len=128, d_model=512, d_ff=2048, layers=6, perturb=0.0):
    """Parameters dict: embeddings N(0, 0.02), linear weights uniform +-1/sqrt(fan_in) with biases alike,
    layer-norm scale 1 / shift 0 (moved by `perturb` in tests)."""
    seed = _seed(workload_id)
    out = {}
    for t, (name, shape) in enumerate(transformer_tensor_specs(vocab, seq_len, d_model, d_ff, layers)):
        n = int(np.prod(shape))
        stream = 20000 + 4 * t
        if name.endswith("emb.weight"):
            out[name] = (0.02 * rng.normal(seed, stream, n)).reshape(shape).astype(np.float32)
        elif ".ln" in name:
            base = 1.0 if name.endswith("weight") else 0.0
            out[name] = (base + perturb * (2.0 * rng.uniform01(seed, stream, n) - 1.0)).astype(np.float32)
        else:
            fan_in = shape[1] if len(shape) == 2 else {"fc2": d_ff}.get(name.split(".")[-2], d_model)
            out[name] = ((2.0 * rng.uniform01(seed, stream, n) - 1.0) / np.sqrt(fan_in)).reshape(shape).astype(np.float32)
    return out


def token_pool(workload_id, n, seq_len=128, vocab=32000, zipf_s=1.1, stream=0):
    """(inputs int32 [n, seq_len], targets int32 [n, seq_len]): token ranks drawn from a Zipf(s) law truncated to the
    vocabulary by inverse CDF, id = rank - 1; seq_len + 1 tokens per sequence, the target of a position is the next token."""
    seed = _seed(workload_id)
    w = 1.0 / np.arange(1, vocab + 1, dtype=np.float64) ** zipf_s
    cdf = np.cumsum(w) / w.sum()
    u = rng.uniform01(seed, 400 + stream, n * (seq_len + 1))
    ids = np.minimum(np.searchsorted(cdf, u, side="left"), vocab - 1).astype(np.int32).reshape(n, seq_len + 1)
    return np.ascontiguousarray(ids[:, :-1]), np.ascontiguousarray(ids[:, 1:])


def replicas(base, P, workload_id, scale=0.01):
    """P distinct copies of a flat float32 vector: base + scale * N(0, I), float32 [P, d]."""
    seed = _seed(workload_id)
    d = base.size
    out = np.empty((P, d), dtype=np.float32)
    for i in range(P):
        out[i] = (base.astype(np.float64) + scale * rng.normal(seed, 9000 + i, d)).astype(np.float32)
    return out


LOSS_ARRAY_KINDS = ("halfnormal", "ties16", "equal", "ascending", "descending", "specials")


def loss_array(kind, n, seed=BASE_SEED, classes=10):
    """float32 loss arrays for selection tests and sweeps.

    halfnormal: |N(0,1)| + ln(classes); ties16: the same quantised to 16 distinct values;
    equal: one value; ascending / descending: strictly monotone; specials: halfnormal with
    NaN, +-inf, +-0 and repeated values planted at seeded positions.
    """
    base = (np.abs(rng.normal(seed, 7000, n)) + np.log(classes)).astype(np.float32)
    if kind == "halfnormal":
        return base
    if kind == "ties16":
        lo, hi = float(base.min()), float(base.max()) + 1e-6
        q = np.floor((base - lo) / (hi - lo) * 16.0)
        return (lo + q * (hi - lo) / 16.0).astype(np.float32)
    if kind == "equal":
        return np.full(n, np.float32(np.log(classes)), dtype=np.float32)
    if kind == "ascending":
        return (np.arange(n, dtype=np.float64) / max(n, 1)).astype(np.float32) if n < (1 << 24) else \
            np.arange(n, dtype=np.float32)
    if kind == "descending":
        return loss_array("ascending", n, seed, classes)[::-1].copy()
    if kind == "specials":
        out = base.copy()
        if n:
            pos = rng.randint(seed, 7001, min(n, 64), n)
            vals = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 1.0, 1.0, -np.nan], dtype=np.float32)
            out[pos] = vals[np.arange(pos.size) % vals.size]
        return out
    raise ValueError(kind)
