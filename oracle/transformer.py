"""Transformer encoder language model of the sequence workload, forward and backward, in float64.

The paper's language workload fine-tunes a pretrained encoder for classification (Section 5); the measured
configuration here is a stand-in of the same shape class trained from scratch: token + learned position
embeddings, `layers` post-layer-norm encoder blocks
    h = LN1(h + MHA(h)),   h = LN2(h + W2 gelu(W1 h + b1) + b2)
with full (unmasked) self-attention over `heads` heads, the erf form of GELU, layer-norm eps 1e-5, and an
untied, bias-free output projection to the vocabulary.  The target of position t is the token that follows
it in the generated sequence; the loss of a sample is the mean of its per-position cross-entropies, so that
the sampler still ranks one float per sample (Section 4.3).
Linear weights are [out, in]; parameters are a dict keyed by tensor name; there are no buffers.

Mixed precision: with `operand` set (e.g. round_bf16) both operands of every matrix product, forward and backward,
pass through it before they are multiplied; sums, activations and everything else stay float64.  The default is the
exact model.
"""
import math

import numpy as np

LN_EPS = 1e-5
_SQRT2 = math.sqrt(2.0)
try:
    from scipy.special import erf as _erf          # the same function, evaluated array-wise
except ImportError:                                 # pragma: no cover
    _erf = np.vectorize(math.erf, otypes=[np.float64])


def gelu(x):
    return 0.5 * x * (1.0 + _erf(x / _SQRT2))


def gelu_grad(x):
    return 0.5 * (1.0 + _erf(x / _SQRT2)) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def layernorm(x, g, b):
    """Normalisation over the last axis; returns (y, cache)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    inv = 1.0 / np.sqrt(var + LN_EPS)
    xhat = (x - mu) * inv
    return xhat * g + b, (xhat, inv, g)


def layernorm_backward(dy, cache):
    xhat, inv, g = cache
    d = dy.shape[-1]
    dg = (dy * xhat).reshape(-1, d).sum(axis=0)
    db = dy.reshape(-1, d).sum(axis=0)
    dxhat = dy * g
    dx = inv * (dxhat - dxhat.mean(axis=-1, keepdims=True) - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


def token_cross_entropy(logits, targets):
    """logits [B, L, V], targets int [B, L] -> (per-sample loss [B] = mean over positions, d loss_b / d logits)."""
    z = np.asarray(logits, dtype=np.float64)
    B, L, V = z.shape
    m = z.max(axis=-1, keepdims=True)
    e = np.exp(z - m)
    s = e.sum(axis=-1, keepdims=True)
    bi, li = np.meshgrid(np.arange(B), np.arange(L), indexing="ij")
    tok = (m[..., 0] + np.log(s[..., 0])) - z[bi, li, targets]
    p = e / s
    p[bi, li, targets] -= 1.0
    return tok.mean(axis=1), p / L


class TransformerLM:
    has_buffers = False

    def __init__(self, vocab=32000, seq_len=128, d_model=512, heads=8, d_ff=2048, layers=6, operand=None):
        self.vocab, self.seq_len, self.d_model, self.heads, self.d_ff, self.layers = vocab, seq_len, d_model, heads, d_ff, layers
        self.operand = operand if operand is not None else (lambda a: a)

    def _mm(self, a, b):
        """a @ b with both operands passed through the operand hook."""
        return self.operand(a) @ self.operand(b)

    def _outer_sum(self, dy, x):
        """sum over tokens of dy (outer) x: the weight gradient [out, in] of y = x W^T."""
        return np.tensordot(self.operand(dy), self.operand(x), axes=([0, 1], [0, 1]))

    def sample_losses(self, logits, targets):
        return token_cross_entropy(logits, targets)

    def forward(self, params, buffers, tokens, train):
        p = {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}
        tokens = np.asarray(tokens).astype(np.int64)
        B, L = tokens.shape
        D, H = self.d_model, self.heads
        dh = D // H
        h = p["tok_emb.weight"][tokens] + p["pos_emb.weight"][:L]
        cache = {"p": p, "tokens": tokens, "layers": []}
        for l in range(self.layers):
            n = "l%d." % l
            c = {"x": h}
            lin = lambda name, x: self._mm(x, p[n + name + ".weight"].T) + p[n + name + ".bias"]
            split = lambda t: t.reshape(B, L, H, dh).transpose(0, 2, 1, 3)          # [B, H, L, dh]
            q, k, v = split(lin("attn.q", h)), split(lin("attn.k", h)), split(lin("attn.v", h))
            s = self._mm(q, k.transpose(0, 1, 3, 2)) / math.sqrt(dh)
            s = s - s.max(axis=-1, keepdims=True)
            a = np.exp(s)
            a = a / a.sum(axis=-1, keepdims=True)
            ctx = self._mm(a, v).transpose(0, 2, 1, 3).reshape(B, L, D)
            c.update(q=q, k=k, v=v, a=a, ctx=ctx)
            h1, c["ln1"] = layernorm(h + lin("attn.o", ctx), p[n + "ln1.weight"], p[n + "ln1.bias"])
            c["h1"] = h1
            u = lin("ffn.fc1", h1)
            gact = gelu(u)
            c.update(u=u, g=gact)
            h, c["ln2"] = layernorm(h1 + lin("ffn.fc2", gact), p[n + "ln2.weight"], p[n + "ln2.bias"])
            cache["layers"].append(c)
        cache["final"] = h
        return self._mm(h, p["head.weight"].T), cache, dict(buffers)

    def backward(self, cache, dlogits):
        p, tokens = cache["p"], cache["tokens"]
        B, L = tokens.shape
        D, H = self.d_model, self.heads
        dh = D // H
        g = {}
        hf = cache["final"]
        g["head.weight"] = self._outer_sum(dlogits, hf)
        dh_ = self._mm(dlogits, p["head.weight"])

        def lin_back(name, x, dy):
            g[name + ".weight"] = self._outer_sum(dy, x)
            g[name + ".bias"] = dy.reshape(-1, dy.shape[-1]).sum(axis=0)
            return self._mm(dy, p[name + ".weight"])

        for l in reversed(range(self.layers)):
            n = "l%d." % l
            c = cache["layers"][l]
            dr, g[n + "ln2.weight"], g[n + "ln2.bias"] = layernorm_backward(dh_, c["ln2"])
            dg = lin_back(n + "ffn.fc2", c["g"], dr)
            dh1 = dr + lin_back(n + "ffn.fc1", c["h1"], dg * gelu_grad(c["u"]))
            dr1, g[n + "ln1.weight"], g[n + "ln1.bias"] = layernorm_backward(dh1, c["ln1"])
            dctx = lin_back(n + "attn.o", c["ctx"], dr1).reshape(B, L, H, dh).transpose(0, 2, 1, 3)
            a, q, k, v = c["a"], c["q"], c["k"], c["v"]
            dv = self._mm(a.transpose(0, 1, 3, 2), dctx)
            da = self._mm(dctx, v.transpose(0, 1, 3, 2))
            ds = a * (da - (da * a).sum(axis=-1, keepdims=True)) / math.sqrt(dh)
            dq, dk = self._mm(ds, k), self._mm(ds.transpose(0, 1, 3, 2), q)
            merge = lambda t: t.transpose(0, 2, 1, 3).reshape(B, L, D)
            x = c["x"]
            dh_ = dr1 + lin_back(n + "attn.q", x, merge(dq)) + lin_back(n + "attn.k", x, merge(dk)) + lin_back(n + "attn.v", x, merge(dv))
        g["pos_emb.weight"] = np.zeros_like(p["pos_emb.weight"])
        g["pos_emb.weight"][:L] = dh_.sum(axis=0)
        g["tok_emb.weight"] = np.zeros_like(p["tok_emb.weight"])
        np.add.at(g["tok_emb.weight"], tokens.reshape(-1), dh_.reshape(-1, D))
        return g
