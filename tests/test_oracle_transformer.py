"""Pins of the encoder language model in the oracle: parameter count worked by hand, finite-difference
gradients on a tiny instance, layer norm / GELU / attention against their definitions, loss special cases."""
import math

import numpy as np

import oracle
import synth
from oracle import transformer as T


def test_parameter_count_of_the_measured_configuration():
    # embeddings 32000*512 + 128*512; per layer 4*(512*512 + 512) + 2*512 + (2048*512 + 2048) + (512*2048 + 512) + 2*512
    # = 3 152 384; six layers; output projection 32000*512
    specs = synth.transformer_tensor_specs()
    total = sum(int(np.prod(s)) for _, s in specs)
    assert total == 16384000 + 65536 + 6 * 3152384 + 16384000 == 51747840


def test_gelu_and_layernorm_definitions():
    x = np.linspace(-4, 4, 41)
    np.testing.assert_allclose(T.gelu(x), [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x], rtol=1e-15)
    eps = 1e-6
    np.testing.assert_allclose(T.gelu_grad(x), (T.gelu(x + eps) - T.gelu(x - eps)) / (2 * eps), rtol=1e-7, atol=1e-9)
    assert T.gelu(0.0) == 0.0 and abs(T.gelu(10.0) - 10.0) < 1e-12 and abs(T.gelu(-10.0)) < 1e-12
    rs = np.random.RandomState(0)
    v = rs.standard_normal((3, 5, 8)) * 3 + 1
    y, _ = T.layernorm(v, np.ones(8), np.zeros(8))
    np.testing.assert_allclose(y.mean(axis=-1), 0, atol=1e-12)
    np.testing.assert_allclose((y ** 2).mean(axis=-1), v.var(axis=-1) / (v.var(axis=-1) + 1e-5), rtol=1e-12)


def test_token_cross_entropy():
    rs = np.random.RandomState(1)
    z = rs.standard_normal((2, 3, 7))
    t = rs.randint(0, 7, (2, 3))
    loss, dz = T.token_cross_entropy(z, t)
    for b in range(2):
        ref = np.mean([-math.log(math.exp(z[b, l, t[b, l]]) / np.exp(z[b, l]).sum()) for l in range(3)])
        assert abs(loss[b] - ref) < 1e-12
    np.testing.assert_allclose(dz.sum(axis=-1), 0, atol=1e-14)
    l0, _ = T.token_cross_entropy(np.zeros((1, 4, 9)), np.zeros((1, 4), dtype=int))
    assert abs(l0[0] - math.log(9)) < 1e-14


def _tiny():
    m = oracle.TransformerLM(vocab=11, seq_len=5, d_model=8, heads=2, d_ff=12, layers=2)
    p = synth.transformer_init(7, 11, 5, 8, 12, 2, perturb=0.3)
    p = {k: v.astype(np.float64) * (5.0 if "emb" in k else 1.0) for k, v in p.items()}
    x, y = synth.token_pool(7, 4, 5, 11)
    return m, p, x, y


def test_attention_matches_a_direct_loop():
    m, p, x, y = _tiny()
    logits, cache, _ = m.forward(p, {}, x, train=True)
    c = cache["layers"][0]
    h = c["x"]
    b, head, dh = 1, 1, 4
    Wq, Wk, Wv = p["l0.attn.q.weight"], p["l0.attn.k.weight"], p["l0.attn.v.weight"]
    sl = slice(head * dh, (head + 1) * dh)
    q = h[b] @ Wq.T[:, sl] + p["l0.attn.q.bias"][sl]
    k = h[b] @ Wk.T[:, sl] + p["l0.attn.k.bias"][sl]
    v = h[b] @ Wv.T[:, sl] + p["l0.attn.v.bias"][sl]
    for i in range(5):
        w = np.array([math.exp(q[i] @ k[j] / 2.0) for j in range(5)])
        np.testing.assert_allclose(c["ctx"][b, i, sl], (w / w.sum()) @ v, rtol=1e-12)
    # no causal mask: the first position attends to later ones
    assert c["a"][b, head, 0, 4] > 0


def test_gradients_finite_differences():
    m, p, x, y = _tiny()
    losses, grads, _ = oracle.loss_and_grads(m, p, {}, x, y)
    assert set(grads) == set(p) and losses.shape == (4,)
    eps = 1e-6
    for name, t in p.items():
        flat = t.reshape(-1)
        picks = range(flat.size) if flat.size <= 10 else synth.randint(8, len(name), 10, flat.size)
        for i in picks:
            old = flat[i]
            flat[i] = old + eps
            lp = oracle.loss_and_grads(m, p, {}, x, y)[0].mean()
            flat[i] = old - eps
            lm = oracle.loss_and_grads(m, p, {}, x, y)[0].mean()
            flat[i] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grads[name].reshape(-1)[i]) <= 3e-5 * max(1e-4, abs(fd)), (name, i, fd, grads[name].reshape(-1)[i])


def test_scores_and_zero_head():
    m, p, x, y = _tiny()
    s = oracle.score_losses(m, p, {}, x, y)
    np.testing.assert_allclose(oracle.score_losses(m, p, {}, x[1:3], y[1:3]), s[1:3], rtol=1e-13)
    p2 = dict(p)
    p2["head.weight"] = np.zeros_like(p["head.weight"])
    np.testing.assert_allclose(oracle.score_losses(m, p2, {}, x, y), math.log(11), rtol=1e-14)


def test_token_pool_follows_the_zipf_law():
    x, y = synth.token_pool(4, 400, 128, 32000)
    assert x.shape == (400, 128) and y.shape == (400, 128) and x.dtype == np.int32
    np.testing.assert_array_equal(x[:, 1:], y[:, :-1])            # targets are the next tokens
    assert x.min() >= 0 and max(x.max(), y.max()) < 32000
    ids = np.concatenate([x.reshape(-1), y[:, -1]])
    w = 1.0 / np.arange(1, 32001) ** 1.1
    p0 = w[0] / w.sum()
    n = ids.size
    assert abs((ids == 0).mean() - p0) < 5 * math.sqrt(p0 * (1 - p0) / n)
    p9 = w[:10].sum() / w.sum()
    assert abs((ids < 10).mean() - p9) < 5 * math.sqrt(p9 * (1 - p9) / n)


def test_operand_hook_rounds_exactly_the_factors_of_every_product():
    """Mixed-precision reading: only the two factors of a matrix product are rounded.  Pinned by products worked by hand,
    by a model whose every factor is already representable (nothing may change), and by counting the hook's calls."""
    m = T.TransformerLM(20, 4, 8, 2, 8, 1, operand=oracle.round_bf16)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 and goes to the even 1; 1 + 3 * 2^-9 is nearest to 1 + 2^-7
    assert m._mm(np.array([[1.0 + 2.0 ** -8]]), np.array([[3.0]]))[0, 0] == 3.0
    assert m._mm(np.array([[1.0 + 3 * 2.0 ** -9]]), np.array([[3.0]]))[0, 0] == 3.0 * (1.0 + 2.0 ** -7)
    assert m._outer_sum(np.full((1, 2, 1), 1.0 + 2.0 ** -8), np.full((1, 2, 1), 0.5))[0, 0] == 1.0
    # factors that bf16 holds exactly (multiples of 1/8 below 16) are left alone
    a, b = np.arange(-12, 12).reshape(4, 6) / 8.0, np.arange(30).reshape(6, 5) / 8.0
    assert np.array_equal(m._mm(a, b), a @ b)
    # one forward and backward pass calls the hook twice per product: per layer 6 linear + 2 attention products forward,
    # 6 weight gradients + 6 input gradients + 4 attention products backward; the head adds 1 + 2
    calls = []
    counted = T.TransformerLM(20, 4, 8, 2, 8, 2, operand=lambda t: (calls.append(1), t)[1])
    p = synth.transformer_init(4, 20, 4, 8, 8, 2, perturb=0.1)
    x, y = synth.token_pool(4, 3, 4, 20)
    exact = T.TransformerLM(20, 4, 8, 2, 8, 2)
    l0, g0, _ = oracle.loss_and_grads(exact, p, {}, x, y)
    l1, g1, _ = oracle.loss_and_grads(counted, p, {}, x, y)
    assert len(calls) == 2 * (2 * (8 + 16) + 3)
    assert np.array_equal(l0, l1) and all(np.array_equal(g0[k], g1[k]) for k in g0)   # the identity hook changes nothing
    # rounding moves losses and gradients by about the bf16 spacing, not more and not zero
    rounded = T.TransformerLM(20, 4, 8, 2, 8, 2, operand=oracle.round_bf16)
    l2, g2, _ = oracle.loss_and_grads(rounded, p, {}, x, y)
    assert 0 < np.abs(l2 - l0).max() < 2e-2 * np.abs(l0).max()
    err = max(np.linalg.norm(g2[k] - g0[k]) / np.linalg.norm(g0[k]) for k in g0 if not k.endswith("attn.k.bias"))
    assert 1e-4 < err < 0.15, err
