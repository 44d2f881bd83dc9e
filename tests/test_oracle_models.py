"""Pins for oracle/models.py and oracle/wnet.py: float64 PyTorch library modules with autograd as an
independent implementation of the same functions, plus explicit loops on tiny shapes."""
import numpy as np
import pytest
import torch
from datagen import CounterRNG, param_layout, param_count
from oracle import models, wnet


def _theta(n, seed, scale=0.2):
    return scale * CounterRNG(seed).normal(1, n)


def test_layouts_agree_with_datagen():
    for kind, dims in (("mlp", (32, 2)), ("mlp", (7, 5, 3)), ("encoder", (2, 16, 4, 32, 8, 50, 3))):
        m = models.make_model(kind, dims)
        assert m.n == param_count(kind, dims)
        for name, shape, off in param_layout(kind, dims):
            assert m.slices[name] == (off, tuple(shape))


def test_logreg_by_loops():
    m = models.MLP((4, 3))
    th = _theta(m.n, 1, 1.0)
    r = CounterRNG(2)
    x = r.normal(1, 5 * 4).reshape(5, 4); y = r.integers(2, 5, 3); coef = r.uniform(3, 5)
    W = th[:12].reshape(3, 4); b = th[12:]
    l_ref = np.zeros(5); g_ref = np.zeros(m.n)
    for i in range(5):
        z = [sum(W[c, f] * x[i, f] for f in range(4)) + b[c] for c in range(3)]
        lse = np.log(sum(np.exp(zc) for zc in z))
        l_ref[i] = lse - z[y[i]]
        for c in range(3):
            dz = coef[i] * (np.exp(z[c] - lse) - (1.0 if c == y[i] else 0.0))
            for f in range(4):
                g_ref[c * 4 + f] += dz * x[i, f]
            g_ref[12 + c] += dz
    l, g = m.loss_grad(th, x, y, coef)
    assert np.allclose(l, l_ref, rtol=1e-12) and np.allclose(g, g_ref, rtol=1e-12, atol=1e-14)
    assert np.allclose(m.losses(th, x, y), l_ref, rtol=1e-12)


def test_mlp_vs_torch_autograd():
    widths = (6, 5, 4, 3)
    m = models.MLP(widths)
    th = _theta(m.n, 3, 0.7)
    r = CounterRNG(4)
    x = r.normal(1, 9 * 6).reshape(9, 6); y = r.integers(2, 9, 3); coef = r.uniform(3, 9)
    t = torch.tensor(th, dtype=torch.float64, requires_grad=True)
    h = torch.tensor(x)
    for l in range(3):
        off, shape = m.slices[f"W{l}"]; offb, _ = m.slices[f"b{l}"]
        W = t[off:off + shape[0] * shape[1]].reshape(shape); b = t[offb:offb + shape[0]]
        h = h @ W.T + b
        if l < 2:
            h = torch.relu(h)
    lt = torch.nn.functional.cross_entropy(h, torch.tensor(y), reduction="none")
    (lt * torch.tensor(coef)).sum().backward()
    l, g = m.loss_grad(th, x, y, coef)
    assert np.allclose(l, lt.detach().numpy(), rtol=1e-12)
    assert np.allclose(g, t.grad.numpy(), rtol=1e-10, atol=1e-13)


def _torch_encoder_losses(enc, th, ids, y, lens=None):
    """The same classifier assembled from torch.nn library layers (post-LN TransformerEncoderLayer,
    exact GELU), float64, parameters sliced out of one flat leaf tensor; lens = the library's key_padding_mask."""
    t = torch.tensor(th, dtype=torch.float64, requires_grad=True)

    def P(name):
        off, shape = enc.slices[name]
        return t[off:off + int(np.prod(shape))].reshape(shape)
    F = torch.nn.functional
    ids_t = torch.tensor(np.asarray(ids), dtype=torch.long)
    B, S = ids_t.shape
    kpm = None if lens is None else torch.arange(S)[None, :] >= torch.tensor(np.asarray(lens))[:, None]
    x = F.embedding(ids_t, P("tok_emb")) + P("pos_emb")[:S]
    x = F.layer_norm(x, (enc.d,), P("emb_ln_g"), P("emb_ln_b"), 1e-5)
    for l in range(enc.L):
        p = f"l{l}."
        xs = x.transpose(0, 1)                                    # [S,B,d] for the functional MHA
        a, _ = F.multi_head_attention_forward(xs, xs, xs, enc.d, enc.heads, P(p + "Wqkv"), P(p + "bqkv"), None, None,
                                              False, 0.0, P(p + "Wo"), P(p + "bo"), training=False, need_weights=False,
                                              key_padding_mask=kpm)
        x = F.layer_norm(x + a.transpose(0, 1), (enc.d,), P(p + "ln1_g"), P(p + "ln1_b"), 1e-5)
        f = F.linear(F.gelu(F.linear(x, P(p + "W1"), P(p + "b1"))), P(p + "W2"), P(p + "b2"))
        x = F.layer_norm(x + f, (enc.d,), P(p + "ln2_g"), P(p + "ln2_b"), 1e-5)
    logits = F.linear(x[:, 0, :], P("Wc"), P("bc"))
    return t, F.cross_entropy(logits, torch.tensor(y, dtype=torch.long), reduction="none")


@pytest.mark.parametrize("dims", [(2, 16, 4, 32, 8, 50, 3), (1, 24, 3, 40, 5, 30, 2), (2, 128, 2, 256, 128, 300, 3)])   # the last: S = 128, head width 64 as on the GPU
def test_encoder_vs_torch_autograd(dims):
    enc = models.Encoder(*dims)
    L, d, heads, ffn, S, V, C = dims
    th = _theta(enc.n, 5, 0.3)
    for name in ("emb_ln_g",) + tuple(f"l{l}.ln{k}_g" for l in range(L) for k in (1, 2)):
        enc.get(th, name)[...] += 1.0
    r = CounterRNG(6)
    B = 4
    ids = r.integers(1, B * S, V).reshape(B, S); ids[:, 0] = 0; ids[1, 3] = ids[1, 2]     # a repeated token
    y = r.integers(2, B, C); coef = r.uniform(3, B)
    t, lt = _torch_encoder_losses(enc, th, ids, y)
    (lt * torch.tensor(coef)).sum().backward()
    l, g = enc.loss_grad(th, ids, y, coef)
    assert np.allclose(l, lt.detach().numpy(), rtol=1e-11)
    assert np.allclose(enc.losses(th, ids, y), l, rtol=1e-13)
    gt = t.grad.numpy()
    assert np.max(np.abs(g - gt)) <= 1e-10 * np.max(np.abs(gt))
    for name, (off, shape) in enc.slices.items():                 # every parameter group on its own scale
        sl = slice(off, off + int(np.prod(shape)))
        assert np.max(np.abs(g[sl] - gt[sl])) <= 1e-9 * (np.max(np.abs(gt[sl])) + 1e-12), name


@pytest.mark.parametrize("dims", [(2, 16, 4, 32, 8, 50, 3), (1, 128, 2, 128, 128, 90, 2)])
def test_encoder_padding_vs_torch_key_padding_mask(dims):
    """Padded batches: losses and every gradient group against torch's multi-head attention with key_padding_mask;
    what sits in the padded positions must not matter; ids that occur only as padding get exactly no gradient; full
    lengths are the unpadded model bit for bit."""
    enc = models.Encoder(*dims)
    L, d, heads, ffn, S, V, C = dims
    th = _theta(enc.n, 15, 0.3)
    r = CounterRNG(16)
    B = 5
    ids = r.integers(1, B * S, V - 1).reshape(B, S); ids[:, 0] = 0
    lens = np.array([S, 1, S // 2, 3, S - 1])
    y = r.integers(2, B, C); coef = r.uniform(3, B)
    t, lt = _torch_encoder_losses(enc, th, ids, y, lens)
    (lt * torch.tensor(coef)).sum().backward()
    l, g = enc.loss_grad(th, models.with_lengths(ids, lens), y, coef)
    assert np.allclose(l, lt.detach().numpy(), rtol=1e-11)
    gt = t.grad.numpy()
    for name, (off, shape) in enc.slices.items():
        sl = slice(off, off + int(np.prod(shape)))
        assert np.max(np.abs(g[sl] - gt[sl])) <= 1e-9 * (np.max(np.abs(gt[sl])) + 1e-12), name
    # the mask matters on this input
    l_nomask = enc.losses(th, ids, y)
    assert np.max(np.abs(l_nomask - l)) > 1e-3
    # padded positions: any token there gives the same numbers; the pad token itself gets no gradient
    ids2 = ids.copy()
    for b in range(B):
        ids2[b, lens[b]:] = V - 1
    l2, g2 = enc.loss_grad(th, models.with_lengths(ids2, lens), y, coef)
    assert np.allclose(l2, l, rtol=1e-13)
    tok = enc.slices["tok_emb"][0]
    others = np.ones(enc.n, dtype=bool); others[tok:tok + V * d] = False
    assert np.allclose(g2[others], g[others], rtol=1e-11, atol=1e-14)
    assert np.all(enc.get(g2, "tok_emb")[V - 1] == 0.0)
    # full lengths = no mask
    lf, gf = enc.loss_grad(th, models.with_lengths(ids, np.full(B, S)), y, coef)
    l0, g0 = enc.loss_grad(th, ids, y, coef)
    assert np.array_equal(lf, l0) and np.array_equal(gf, g0)


def test_wnet_vs_torch_and_loops():
    H, B = 7, 6
    r = CounterRNG(7)
    lam = r.normal(1, 3 * H + 1); losses = np.abs(r.normal(2, B)) + 0.1
    mask = np.array([1, 1, 0, 1, 1, 0], dtype=np.uint8)
    # loops
    w_ref = np.zeros(B)
    for i in range(B):
        z = lam[3 * H]
        for h in range(H):
            z += lam[2 * H + h] * max(lam[h] * losses[i] + lam[H + h], 0.0)
        w_ref[i] = 1 / (1 + np.exp(-z))
    assert np.allclose(wnet.weights(losses, lam), w_ref, rtol=1e-13)
    assert abs(wnet.base_loss(losses, lam, mask) - (w_ref * losses * mask).sum() / 4) < 1e-14
    # autograd
    t = torch.tensor(lam, requires_grad=True)
    lt = torch.tensor(losses)
    a = torch.relu(lt[:, None] * t[:H] + t[H:2 * H])
    w = torch.sigmoid(a @ t[2 * H:3 * H] + t[3 * H])
    ((w * lt * torch.tensor(mask.astype(np.float64))).sum() / 4).backward()
    assert np.allclose(wnet.base_loss_grad_lambda(losses, lam, mask), t.grad.numpy(), rtol=1e-11, atol=1e-14)
    # a masked-out sample cannot matter, whatever its loss
    losses2 = losses.copy(); losses2[2] = 1e6
    assert np.array_equal(wnet.base_loss_grad_lambda(losses, lam, mask), wnet.base_loss_grad_lambda(losses2, lam, mask))
