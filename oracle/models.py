"""Base learners f(x; theta) with per-sample cross-entropy and hand-written backward. Float64.

Two families: a ReLU MLP (zero hidden layers = multinomial logistic regression) and a post-LN
transformer encoder classifier (the BERT/RoBERTa-shaped base learners of Sec. 4.1).  Both expose
    losses(theta, x, y)            -> l[B]            per-sample CE, l_i = logsumexp(z_i) - z_i[y_i]
                                                      (y may also be soft targets [B, C]: l_i = -sum_k y_ik log p_ik)
    loss_grad(theta, x, y, coef)   -> (l[B], d/dtheta sum_i coef_i l_i)
theta is one flat vector.  Layout (the interface of the C library, restated here independently):
every weight matrix ([out x in], row-major) in layer order, then every other tensor in layer order.
"""
import numpy as np
from scipy.special import erf


def _ce(logits, y):
    """Per-sample cross-entropy against integer labels y[B], or against soft targets y[B, C] (rows summing to 1):
    l_i = -sum_k y_ik log softmax(z_i)_k = logsumexp(z_i) - y_i . z_i."""
    zmax = logits.max(axis=1, keepdims=True)
    lse = np.log(np.exp(logits - zmax).sum(axis=1)) + zmax[:, 0]
    y = np.asarray(y)
    if y.ndim == 2:
        return lse - (y * logits).sum(axis=1)
    return lse - logits[np.arange(len(y)), y]


def _dce(logits, y, coef):
    """d/dlogits of sum_i coef_i l_i = coef_i (softmax(z_i) - target_i), target = onehot(y_i) or the soft row y_i."""
    p = np.exp(logits - logits.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    y = np.asarray(y)
    if y.ndim == 2:
        p -= y
    else:
        p[np.arange(len(y)), y] -= 1.0
    return p * coef[:, None]


class MLP:
    def __init__(self, widths):
        self.widths = tuple(int(w) for w in widths)
        self.slices = {}
        off = 0
        L = len(self.widths) - 1
        for l in range(L):
            sz = self.widths[l + 1] * self.widths[l]
            self.slices[f"W{l}"] = (off, (self.widths[l + 1], self.widths[l])); off += sz
        for l in range(L):
            self.slices[f"b{l}"] = (off, (self.widths[l + 1],)); off += self.widths[l + 1]
        self.n = off
        self.L = L

    def get(self, theta, name):
        off, shape = self.slices[name]
        return theta[off:off + int(np.prod(shape))].reshape(shape)

    def _forward(self, theta, x):
        acts = [np.asarray(x, dtype=np.float64)]
        pre = []
        for l in range(self.L):
            a = acts[-1] @ self.get(theta, f"W{l}").T + self.get(theta, f"b{l}")
            pre.append(a)
            acts.append(np.maximum(a, 0.0) if l < self.L - 1 else a)
        return acts, pre

    def logits(self, theta, x):
        return self._forward(theta, x)[0][-1]

    def losses(self, theta, x, y):
        return _ce(self.logits(theta, x), y)

    def loss_grad(self, theta, x, y, coef):
        acts, pre = self._forward(theta, x)
        l = _ce(acts[-1], y)
        g = np.zeros(self.n)
        d = _dce(acts[-1], y, np.asarray(coef, dtype=np.float64))
        for k in reversed(range(self.L)):
            self.get(g, f"W{k}")[...] = d.T @ acts[k]
            self.get(g, f"b{k}")[...] = d.sum(axis=0)
            if k > 0:
                d = (d @ self.get(theta, f"W{k}")) * (pre[k - 1] > 0.0)
        return l, g


def _ln_fwd(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xh = (x - mu) * rstd
    return xh * g + b, (xh, rstd)


def _ln_bwd(dy, g, cache):
    xh, rstd = cache
    dg = (dy * xh).reshape(-1, xh.shape[-1]).sum(axis=0)
    db = dy.reshape(-1, xh.shape[-1]).sum(axis=0)
    dxh = dy * g
    dx = rstd * (dxh - dxh.mean(axis=-1, keepdims=True) - xh * (dxh * xh).mean(axis=-1, keepdims=True))
    return dx, dg, db


def _gelu(a):
    return 0.5 * a * (1.0 + erf(a / np.sqrt(2.0)))


def _dgelu(a):
    return 0.5 * (1.0 + erf(a / np.sqrt(2.0))) + a * np.exp(-0.5 * a * a) / np.sqrt(2.0 * np.pi)


def with_lengths(ids, lens):
    """An encoder input with padding: ids [B, S] and the number of real tokens of each sequence.  Every method of
    Encoder that takes `ids` takes this pair as well."""
    ids, lens = np.asarray(ids), np.asarray(lens)
    assert ids.ndim == 2 and lens.shape == (ids.shape[0],) and lens.min() >= 1 and lens.max() <= ids.shape[1]
    return (ids, lens)


def split_lengths(x):
    """(ids, lens or None) of an encoder input."""
    if isinstance(x, tuple):
        return np.asarray(x[0]), np.asarray(x[1])
    return np.asarray(x), None


def cat_inputs(a, b):
    """Two encoder inputs stacked along the batch axis (lengths kept if either has them)."""
    (ia, la), (ib, lb) = split_lengths(a), split_lengths(b)
    ids = np.concatenate([ia, ib], axis=0)
    if la is None and lb is None:
        return ids
    S = ids.shape[1]
    la = np.full(len(ia), S) if la is None else la
    lb = np.full(len(ib), S) if lb is None else lb
    return (ids, np.concatenate([la, lb]))


class Encoder:
    """Post-LN encoder: x0 = LN(tok[ids] + pos); per layer x <- LN1(x + Attn(x)), x <- LN2(x + FFN(x));
    logits = x_L[:, 0] Wc^T + bc.  erf-GELU, LN eps 1e-5, softmax(q k^T / sqrt(d_h)).  Padding (reading: the usual
    key-padding mask of text batches, which the paper's language-model workloads imply): with lengths given
    (with_lengths), keys at positions >= len_b get no attention weight; nothing else changes.
    mlm=True adds the masked-token head of the auxiliary task (Sec. 4.3): token logits x_L[b, s] Wmlm^T + bmlm at the
    masked positions (reading: an untied linear decoder on the last LayerNorm's output)."""
    LN_EPS = 1e-5

    def __init__(self, L, d, heads, ffn, S, V, C, mlm=False):
        self.L, self.d, self.heads, self.ffn, self.S, self.V, self.C = L, d, heads, ffn, S, V, C
        self.mlm = bool(mlm)
        self.slices = {}
        off = 0

        def add(name, shape):
            nonlocal off
            self.slices[name] = (off, shape)
            off += int(np.prod(shape))
        for l in range(L):
            add(f"l{l}.Wqkv", (3 * d, d)); add(f"l{l}.Wo", (d, d))
            add(f"l{l}.W1", (ffn, d)); add(f"l{l}.W2", (d, ffn))
        if mlm:
            add("Wmlm", (V, d))
        for l in range(L):
            add(f"l{l}.bqkv", (3 * d,)); add(f"l{l}.bo", (d,))
            add(f"l{l}.ln1_g", (d,)); add(f"l{l}.ln1_b", (d,))
            add(f"l{l}.b1", (ffn,)); add(f"l{l}.b2", (d,))
            add(f"l{l}.ln2_g", (d,)); add(f"l{l}.ln2_b", (d,))
        add("tok_emb", (V, d)); add("pos_emb", (S, d))
        add("emb_ln_g", (d,)); add("emb_ln_b", (d,))
        if mlm:
            add("bmlm", (V,))
        add("Wc", (C, d)); add("bc", (C,))
        self.n = off

    def get(self, theta, name):
        off, shape = self.slices[name]
        return theta[off:off + int(np.prod(shape))].reshape(shape)

    def _forward(self, theta, ids, keep):
        ids, lens = split_lengths(ids)
        P = lambda name: self.get(theta, name)
        B, S = ids.shape
        pad = None if lens is None else (np.arange(S)[None, :] >= lens[:, None])[:, None, None, :]   # [B,1,1,S] keys
        d, nh = self.d, self.heads
        dh = d // nh
        cache = []
        x, c0 = _ln_fwd(P("tok_emb")[ids] + P("pos_emb")[None, :S], P("emb_ln_g"), P("emb_ln_b"), self.LN_EPS)
        for l in range(self.L):
            p = f"l{l}."
            qkv = x @ P(p + "Wqkv").T + P(p + "bqkv")                      # [B,S,3d]
            q, k, v = (qkv[..., i * d:(i + 1) * d].reshape(B, S, nh, dh).transpose(0, 2, 1, 3) for i in range(3))
            s = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(dh)               # [B,nh,S,S]
            if pad is not None:
                s = np.where(pad, -np.inf, s)
            s = s - s.max(axis=-1, keepdims=True)
            pr = np.exp(s)
            pr /= pr.sum(axis=-1, keepdims=True)
            o = (pr @ v).transpose(0, 2, 1, 3).reshape(B, S, d)
            x1, c1 = _ln_fwd(x + o @ P(p + "Wo").T + P(p + "bo"), P(p + "ln1_g"), P(p + "ln1_b"), self.LN_EPS)
            a = x1 @ P(p + "W1").T + P(p + "b1")
            hgelu = _gelu(a)
            x2, c2 = _ln_fwd(x1 + hgelu @ P(p + "W2").T + P(p + "b2"), P(p + "ln2_g"), P(p + "ln2_b"), self.LN_EPS)
            if keep:
                cache.append((x, q, k, v, pr, o, c1, x1, a, hgelu, c2))
            x = x2
        logits = x[:, 0, :] @ P("Wc").T + P("bc")
        return logits, (c0, cache, x)

    def logits(self, theta, ids):
        return self._forward(theta, ids, False)[0]

    def losses(self, theta, ids, y):
        return _ce(self.logits(theta, ids), y)

    def mlm_logits(self, xL, theta, seq, pos):
        return xL[seq, pos, :] @ self.get(theta, "Wmlm").T + self.get(theta, "bmlm")

    def mlm_losses(self, theta, ids, seq, pos, tgt):
        """Cross-entropy over the vocabulary at each masked position (seq[j], pos[j]) against tgt[j]."""
        xL = self._forward(theta, ids, False)[1][2]
        return _ce(self.mlm_logits(xL, theta, seq, pos), tgt)

    def loss_grad(self, theta, ids, y, coef):
        """(l, g): l_i = CE(z_i, y_i), g = d/dtheta sum_i coef_i l_i."""
        l, _, g = self.loss_grad_mlm(theta, ids, y, coef, None, None, None, None)
        return l, g

    def loss_grad_mlm(self, theta, ids, y, coef, seq, pos, tgt, coef_pos):
        """(l, l_pos, g): classification losses l_i, masked-token losses l_pos_j, and
        g = d/dtheta [sum_i coef_i l_i + sum_j coef_pos_j l_pos_j] from ONE forward/backward over `ids`."""
        x_in = ids
        ids = split_lengths(ids)[0]
        P = lambda name: self.get(theta, name)
        g = np.zeros(self.n)
        G = lambda name: self.get(g, name)
        B, S = ids.shape
        d, nh = self.d, self.heads
        dh = d // nh
        logits, (c0, cache, xL) = self._forward(theta, x_in, True)
        l = _ce(logits, y)
        dlog = _dce(logits, y, np.asarray(coef, dtype=np.float64))        # [B,C]
        G("Wc")[...] = dlog.T @ xL[:, 0, :]
        G("bc")[...] = dlog.sum(axis=0)
        dx = np.zeros((B, S, d))
        dx[:, 0, :] = dlog @ P("Wc")
        l_pos = None
        if seq is not None:
            zt = self.mlm_logits(xL, theta, seq, pos)                      # [n_mask, V]
            l_pos = _ce(zt, tgt)
            dzt = _dce(zt, tgt, np.asarray(coef_pos, dtype=np.float64))
            G("Wmlm")[...] = dzt.T @ xL[seq, pos, :]
            G("bmlm")[...] = dzt.sum(axis=0)
            np.add.at(dx, (seq, pos), dzt @ P("Wmlm"))
        for l_ in reversed(range(self.L)):
            p = f"l{l_}."
            x, q, k, v, pr, o, c1, x1, a, hgelu, c2 = cache[l_]
            dsum, dg_, db_ = _ln_bwd(dx, P(p + "ln2_g"), c2)
            G(p + "ln2_g")[...] = dg_; G(p + "ln2_b")[...] = db_
            G(p + "W2")[...] = dsum.reshape(-1, d).T @ hgelu.reshape(-1, self.ffn)
            G(p + "b2")[...] = dsum.reshape(-1, d).sum(axis=0)
            da = (dsum @ P(p + "W2")) * _dgelu(a)
            G(p + "W1")[...] = da.reshape(-1, self.ffn).T @ x1.reshape(-1, d)
            G(p + "b1")[...] = da.reshape(-1, self.ffn).sum(axis=0)
            dx1 = dsum + da @ P(p + "W1")
            dsum1, dg_, db_ = _ln_bwd(dx1, P(p + "ln1_g"), c1)
            G(p + "ln1_g")[...] = dg_; G(p + "ln1_b")[...] = db_
            G(p + "Wo")[...] = dsum1.reshape(-1, d).T @ o.reshape(-1, d)
            G(p + "bo")[...] = dsum1.reshape(-1, d).sum(axis=0)
            do = (dsum1 @ P(p + "Wo")).reshape(B, S, nh, dh).transpose(0, 2, 1, 3)     # [B,nh,S,dh]
            dv = pr.transpose(0, 1, 3, 2) @ do
            dpr = do @ v.transpose(0, 1, 3, 2)
            ds = pr * (dpr - (dpr * pr).sum(axis=-1, keepdims=True)) / np.sqrt(dh)
            dq = ds @ k
            dk = ds.transpose(0, 1, 3, 2) @ q
            dqkv = np.concatenate([t.transpose(0, 2, 1, 3).reshape(B, S, d) for t in (dq, dk, dv)], axis=-1)
            G(p + "Wqkv")[...] = dqkv.reshape(-1, 3 * d).T @ x.reshape(-1, d)
            G(p + "bqkv")[...] = dqkv.reshape(-1, 3 * d).sum(axis=0)
            dx = dsum1 + dqkv @ P(p + "Wqkv")
        demb, dg_, db_ = _ln_bwd(dx, P("emb_ln_g"), c0)
        G("emb_ln_g")[...] = dg_; G("emb_ln_b")[...] = db_
        G("pos_emb")[:S] = demb.sum(axis=0)
        np.add.at(G("tok_emb"), ids.reshape(-1), demb.reshape(-1, d))
        return l, l_pos, g


def make_model(kind, dims, mlm=False):
    if kind == "mlp":
        return MLP(dims)
    if kind == "encoder":
        return Encoder(*dims, mlm=mlm)
    raise ValueError(kind)
