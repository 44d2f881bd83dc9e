"""Label-correction meta learner c(x, y; lambda_c) of the noisy-finetuning problem (Sec. 4.1): the base loss of a noisy
sample is the cross-entropy against a corrected soft label,

    L_base = (1/B_eff) sum_i mask_i w(l_i; lambda_r) l_i,    l_i = -sum_k c_ik log softmax(z_i)_k,   c_i = c(x_i, y_i; lambda_c).

The paper names the corrector only as a "2-layer MLP" (Table 4) and cites meta label correction; its inputs and
parametrisation are not given.  reading (defined here, where the paper is silent): the corrector sees the given label
and the base learner's current prediction, both as constants,

    u_i = [onehot(y_i), softmax(z_i)]  (2C inputs),   s_i = kappa onehot(y_i) + W2 relu(W1 u_i + b1) + b2,   c_i = softmax(s_i),

a 2C -> Hc -> C MLP with ReLU hidden layer (subgradient 0 at 0) on top of a fixed prior kappa on the given label, so
that an untrained corrector leaves the labels nearly unchanged.  lambda_c is flat [W1(Hc x 2C), b1(Hc), W2(C x Hc),
b2(C)].  Float64.  Test infrastructure: only tests, smoke() and bench.py's cpu_baseline may use it."""
import numpy as np


def size(C, Hc):
    return Hc * 2 * C + Hc + C * Hc + C


def split(lam_c, C, Hc):
    o = 0
    W1 = lam_c[o:o + Hc * 2 * C].reshape(Hc, 2 * C); o += Hc * 2 * C
    b1 = lam_c[o:o + Hc]; o += Hc
    W2 = lam_c[o:o + C * Hc].reshape(C, Hc); o += C * Hc
    b2 = lam_c[o:o + C]
    return W1, b1, W2, b2


def softmax(z):
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def forward(lam_c, y, p, Hc, kappa):
    """Soft labels c[B, C] and what the backward pass needs.  y: int labels [B]; p: softmax of the logits [B, C]."""
    B, C = p.shape
    W1, b1, W2, b2 = split(lam_c, C, Hc)
    onehot = np.zeros((B, C)); onehot[np.arange(B), y] = 1.0
    u = np.concatenate([onehot, p], axis=1)                 # [B, 2C]
    a = u @ W1.T + b1                                       # [B, Hc]
    h = np.maximum(a, 0.0)
    s = kappa * onehot + h @ W2.T + b2                      # [B, C]
    c = softmax(s)
    return c, (u, a, h, c)


def backward(lam_c, cache, dc, Hc):
    """d/dlambda_c of sum_ik dc_ik c_ik at fixed inputs u."""
    u, a, h, c = cache
    C = c.shape[1]
    W1, b1, W2, b2 = split(lam_c, C, Hc)
    ds = c * (dc - (dc * c).sum(axis=1, keepdims=True))     # softmax backward
    dW2 = ds.T @ h
    db2 = ds.sum(axis=0)
    da = (ds @ W2) * (a > 0.0)
    dW1 = da.T @ u
    db1 = da.sum(axis=0)
    return np.concatenate([dW1.ravel(), db1, dW2.ravel(), db2])
