"""Meta-Weight-Net style sample weighting w(loss; lambda) (Sec. 4.1): a 1 -> H -> 1 MLP, ReLU hidden
layer, sigmoid output.  lambda is flat [W1(H), b1(H), W2(H), b2(1)].  Float64."""
import numpy as np


def split(lam):
    H = (len(lam) - 1) // 3
    return lam[:H], lam[H:2 * H], lam[2 * H:3 * H], lam[3 * H]


def weights(losses, lam):
    """w_i = sigmoid(W2 . relu(W1 l_i + b1) + b2)."""
    W1, b1, W2, b2 = split(lam)
    a = np.outer(losses, W1) + b1
    z = np.maximum(a, 0.0) @ W2 + b2
    return 1.0 / (1.0 + np.exp(-z))


def base_loss(losses, lam, mask=None):
    """L_base = (1/B_eff) sum_i mask_i w(l_i; lambda) l_i (Sec. 4.1)."""
    mask = np.ones_like(losses) if mask is None else mask.astype(np.float64)
    return float(np.sum(mask * weights(losses, lam) * losses) / np.sum(mask))


def base_loss_grad_lambda(losses, lam, mask=None):
    """dL_base/dlambda at fixed per-sample losses: lambda reaches L_base only through w, so
    d/dlambda = (1/B_eff) sum_i mask_i l_i dw(l_i; lambda)/dlambda."""
    W1, b1, W2, b2 = split(lam)
    mask = np.ones_like(losses) if mask is None else mask.astype(np.float64)
    a = np.outer(losses, W1) + b1                      # [B, H]
    r = np.maximum(a, 0.0)
    z = r @ W2 + b2
    w = 1.0 / (1.0 + np.exp(-z))
    dz = w * (1.0 - w) * losses * mask / np.sum(mask)  # [B]
    da = np.outer(dz, W2) * (a > 0.0)                  # ReLU subgradient 0 at 0
    return np.concatenate([da.T @ losses, da.sum(axis=0), r.T @ dz, [dz.sum()]])
