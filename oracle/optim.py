"""Base-level solvers u and their diagonal adaptation du/dg (Sec. 3.2 Eq. 4; App. C). Float64."""
import numpy as np

ADAPT_ADAM, ADAPT_NONE = 0, 1


def adam_update(theta, m, v, g, t, lr, beta1, beta2, eps):
    """One bias-corrected Adam step (Kingma & Ba, Alg. 1); t is the 1-based count of this step.
    Returns (theta', m', v').  In the paper's notation theta' = theta - u(g)."""
    m2 = beta1 * m + (1.0 - beta1) * g
    v2 = beta2 * v + (1.0 - beta2) * g * g
    mhat = m2 / (1.0 - beta1 ** t)
    vhat = v2 / (1.0 - beta2 ** t)
    return theta - lr * mhat / (np.sqrt(vhat) + eps), m2, v2


def sgd_update(theta, g, lr):
    """theta' = theta - u, u = lr * g (Sec. 2, the solver below Eq. 2)."""
    return theta - lr * g


def sgd_momentum_update(theta, buf, g, lr, mu):
    """SGD with heavy-ball momentum mu, the form the common frameworks' SGD takes with a `momentum` argument
    (no dampening, no Nesterov look-ahead): b' = mu b + g, theta' = theta - lr b'.  The paper's hyperparameter
    tables (App. B) name only "SGD"; reading: this form.  Returns (theta', b').  In the paper's notation
    u(g) = lr (mu b + g), so du/dg = lr as for plain SGD (sgd_adaptation)."""
    b2 = mu * buf + g
    return theta - lr * b2, b2


def adam_adaptation(g, m_post, v_post, t, lr, beta1, beta2, eps, keep_eps_term=False):
    """Diagonal of du_adam/dg (App. C), evaluated with the moments AFTER the step that consumed g
    (m' = beta1 m + (1-beta1) g, v' = beta2 v + (1-beta2) g^2) and that step's bias corrections.

    With c1 = 1/(1-beta1^t), c2 = 1/sqrt(1-beta2^t), s = sqrt(v'):
        u(g)  = lr c1 m' / (c2 s + eps)
        du/dg = lr c1 [ c2((1-beta1) v' - (1-beta2) m' g) + (1-beta1) eps s ] / [ s (c2 s + eps)^2 ]
    The appendix drops the eps term of the numerator (eps << 1); that is the default here.
    Elements with s = 0 (no gradient history) get 0.
    """
    c1 = 1.0 / (1.0 - beta1 ** t)
    c2 = 1.0 / np.sqrt(1.0 - beta2 ** t)
    s = np.sqrt(v_post)
    num = c2 * ((1.0 - beta1) * v_post - (1.0 - beta2) * m_post * g)
    if keep_eps_term:
        num = num + (1.0 - beta1) * eps * s
    den = s * (c2 * s + eps) ** 2
    out = np.zeros_like(g)
    nz = s > 0
    out[nz] = lr * c1 * num[nz] / den[nz]
    return out


def sgd_adaptation(g, lr):
    """du/dg for u = lr g: the scalar lr on the diagonal (identity up to the step size, Sec. 3.2)."""
    return np.full_like(g, lr)
