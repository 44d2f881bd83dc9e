"""The optimizer- and problem-agnostic part of SAMA (Sec. 3.2, Eq. 5). Float64.

Callers supply the base problem as a function glam(theta) = dL_base(theta, lambda)/dlambda.
"""
import numpy as np


def perturbation(D, g_meta):
    """v = (du/dg) . dL_meta/dtheta with a diagonal adaptation (Eq. 4-5)."""
    return D * g_meta


def step_size(v, alpha):
    """eps = alpha / ||v||_2, one norm over every element of theta (below Eq. 5).
    Returns 0.0 when the norm is zero or not finite (the step is then skipped)."""
    nrm = float(np.sqrt(np.sum(v * v)))
    if not np.isfinite(nrm) or nrm == 0.0:
        return 0.0
    return alpha / nrm


def central_difference(glam, theta, v, eps):
    """-(dL_base(theta+,.)/dlambda - dL_base(theta-,.)/dlambda) / (2 eps), theta+- = theta +- eps v (Eq. 5)."""
    gp = glam(theta + eps * v)
    gm = glam(theta - eps * v)
    if eps == 0.0:
        return np.zeros_like(gp), gp, gm
    return -(gp - gm) / (2.0 * eps), gp, gm


def hypergradient(glam, theta, D, g_meta, alpha):
    """Whole Eq. 5: returns (h, eps, v)."""
    v = perturbation(D, g_meta)
    eps = step_size(v, alpha)
    h, _, _ = central_difference(glam, theta, v, eps)
    return h, eps, v


def nudge(theta, v, eps):
    """theta <- theta - eps v at every meta update (end of Sec. 3.2)."""
    return theta - eps * v
