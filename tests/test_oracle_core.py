"""Pins for oracle/sama_core.py (Eq. 5) on problems whose hypergradient has a closed form:
per-sample-weighted least squares and the biased-regression setting of App. D."""
import numpy as np
from datagen import CounterRNG
from oracle import sama_core


def _sig(z):
    return 1.0 / (1.0 + np.exp(-z))


def test_weighted_least_squares_closed_form():
    """L_base = (1/B) sum sigma(lam_i) 1/2 (x_i.theta - y_i)^2 : dL_base/dlam is quadratic in theta, so the
    central difference is exact: h_i = -(1/B) sigma'(lam_i) r_i (x_i . v)."""
    r = CounterRNG(11)
    B, n = 12, 5
    X = r.normal(1, B * n).reshape(B, n); y = r.normal(2, B); lam = r.normal(3, B)
    theta = r.normal(4, n); D = np.abs(r.normal(5, n)); gmeta = r.normal(6, n)
    sp = _sig(lam) * (1 - _sig(lam))
    glam = lambda th: sp * 0.5 * (X @ th - y) ** 2 / B
    for alpha in (1.0, 1e-2, 7.0):
        h, eps, v = sama_core.hypergradient(glam, theta, D, gmeta, alpha)
        assert np.allclose(v, D * gmeta, rtol=0, atol=0)
        assert abs(eps * np.linalg.norm(v) - alpha) < 1e-14 * alpha
        want = -sp * (X @ theta - y) * (X @ v) / B
        assert np.allclose(h, want, rtol=1e-10, atol=1e-13)
    th2 = sama_core.nudge(theta, v, eps)
    assert np.allclose(th2, theta - eps * v, rtol=0, atol=0)


def test_zero_direction_is_skipped():
    h, eps, v = sama_core.hypergradient(lambda th: th[:2], np.ones(3), np.zeros(3), np.ones(3), 1.0)
    assert eps == 0.0 and np.all(h == 0.0)
    assert sama_core.step_size(np.array([np.nan, 1.0]), 1.0) == 0.0


def _biased(seed=21, N=40, Nm=30, n=8, beta=0.1, ortho=False):
    r = CounterRNG(seed)
    X = r.normal(1, N * n).reshape(N, n)
    if ortho:
        X = 1.7 * np.linalg.qr(X)[0]               # X^T X = 1.7^2 I
    Xm = r.normal(2, Nm * n).reshape(Nm, n)
    wt = r.normal(3, n)
    y = X @ wt + 0.1 * r.normal(4, N); ym = Xm @ wt + 0.1 * r.normal(5, Nm)
    return X, y, Xm, ym, beta


def _wstar(X, y, beta, lam):
    n = X.shape[1]
    return np.linalg.solve(X.T @ X + beta * np.eye(n), X.T @ y + beta * lam)


def test_biased_regression_closed_forms_hold():
    """App. D's g_lambda and lambda* (objectives read with a factor 1/2) against a numerical derivative of
    L_meta(w*(lambda)) and against the stationarity of lambda*."""
    X, y, Xm, ym, beta = _biased()
    n = X.shape[1]
    lam = CounterRNG(22).normal(1, n)
    Hinv = np.linalg.inv(X.T @ X + beta * np.eye(n))
    w = _wstar(X, y, beta, lam)
    g_closed = beta * Hinv @ (Xm.T @ Xm @ w - Xm.T @ ym)
    Lm = lambda l: 0.5 * np.sum((Xm @ _wstar(X, y, beta, l) - ym) ** 2)
    fd = np.array([(Lm(lam + 1e-5 * e) - Lm(lam - 1e-5 * e)) / 2e-5 for e in np.eye(n)])
    assert np.allclose(g_closed, fd, rtol=1e-6, atol=1e-9)
    A = beta * Xm @ Hinv; b = ym - Xm @ Hinv @ X.T @ y
    lam_star = np.linalg.solve(A.T @ A, A.T @ b)
    ws = _wstar(X, y, beta, lam_star)
    assert np.max(np.abs(beta * Hinv @ (Xm.T @ Xm @ ws - Xm.T @ ym))) < 1e-8


def test_biased_regression_sama_sgd():
    """dL_base/dlambda = -beta (w - lambda) is linear in w: Eq. 5 gives h = beta * v exactly; with an SGD base
    solver v = gamma dL_meta/dw.  When X^T X + beta I = c I this is c*gamma times the exact hypergradient."""
    for ortho in (False, True):
        X, y, Xm, ym, beta = _biased(ortho=ortho)
        n = X.shape[1]
        lam = CounterRNG(23).normal(1, n)
        w = _wstar(X, y, beta, lam)
        gmeta = Xm.T @ (Xm @ w - ym)
        gamma = 0.05
        glam = lambda wv: -beta * (wv - lam)
        h, eps, v = sama_core.hypergradient(glam, w, np.full(n, gamma), gmeta, 1.0)
        assert np.allclose(h, beta * gamma * gmeta, rtol=1e-9, atol=1e-12)
        exact = beta * np.linalg.solve(X.T @ X + beta * np.eye(n), gmeta)
        if ortho:
            c = 1.7 ** 2 + beta
            assert np.allclose(h, c * gamma * exact, rtol=1e-8)
        cos = h @ exact / np.linalg.norm(h) / np.linalg.norm(exact)
        assert cos > 0.5


def test_biased_regression_converges():
    """App. D / Fig. 5 protocol: beta = 0.1, 100 meta updates; the identity-approximated meta gradient keeps
    a high cosine with the closed form and ||lambda_t - lambda*|| falls."""
    X, y, Xm, ym, beta = _biased(seed=31)
    n = X.shape[1]
    Hinv = np.linalg.inv(X.T @ X + beta * np.eye(n))
    A = beta * Xm @ Hinv; b = ym - Xm @ Hinv @ X.T @ y
    lam_star = np.linalg.solve(A.T @ A, A.T @ b)
    lam = np.zeros(n)
    d0 = np.linalg.norm(lam - lam_star)
    dist, coss = [], []
    for _ in range(100):
        w = _wstar(X, y, beta, lam)
        gmeta = Xm.T @ (Xm @ w - ym)
        h, eps, v = sama_core.hypergradient(lambda wv: -beta * (wv - lam), w, np.ones(n), gmeta, 1.0)
        exact = beta * Hinv @ gmeta
        coss.append(h @ exact / (np.linalg.norm(h) * np.linalg.norm(exact) + 1e-300))
        lam = lam - 2.0 * h
        dist.append(np.linalg.norm(lam - lam_star))
    assert min(coss) > 0.5
    assert dist[-1] < 0.8 * d0 and all(b_ <= a_ + 1e-12 for a_, b_ in zip(dist, dist[1:]))
