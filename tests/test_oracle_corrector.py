"""Pins for the label-correction part of the oracle (oracle/corrector.py and its use in oracle/reweight.py; Sec. 4.1):
a second implementation of the corrector with torch autograd, differences of the scalar base loss, the soft-target
cross-entropy against its hard-label special case, and the limit of a dominant label prior in which everything must
reduce to plain data reweighting."""
import numpy as np
import pytest
from datagen import CounterRNG
from oracle import corrector, models, wnet
from oracle.reweight import SamaOracle


def _tiny(seed=77, B=18, Bm=9, F=6, C=4, H=5, Hc=7):
    r = CounterRNG(seed)
    model = models.MLP((F, 8, C))
    x = r.normal(1, B * F).reshape(B, F); y = r.integers(2, B, C)
    xm = r.normal(3, Bm * F).reshape(Bm, F); ym = r.integers(4, Bm, C)
    th = 0.5 * r.normal(5, model.n)
    lam_r = np.concatenate([r.normal(6, H), np.abs(r.normal(7, H)), r.normal(8, H), [0.1]])
    lam_c = 0.7 * r.normal(9, corrector.size(C, Hc))
    return model, x, y, xm, ym, th, lam_r, lam_c, C, Hc


def test_soft_target_cross_entropy_reduces_to_hard_labels_and_matches_differences():
    model, x, y, *_ , th, lam_r, lam_c, C, Hc = _tiny()
    onehot = np.eye(C)[y]
    coef = np.linspace(0.2, 1.0, len(y))
    l_h, g_h = model.loss_grad(th, x, y, coef)
    l_s, g_s = model.loss_grad(th, x, onehot, coef)
    assert np.allclose(l_h, l_s, rtol=0, atol=1e-13) and np.allclose(g_h, g_s, rtol=0, atol=1e-13)
    r = CounterRNG(5)
    soft = np.abs(r.normal(1, len(y) * C)).reshape(len(y), C); soft /= soft.sum(axis=1, keepdims=True)
    l, g = model.loss_grad(th, x, soft, coef)
    p = corrector.softmax(model.logits(th, x))
    assert np.allclose(l, -(soft * np.log(p)).sum(axis=1), rtol=1e-12)              # the definition written out
    S = lambda t: float(np.sum(coef * model.losses(t, x, soft)))
    for k in (0, 7, model.n // 2, model.n - 1):
        e = np.zeros(model.n); e[k] = 1e-6
        assert abs((S(th + e) - S(th - e)) / 2e-6 - g[k]) < 1e-7 * (1 + abs(g[k]))


def test_corrector_matches_torch_autograd():
    torch = pytest.importorskip("torch")
    _, _, y, _, _, _, _, lam_c, C, Hc = _tiny()
    r = CounterRNG(11)
    B = len(y)
    p = corrector.softmax(r.normal(1, B * C).reshape(B, C))
    dc = r.normal(2, B * C).reshape(B, C)
    kappa = 1.3
    c, cache = corrector.forward(lam_c, y, p, Hc, kappa)
    g = corrector.backward(lam_c, cache, dc, Hc)
    t = torch.tensor(lam_c, dtype=torch.float64, requires_grad=True)
    o = 0
    W1 = t[o:o + Hc * 2 * C].reshape(Hc, 2 * C); o += Hc * 2 * C
    b1 = t[o:o + Hc]; o += Hc
    W2 = t[o:o + C * Hc].reshape(C, Hc); o += C * Hc
    b2 = t[o:o + C]
    onehot = torch.nn.functional.one_hot(torch.tensor(y), C).double()
    u = torch.cat([onehot, torch.tensor(p)], dim=1)
    s = kappa * onehot + torch.nn.functional.linear(torch.relu(torch.nn.functional.linear(u, W1, b1)), W2, b2)
    ct = torch.softmax(s, dim=1)
    (ct * torch.tensor(dc)).sum().backward()
    assert np.allclose(c, ct.detach().numpy(), rtol=1e-12, atol=1e-14)
    assert np.allclose(g, t.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.allclose(c.sum(axis=1), 1.0)


def test_glam_equals_differences_of_the_scalar_base_loss_with_the_stated_stop_gradients():
    """lambda_r part: d/dlambda_r of (1/B_eff) sum mask w(l_i; lambda_r) l_i at fixed l_i; lambda_c part:
    d/dlambda_c of (1/B_eff) sum mask w_i l_i(lambda_c) at fixed w_i and fixed softmax(z_i)."""
    model, x, y, xm, ym, th, lam_r, lam_c, C, Hc = _tiny()
    mask = (np.arange(len(y)) % 4 != 1).astype(np.uint8)
    kappa = 2.0
    lam = np.concatenate([lam_r, lam_c])
    orc = SamaOracle(model, th, lam, corr_hidden=Hc, corr_kappa=kappa, n_classes=C)
    got = orc.glam(th, x, y, mask)
    z = model.logits(th, x)
    p = corrector.softmax(z)
    logp = np.log(p)
    mk = mask.astype(np.float64)
    c0 = corrector.forward(lam_c, y, p, Hc, kappa)[0]
    l0 = -(c0 * logp).sum(axis=1)
    w0 = wnet.weights(l0, lam_r)
    Lr = lambda lr: float(np.sum(mk * wnet.weights(l0, lr) * l0) / mk.sum())
    Lc = lambda lc: float(np.sum(mk * w0 * -(corrector.forward(lc, y, p, Hc, kappa)[0] * logp).sum(axis=1)) / mk.sum())
    nr = len(lam_r)
    fd_r = np.array([(Lr(lam_r + 1e-6 * e) - Lr(lam_r - 1e-6 * e)) / 2e-6 for e in np.eye(nr)])
    fd_c = np.array([(Lc(lam_c + 1e-6 * e) - Lc(lam_c - 1e-6 * e)) / 2e-6 for e in np.eye(len(lam_c))])
    assert np.allclose(got[:nr], fd_r, rtol=1e-6, atol=1e-9)
    assert np.allclose(got[nr:], fd_c, rtol=1e-6, atol=1e-9)
    assert np.linalg.norm(got[nr:]) > 1e-4                 # a dropped corrector term would pass a zero here


def test_dominant_label_prior_reduces_to_plain_reweighting():
    """kappa -> large makes c_i = onehot(y_i) to machine precision: base step, direction, eps, the lambda_r part of
    the hypergradient and the updated theta must equal the oracle without label correction, and the lambda_c part of
    the hypergradient must vanish."""
    model, x, y, xm, ym, th, lam_r, lam_c, C, Hc = _tiny()
    plain = SamaOracle(model, th, lam_r, base_lr=1e-2)
    corr = SamaOracle(model, th, np.concatenate([lam_r, lam_c]), base_lr=1e-2, corr_hidden=Hc, corr_kappa=200.0, n_classes=C)
    for _ in range(3):
        a = plain.base_step(x, y); b = corr.base_step(x, y)
        assert abs(a - b) < 1e-12 * (1 + abs(a))
    assert np.allclose(plain.g, corr.g, rtol=0, atol=1e-13)
    rp = plain.meta_step(x, y, xm, ym); rc = corr.meta_step(x, y, xm, ym)
    nr = len(lam_r)
    assert np.allclose(rp["v"], rc["v"], rtol=1e-12, atol=0) and abs(rp["eps"] - rc["eps"]) < 1e-12 * rp["eps"]
    assert np.allclose(rp["h"], rc["h"][:nr], rtol=1e-9, atol=1e-12 * np.linalg.norm(rp["h"]))
    assert np.linalg.norm(rc["h"][nr:]) < 1e-9 * np.linalg.norm(rp["h"])
    assert np.allclose(plain.theta, corr.theta, rtol=0, atol=1e-13)
    assert np.allclose(plain.lam, corr.lam[:nr], rtol=1e-9, atol=1e-12)


def test_label_correction_moves_both_lambda_groups_and_changes_the_base_gradient():
    model, x, y, xm, ym, th, lam_r, lam_c, C, Hc = _tiny()
    plain = SamaOracle(model, th, lam_r, base_lr=1e-2)
    corr = SamaOracle(model, th, np.concatenate([lam_r, lam_c]), base_lr=1e-2, corr_hidden=Hc, corr_kappa=1.0, n_classes=C)
    plain.base_step(x, y); corr.base_step(x, y)
    assert np.linalg.norm(plain.g - corr.g) > 1e-3 * np.linalg.norm(plain.g)      # soft labels really enter the gradient
    # the base gradient is the theta-gradient of sum coef_i CE(z_i, c_i) at fixed c and w: check by differences
    c = corr.targets(th, x, y)
    l = model.losses(th, x, c); w = wnet.weights(l, lam_r)
    S = lambda t: float(np.sum(w / len(y) * model.losses(t, x, c)))
    for k in (1, model.n // 3, model.n - 2):
        e = np.zeros(model.n); e[k] = 1e-6
        assert abs((S(th + e) - S(th - e)) / 2e-6 - corr.g[k]) < 1e-7 * (1 + abs(corr.g[k]))
    corr.base_step(x, y)
    # Eq. 5 for the whole lambda: the central difference of glam along v, taken on the untouched state
    r0 = corr.meta_grad(x, y, xm, ym)
    gp = corr.glam(corr.theta + r0["eps"] * r0["v"], x, y); gm = corr.glam(corr.theta - r0["eps"] * r0["v"], x, y)
    assert np.allclose(r0["h"], -(gp - gm) / (2 * r0["eps"]), rtol=1e-12, atol=0)
    lam_before = corr.lam.copy()
    r = corr.meta_step(x, y, xm, ym)
    nr = len(lam_r)
    assert np.array_equal(r["h"], r0["h"])
    assert np.all(np.isfinite(r["h"])) and np.linalg.norm(r["h"][:nr]) > 0 and np.linalg.norm(r["h"][nr:]) > 0
    moved = corr.lam != lam_before                             # dead ReLU units keep their parameters
    assert moved[:nr].sum() > nr // 2 and moved[nr:].sum() > (len(moved) - nr) // 2
