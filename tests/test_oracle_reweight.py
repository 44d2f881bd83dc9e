"""Pins for the assembled recipe (oracle/reweight.py + sama_core) on tiny problems: brute-force second
derivatives of the scalar base loss, the exact implicit-function hypergradient (Eq. 1-2) by re-solving the
base problem, the SGD invariant (Sec. 3.1-3.2) and the bookkeeping of the meta step (end of Sec. 3.2)."""
import numpy as np
import pytest
from datagen import CounterRNG, make_workload, init_theta, init_lambda
from oracle import models, wnet, optim, sama_core
from oracle.reweight import SamaOracle, SGD, ADAM


def _tiny(seed=41, B=24, Bm=10, F=5, C=3, H=4):
    r = CounterRNG(seed)
    model = models.MLP((F, C))
    x = r.normal(1, B * F).reshape(B, F); y = r.integers(2, B, C)
    xm = r.normal(3, Bm * F).reshape(Bm, F); ym = r.integers(4, Bm, C)
    th = 0.5 * r.normal(5, model.n)
    lam = np.concatenate([r.normal(6, H), np.abs(r.normal(7, H)), r.normal(8, H), [0.1]])
    return model, x, y, xm, ym, th, lam


def _after_steps(orc, x, y, k=3):
    for _ in range(k):
        orc.base_step(x, y)
    return orc


def test_glam_is_the_lambda_gradient_of_the_scalar_base_loss():
    model, x, y, xm, ym, th, lam = _tiny()
    mask = (np.arange(len(y)) % 5 != 0).astype(np.uint8)
    orc = SamaOracle(model, th, lam)
    got = orc.glam(th, x, y, mask)
    L = lambda l: wnet.base_loss(model.losses(th, x, y), l, mask)
    fd = np.array([(L(lam + 1e-6 * e) - L(lam - 1e-6 * e)) / 2e-6 for e in np.eye(len(lam))])
    assert np.allclose(got, fd, rtol=1e-6, atol=1e-9)


def test_fd_product_is_the_mixed_partial_times_v():
    """h = -(d2 L_base / dlambda dtheta) v up to O(eps^2): the mixed partial is taken by brute force as a
    four-point difference of the scalar L_base, and halving alpha divides the error by four."""
    model, x, y, xm, ym, th, lam = _tiny()
    orc = _after_steps(SamaOracle(model, th, lam, base_lr=1e-2, alpha=0.2), x, y)
    r = orc.meta_grad(x, y, xm, ym)
    v, theta = r["v"], orc.theta
    L = lambda t_, l_: wnet.base_loss(model.losses(t_, x, y), l_)
    tau, dl = 1e-4 / np.linalg.norm(v), 1e-4
    Mv = np.array([(L(theta + tau * v, lam + dl * e) - L(theta + tau * v, lam - dl * e)
                    - L(theta - tau * v, lam + dl * e) + L(theta - tau * v, lam - dl * e)) / (4 * tau * dl)
                   for e in np.eye(len(lam))])
    errs = []
    for alpha in (0.04, 0.02, 0.01):
        orc.alpha = alpha
        h = orc.meta_grad(x, y, xm, ym)["h"]
        errs.append(np.linalg.norm(h + Mv))
    assert errs[2] < 5e-3 * np.linalg.norm(Mv)
    assert 3.0 < errs[0] / errs[1] < 5.0 and 3.0 < errs[1] / errs[2] < 5.0


def test_exact_hypergradient_by_resolving_the_base_problem():
    """Direct per-sample weights sigma(lam_i) on a tiny L2-regularised logistic regression: theta*(lambda) by
    Newton with a brute-force Hessian; dL_meta/dlambda by differencing L_meta(theta*(lambda)).  Eq. 5's
    central difference with v = H^-1 dL_meta/dtheta reproduces it (Eq. 1-2), and with the identity in
    place of H^-1 (Eq. 3) it equals -M dL_meta/dtheta with M taken by brute force."""
    model, x, y, xm, ym, th, _ = _tiny(seed=43, B=12)
    B, n, rho = len(y), model.n, 0.05
    lam = CounterRNG(44).normal(1, B)
    sig = lambda z: 1 / (1 + np.exp(-z))
    grad = lambda t_, l_: model.loss_grad(t_, x, y, sig(l_) / B)[1] + rho * t_

    def hess(t_, l_):
        return np.array([(grad(t_ + 1e-5 * e, l_) - grad(t_ - 1e-5 * e, l_)) / 2e-5 for e in np.eye(n)])

    def solve(l_):
        t_ = th.copy()
        for _ in range(30):
            t_ = t_ - np.linalg.solve(hess(t_, l_), grad(t_, l_))
        assert np.linalg.norm(grad(t_, l_)) < 1e-10
        return t_
    ts = solve(lam)
    Lmeta = lambda t_: model.losses(t_, xm, ym).mean()
    exact = np.array([(Lmeta(solve(lam + 1e-4 * e)) - Lmeta(solve(lam - 1e-4 * e))) / 2e-4 for e in np.eye(B)])
    gmeta = model.loss_grad(ts, xm, ym, np.full(len(ym), 1 / len(ym)))[1]
    glam = lambda t_: sig(lam) * (1 - sig(lam)) * model.losses(t_, x, y) / B       # dL_base/dlam_i
    Hinv_g = np.linalg.solve(hess(ts, lam), gmeta)
    h_full, _, _ = sama_core.hypergradient(glam, ts, np.ones(n), Hinv_g, 1e-3)
    assert np.allclose(h_full, exact, rtol=2e-4, atol=1e-7)
    # identity approximation: -M g_meta, M_i = (1/B) sigma'(lam_i) dl_i/dtheta by brute force on each l_i
    M = np.array([[sig(lam[i]) * (1 - sig(lam[i])) / B *
                   (model.losses(ts + 1e-6 * e, x[i:i + 1], y[i:i + 1])[0] - model.losses(ts - 1e-6 * e, x[i:i + 1], y[i:i + 1])[0]) / 2e-6
                   for e in np.eye(n)] for i in range(B)])
    h_id, _, _ = sama_core.hypergradient(glam, ts, np.ones(n), gmeta, 1e-3)
    assert np.allclose(h_id, -M @ gmeta, rtol=1e-5, atol=1e-9)
    assert h_id @ exact > 0                                           # a descent direction for the true objective


def test_sgd_invariant():
    """With an SGD base solver the adaptation is the scalar step size: theta+-, eps*||v|| are independent of
    gamma and h(gamma) = gamma h(1); SAMA-NA under Adam is the same thing with gamma = 1."""
    model, x, y, xm, ym, th, lam = _tiny()
    outs = {}
    for tag, kw in (("g1", dict(base_opt=SGD, base_lr=1.0)), ("g2", dict(base_opt=SGD, base_lr=0.037)),
                    ("na", dict(base_opt=ADAM, base_lr=0.5, adapt_mode=optim.ADAPT_NONE))):
        o = SamaOracle(model, th, lam, alpha=0.3, **kw)
        o.base_step(x, y)
        o.theta = th + 0.01                      # identical evaluation point for all three
        outs[tag] = (o, o.meta_grad(x, y, xm, ym))
    r1, r2, rna = outs["g1"][1], outs["g2"][1], outs["na"][1]
    assert np.allclose(r2["v"], 0.037 * r1["v"], rtol=1e-14)
    assert np.allclose(r2["eps"] * 0.037, r1["eps"], rtol=1e-13)
    assert np.allclose(r2["glam_p"], r1["glam_p"], rtol=1e-11) and np.allclose(r2["glam_m"], r1["glam_m"], rtol=1e-11)
    assert np.allclose(r2["h"], 0.037 * r1["h"], rtol=1e-9, atol=1e-15)
    assert np.allclose(rna["h"], r1["h"], rtol=1e-12) and np.allclose(rna["v"], r1["g_meta"], rtol=0, atol=0)


def test_sgd_momentum_in_the_assembled_recipe():
    """Heavy-ball momentum in the SGD base solver: the oracle's trajectory equals steps written out by hand from its own
    kept gradients (velocity in `m`), the adaptation stays the scalar step size (v = gamma g_meta), and mu = 0 is plain
    SGD bit for bit."""
    model, x, y, xm, ym, th, lam = _tiny()
    o = SamaOracle(model, th, lam, base_opt=SGD, base_lr=0.05, momentum=0.8, alpha=0.3)
    p = SamaOracle(model, th, lam, base_opt=SGD, base_lr=0.05, alpha=0.3)
    z = SamaOracle(model, th, lam, base_opt=SGD, base_lr=0.05, momentum=0.0, alpha=0.3)
    b, t_hand = np.zeros_like(th), np.array(th, dtype=np.float64)
    for k in range(3):
        o.base_step(x, y); p.base_step(x, y); z.base_step(x, y)
        b = 0.8 * b + o.g
        t_hand = t_hand - 0.05 * b
        assert np.allclose(o.theta, t_hand, rtol=0, atol=1e-15) and np.allclose(o.m, b, rtol=0, atol=1e-15)
    assert np.array_equal(z.theta, p.theta) and not np.allclose(o.theta, p.theta)
    r = o.meta_grad(x, y, xm, ym)
    assert np.array_equal(r["v"], 0.05 * r["g_meta"])
    with np.testing.assert_raises(ValueError):
        SamaOracle(model, th, lam, base_opt=ADAM, momentum=0.5)


def test_direction_is_ill_conditioned_in_the_first_steps_of_a_run():
    """Conditioning of Eq. 4 free-running from zero moments, from the oracle alone: on the small encoder of the GPU
    tests, a relative noise of 1e-3 (of each tensor's rms) on the three base gradients moves the perturbation vector v
    by more than half its norm at Adam's eps_A = 1e-8, because a handful of entries with sqrt(v') near eps_A carry most
    of ||v||^2; at eps_A = 1e-5 the same noise moves v by under a tenth.  The hypergradient, which only sees v through
    the train batch, moves far less.  This is why the free-running GPU test asserts v and eps at eps_A = 1e-5 only."""
    from datagen import make_workload, init_theta, init_lambda
    from oracle import models
    wl = make_workload(3, n_train=40, n_meta=12, dims=(2, 192, 3, 320, 128, 600, 3), batch=5, meta_batch=3)
    rel = lambda a, b: np.linalg.norm(a - b) / np.linalg.norm(b)
    change = {}
    for aeps in (1e-8, 1e-5):
        runs = []
        for noise in (0.0, 1e-3):
            orc = SamaOracle(models.make_model(wl.kind, wl.dims), init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3,
                             meta_lr=wl.meta_lr, alpha=wl.alpha, adam_eps=aeps)
            rng = np.random.default_rng(0)
            clean = orc.model.loss_grad

            def noisy(theta, x, y, coef):
                l, g = clean(theta, x, y, coef)
                for name, (off, shape) in orc.model.slices.items():
                    sl = slice(off, off + int(np.prod(shape)))
                    g[sl] += (g[sl] != 0) * noise * np.sqrt(np.mean(g[sl] ** 2)) * rng.standard_normal(g[sl].size)
                return l, g
            for k in range(3):
                it = wl.train_batch(k)
                orc.model.loss_grad = noisy if noise else clean
                orc.base_step(wl.x_train[it], wl.y_train[it])
            orc.model.loss_grad = clean
            im = wl.meta_batch_idx(2)
            runs.append(orc.meta_grad(wl.x_train[it], wl.y_train[it], wl.x_meta[im], wl.y_meta[im]))
        change[aeps] = (rel(runs[1]["v"], runs[0]["v"]), rel(runs[1]["h"], runs[0]["h"]))
        if aeps == 1e-8:
            v = runs[0]["v"]
            top10 = np.sort(v * v)[-10:].sum() / np.sum(v * v)
    assert top10 > 0.5                                            # ten entries of 685,507 carry most of ||v||^2
    assert change[1e-8][0] > 0.5 and change[1e-5][0] < 0.1, change
    assert change[1e-8][1] < 0.1 * change[1e-8][0]                # h is far less sensitive than v


def test_meta_step_bookkeeping():
    model, x, y, xm, ym, th, lam = _tiny()
    orc = _after_steps(SamaOracle(model, th, lam, base_lr=1e-2, meta_lr=1e-3, alpha=0.7), x, y, k=4)
    th0, m0, v0, t0, lam0 = orc.theta.copy(), orc.m.copy(), orc.v.copy(), orc.t, orc.lam.copy()
    r0 = orc.meta_grad(x, y, xm, ym)
    assert np.array_equal(orc.theta, th0) and np.array_equal(orc.lam, lam0) and orc.meta_t == 0     # pure
    r = orc.meta_step(x, y, xm, ym)
    assert np.array_equal(r["h"], r0["h"])
    assert abs(np.linalg.norm(r["eps"] * r["v"]) - 0.7) < 1e-13
    assert np.array_equal(orc.theta, th0 - r["eps"] * r["v"])
    assert abs(np.linalg.norm(orc.theta - th0) - 0.7) < 1e-12
    assert np.array_equal(orc.m, m0) and np.array_equal(orc.v, v0) and orc.t == t0
    # first Adam step on lambda moves every entry by lr * h/(|h| + eps_A sqrt-corrected) ~ lr sign(h)
    step = lam0 - orc.lam
    nzh = np.abs(r["h"]) > 1e-6
    assert np.allclose(step[nzh], 1e-3 * np.sign(r["h"][nzh]), rtol=1e-2)
    assert orc.meta_t == 1 and orc.status == 0
    # the direction is the adapted direct gradient
    D = optim.adam_adaptation(orc.g, orc.m, orc.v, orc.t, 1e-2, 0.9, 0.999, 1e-8)
    assert np.array_equal(r["v"], D * r["g_meta"])


def test_first_step_direction_is_degenerate_and_skipped():
    """After a single Adam step from zero moments u = lr sign(g) and du/dg = 0 (up to rounding noise): the
    oracle must either skip (v = 0) or return a finite result; a forced zero direction raises the flag."""
    model, x, y, xm, ym, th, lam = _tiny()
    orc = SamaOracle(model, th, lam)
    orc.base_step(x, y)
    orc.g[...] = 0; orc.m[...] = 0; orc.v[...] = 0
    th0, lam0 = orc.theta.copy(), orc.lam.copy()
    r = orc.meta_step(x, y, xm, ym)
    assert r["eps"] == 0.0 and np.all(r["h"] == 0) and orc.status == 1
    assert np.array_equal(orc.theta, th0) and np.array_equal(orc.lam, lam0) and orc.meta_t == 0
    with pytest.raises(RuntimeError):
        SamaOracle(model, th, lam).meta_grad(x, y, xm, ym)


def test_masked_samples_are_bit_irrelevant():
    model, x, y, xm, ym, th, lam = _tiny()
    mask = np.ones(len(y), dtype=np.uint8); mask[[1, 7, 8]] = 0
    mm = np.ones(len(ym), dtype=np.uint8); mm[2] = 0
    res = []
    for junk in (False, True):
        x2, y2, xm2, ym2 = x.copy(), y.copy(), xm.copy(), ym.copy()
        if junk:
            x2[[1, 7, 8]] = 99.0; y2[[1, 7, 8]] = 0; xm2[2] = -50.0; ym2[2] = (ym2[2] + 1) % 3
        o = SamaOracle(model, th, lam, base_lr=1e-2)
        for _ in range(3):
            o.base_step(x2, y2, mask)
        res.append((o.meta_step(x2, y2, xm2, ym2, mask, mm), o))
    assert np.array_equal(res[0][0]["h"], res[1][0]["h"]) and np.array_equal(res[0][1].theta, res[1][1].theta)
    assert np.array_equal(res[0][1].lam, res[1][1].lam)


def test_workload1_trajectory_runs():
    """Workload 1 end to end, 20 meta steps at unroll 1: finite, the nudge has norm alpha, lambda moves."""
    wl = make_workload(1)
    model = models.make_model(wl.kind, wl.dims)
    o = SamaOracle(model, init_theta(wl), init_lambda(wl), base_lr=wl.base_lr, meta_lr=wl.meta_lr, alpha=wl.alpha)
    lam0 = o.lam.copy()
    o.base_step(wl.x_train, wl.y_train)           # a step of history so that the adaptation is non-zero
    for s in range(wl.steps):
        o.base_step(wl.x_train, wl.y_train)
        r = o.meta_step(wl.x_train, wl.y_train, wl.x_meta, wl.y_meta)
        assert np.all(np.isfinite(r["h"])) and abs(r["eps"] * np.linalg.norm(r["v"]) - wl.alpha) < 1e-12
    assert o.meta_t == wl.steps and np.linalg.norm(o.lam - lam0) > 0


def test_weight_decay_is_an_l2_term_in_front_of_the_solver():
    """wdecay of the base optimizer (App. B tables): with SGD one step is theta - lr (g + wd theta) by hand; with Adam
    the first step moves every element by lr against the sign of g + wd theta; and the kept gradient, the one the
    adaptation differentiates the update with respect to, includes the term."""
    model, x, y, xm, ym, th, lam = _tiny()
    wd, lr = 0.3, 0.05
    l = model.losses(th, x, y)
    w = wnet.weights(l, lam)
    _, g = model.loss_grad(th, x, y, w / len(y))
    o = SamaOracle(model, th, lam, base_opt=SGD, base_lr=lr, weight_decay=wd)
    o.base_step(x, y)
    assert np.allclose(o.theta, th - lr * (g + wd * th), rtol=0, atol=1e-15)
    assert np.allclose(o.g, g + wd * th, rtol=0, atol=1e-15)
    big = 50.0                                    # the decay term decides every sign
    a = SamaOracle(model, th, lam, base_lr=lr, adam_eps=0.0, weight_decay=big)
    a.base_step(x, y)
    assert np.allclose(a.theta, th - lr * np.sign(g + big * th), rtol=1e-12, atol=1e-15)
    # no decay: the same oracle as before
    z = SamaOracle(model, th, lam, base_lr=lr); z0 = SamaOracle(model, th, lam, base_lr=lr, weight_decay=0.0)
    z.base_step(x, y); z0.base_step(x, y)
    assert np.array_equal(z.theta, z0.theta)
    # the adaptation is the derivative of the update with respect to the gradient it was given
    b = SamaOracle(model, th, lam, base_lr=lr, weight_decay=wd)
    for _ in range(3):
        b.base_step(x, y)
    D = b.adaptation()
    m_prev = (b.m - (1 - b.beta1) * b.g) / b.beta1
    v_prev = (b.v - (1 - b.beta2) * b.g ** 2) / b.beta2
    d = 1e-7 * (1 + np.abs(b.g))
    up = lambda gg: th * 0 - optim.adam_update(th * 0, m_prev, v_prev, gg, b.t, lr, b.beta1, b.beta2, 0.0)[0]
    fd = (up(b.g + d) - up(b.g - d)) / (2 * d)
    keep = np.abs(b.v) > 1e-12
    assert np.allclose(D[keep], fd[keep], rtol=2e-4, atol=1e-10)


def test_scheduled_rate_and_the_adaptation_use_the_rate_of_the_step():
    """lr_scheduler of the base optimizer (App. B tables): base_lr may change between base steps.  Each step moves by
    the rate in force when it ran (SGD by hand), and gamma in the adaptation is the rate of the step it differentiates,
    also after the schedule has moved on; a constant schedule is the unscheduled oracle bit for bit."""
    model, x, y, xm, ym, th, lam = _tiny()
    rates = [0.05, 0.02, 0.08]
    o = SamaOracle(model, th, lam, base_opt=SGD, base_lr=rates[0])
    cur = th.copy()
    for lr in rates:
        o.base_lr = lr
        l = model.losses(cur, x, y)
        _, g = model.loss_grad(cur, x, y, wnet.weights(l, lam) / len(y))
        o.base_step(x, y)
        cur = cur - lr * g
        assert np.allclose(o.theta, cur, rtol=0, atol=1e-15)
    o.base_lr = 123.0                                 # the scheduler's next value: not the last step's
    assert np.array_equal(o.adaptation(), np.full_like(th, rates[-1]))
    a = SamaOracle(model, th, lam, base_lr=rates[0])
    for lr in rates:
        a.base_lr = lr
        a.base_step(x, y)
    a.base_lr = 123.0
    m_prev = (a.m - (1 - a.beta1) * a.g) / a.beta1
    v_prev = (a.v - (1 - a.beta2) * a.g ** 2) / a.beta2
    d = 1e-7 * (1 + np.abs(a.g))
    up = lambda gg: -optim.adam_update(th * 0, m_prev, v_prev, gg, a.t, rates[-1], a.beta1, a.beta2, 0.0)[0]
    fd = (up(a.g + d) - up(a.g - d)) / (2 * d)
    keep = np.abs(a.v) > 1e-12
    assert np.allclose(a.adaptation()[keep], fd[keep], rtol=2e-4, atol=1e-10)
    c0 = SamaOracle(model, th, lam, base_lr=0.03); c1 = SamaOracle(model, th, lam, base_lr=0.5)
    for _ in range(3):
        c1.base_lr = 0.03
        c0.base_step(x, y); c1.base_step(x, y)
    r0 = c0.meta_step(x, y, xm, ym); r1 = c1.meta_step(x, y, xm, ym)
    assert np.array_equal(r0["h"], r1["h"]) and np.array_equal(c0.theta, c1.theta)


def test_evaluate_is_the_forward_half_of_the_base_step():
    """evaluate() against the base step's own return value (L_base = sum_i mask_i w_i l_i / B_eff) and against the
    model's plain cross-entropy; it changes nothing."""
    model, x, y, xm, ym, th, lam = _tiny()
    o = SamaOracle(model, th, lam, base_lr=0.05)
    o.base_step(x, y)
    th1 = o.theta.copy()
    z, l, w = o.evaluate(x, y)
    assert np.array_equal(o.theta, th1) and o.t == 1
    mask = np.ones(len(y)); mask[1] = 0
    ref = SamaOracle(model, th1, lam, base_lr=0.05)
    assert abs(ref.base_step(x, y, mask) - np.sum(mask * w * l) / mask.sum()) < 1e-14
    assert np.allclose(l, model.losses(th1, x, y), rtol=0, atol=1e-15)
    assert np.allclose(l, np.log(np.exp(z).sum(axis=1)) - z[np.arange(len(y)), y], rtol=1e-12)
    assert np.all((w > 0) & (w < 1))


def test_frozen_trajectories():
    """Short runs of every oracle variant against tests/golden/oracle_trajectories.json (written by
    tests/golden/make_oracle_golden.py from oracle/ alone): a change to the oracle's arithmetic has to show up here.
    Tolerances leave room for another BLAS summation order, amplified by the difference of Eq. 5, and nothing more."""
    import importlib.util
    import json
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_oracle_golden", os.path.join(here, "golden", "make_oracle_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    want = json.load(open(os.path.join(here, "golden", "oracle_trajectories.json")))
    got = mod.build()
    assert set(got) == set(want)
    for name in want:
        assert len(got[name]) == len(want[name])
        for g, w in zip(got[name], want[name]):
            for key in ("loss", "theta_norm", "lam_norm"):
                assert abs(g[key] - w[key]) <= 1e-10 * abs(w[key]), (name, key)
            for key in ("eps", "v_norm", "h_norm"):
                assert abs(g[key] - w[key]) <= 1e-6 * abs(w[key]), (name, key, g[key], w[key])
            assert np.allclose(g["h_head"], w["h_head"], rtol=0, atol=1e-6 * w["h_norm"]), name
