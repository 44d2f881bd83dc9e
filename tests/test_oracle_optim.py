"""Pins for oracle/optim.py: the Adam adaptation (App. C) against a central difference of the
Adam update itself, closed-form special cases, and the SGD reduction (Sec. 3.2)."""
import numpy as np
from datagen import CounterRNG
from oracle import optim


def _u(g, m, v, t, lr, b1, b2, eps):
    """u(g) = theta - theta' for one Adam step, through the oracle's update routine."""
    th = np.zeros_like(g)
    th2, _, _ = optim.adam_update(th, m, v, g, t, lr, b1, b2, eps)
    return th - th2


def _cases(seed, n=400):
    r = CounterRNG(seed)
    g = r.normal(1, n)
    m = 0.3 * r.normal(2, n)
    v = (0.5 * r.normal(3, n)) ** 2 + 1e-3
    return g, m, v


def test_adam_update_textbook_scalar():
    # two steps of Adam on a scalar by hand (Kingma & Ba Alg. 1)
    th, m, v = 1.0, 0.0, 0.0
    lr, b1, b2, eps = 0.1, 0.9, 0.999, 1e-8
    for t, g in ((1, 0.5), (2, -0.25)):
        m = b1 * m + (1 - b1) * g
        v = b2 * v + (1 - b2) * g * g
        th = th - lr * (m / (1 - b1**t)) / (np.sqrt(v / (1 - b2**t)) + eps)
    A = (np.array([1.0]), np.array([0.0]), np.array([0.0]))
    for t, g in ((1, 0.5), (2, -0.25)):
        A = optim.adam_update(A[0], A[1], A[2], np.array([g]), t, lr, b1, b2, eps)
    assert abs(A[0][0] - th) < 1e-15
    # first step from zero moments moves by lr * sign(g)
    th1, _, _ = optim.adam_update(np.zeros(3), np.zeros(3), np.zeros(3), np.array([2.0, -3.0, 0.1]), 1, 0.01, 0.9, 0.999, 0.0)
    assert np.allclose(th1, [-0.01, 0.01, -0.01], atol=1e-15)


def test_adaptation_matches_central_difference_eps0():
    for seed, t in ((1, 1), (2, 3), (3, 50), (4, 5000)):
        g, m, v = _cases(seed)
        lr, b1, b2 = 1e-3, 0.9, 0.999
        m2 = b1 * m + (1 - b1) * g
        v2 = b2 * v + (1 - b2) * g * g
        D = optim.adam_adaptation(g, m2, v2, t, lr, b1, b2, 0.0)
        h = 1e-5
        fd = (_u(g + h, m, v, t, lr, b1, b2, 0.0) - _u(g - h, m, v, t, lr, b1, b2, 0.0)) / (2 * h)
        assert np.max(np.abs(D - fd)) <= 1e-7 * np.max(np.abs(fd))


def test_adaptation_eps_term():
    g, m, v = _cases(5)
    lr, b1, b2, eps, t = 1e-3, 0.9, 0.999, 1e-3, 7         # large eps_A so that the term is visible
    m2 = b1 * m + (1 - b1) * g
    v2 = b2 * v + (1 - b2) * g * g
    h = 1e-5
    fd = (_u(g + h, m, v, t, lr, b1, b2, eps) - _u(g - h, m, v, t, lr, b1, b2, eps)) / (2 * h)
    D_exact = optim.adam_adaptation(g, m2, v2, t, lr, b1, b2, eps, keep_eps_term=True)
    assert np.max(np.abs(D_exact - fd)) <= 1e-7 * np.max(np.abs(fd))
    # the default form drops exactly (1-b1) eps s / (s (c2 s + eps)^2) and nothing else
    D = optim.adam_adaptation(g, m2, v2, t, lr, b1, b2, eps)
    c1, c2, s = 1 / (1 - b1**t), 1 / np.sqrt(1 - b2**t), np.sqrt(v2)
    assert np.allclose(D_exact - D, lr * c1 * (1 - b1) * eps / (c2 * s + eps) ** 2, rtol=1e-8, atol=0)
    # and at the default eps_A = 1e-8 the two agree to O(eps_A / s)
    De = optim.adam_adaptation(g, m2, v2, t, lr, b1, b2, 1e-8, keep_eps_term=True)
    Dd = optim.adam_adaptation(g, m2, v2, t, lr, b1, b2, 1e-8)
    assert np.max(np.abs(De - Dd)) <= 1e-6 * np.max(np.abs(De))


def test_adaptation_special_cases():
    g = np.array([0.7, -1.3, 2.0])
    lr, b1, b2 = 0.01, 0.9, 0.999
    # first step from zero moments: u = lr sign(g), so du/dg = 0
    D = optim.adam_adaptation(g, (1 - b1) * g, (1 - b2) * g * g, 1, lr, b1, b2, 0.0)
    assert np.max(np.abs(D)) < 1e-15
    # no history at all (s = 0): defined as 0, not inf/nan
    D0 = optim.adam_adaptation(np.zeros(4), np.zeros(4), np.zeros(4), 3, lr, b1, b2, 1e-8)
    assert np.all(D0 == 0.0)
    # beta2 -> 1 with a frozen second moment: u = lr c1 m'/(c2 sqrt(v)) is linear in g with slope lr c1 (1-b1)/(c2 sqrt v)
    v = np.array([0.5, 2.0, 4.0]); m = np.array([0.1, 0.2, -0.3]); t = 4
    b2x = 1.0 - 1e-12
    D2 = optim.adam_adaptation(g, b1 * m + (1 - b1) * g, b2x * v + (1 - b2x) * g * g, t, lr, b1, b2x, 0.0)
    c1, c2 = 1 / (1 - b1**t), 1 / np.sqrt(1 - b2x**t)
    assert np.allclose(D2, lr * c1 * (1 - b1) / (c2 * np.sqrt(v)), rtol=1e-6)


def test_sgd_reduction():
    g = np.arange(5.0)
    assert np.all(optim.sgd_adaptation(g, 0.3) == 0.3)
    assert np.allclose(optim.sgd_update(np.ones(5), g, 0.1), 1.0 - 0.1 * g)


def test_sgd_momentum_by_hand_and_its_adaptation():
    """Heavy-ball SGD (reading of "SGD" in the tables of App. B): two steps on a scalar written out by hand; the update's
    derivative in the gradient it was given is the learning rate (central difference), as sgd_adaptation says; zero
    momentum is plain SGD bit for bit."""
    lr, mu = 0.1, 0.9
    th, b = 1.0, 0.0
    b = mu * b + 0.5; th = th - lr * b            # step 1, g = 0.5: b = 0.5, theta = 0.95
    b = mu * b - 0.25; th = th - lr * b           # step 2, g = -0.25: b = 0.2, theta = 0.93
    assert abs(b - 0.2) < 1e-15 and abs(th - 0.93) < 1e-15
    T, B = np.array([1.0]), np.array([0.0])
    for g in (0.5, -0.25):
        T, B = optim.sgd_momentum_update(T, B, np.array([g]), lr, mu)
    assert abs(T[0] - 0.93) < 1e-15 and abs(B[0] - 0.2) < 1e-15
    r = CounterRNG(11)
    g, buf, th0 = r.normal(1, 50), r.normal(2, 50), r.normal(3, 50)
    u = lambda gg: th0 - optim.sgd_momentum_update(th0, buf, gg, lr, mu)[0]
    fd = (u(g + 1e-4) - u(g - 1e-4)) / 2e-4
    assert np.allclose(fd, optim.sgd_adaptation(g, lr), rtol=1e-9)
    t2, b2 = optim.sgd_momentum_update(th0, buf, g, lr, 0.0)
    assert np.array_equal(t2, optim.sgd_update(th0, g, lr)) and np.array_equal(b2, g)


def test_adaptation_peaks_where_the_second_moment_meets_eps():
    """Closed form of a special case of App. C: an entry whose last gradient is zero (g = 0, so m' = beta1 m, v' = beta2 v)
    has D(s) = lr c1 c2 (1 - beta1) s / (c2 s + eps)^2 with s = sqrt(v'), which peaks at c2 s = eps with the value
    lr c1 (1 - beta1) / (4 eps) -- for eps = 1e-8 seven orders of magnitude above D of an entry with |g| ~ 1.  Around
    that peak D follows the entry's tiny gradient history with unit relative sensitivity, which is why the perturbation
    vector of Eq. 4 is ill-conditioned in the first steps of a run (many entries with almost no history)."""
    lr, b1, b2, eps, t = 1e-3, 0.9, 0.999, 1e-8, 3
    c1, c2 = 1 / (1 - b1**t), 1 / np.sqrt(1 - b2**t)
    s = np.logspace(-12, -2, 2001) * 1.0
    D = optim.adam_adaptation(np.zeros_like(s), np.full_like(s, 0.3), s * s, t, lr, b1, b2, eps)
    assert np.allclose(D, lr * c1 * c2 * (1 - b1) * s / (c2 * s + eps) ** 2, rtol=1e-12)
    k = int(np.argmax(D))
    assert abs(c2 * s[k] / eps - 1.0) < 2e-2 and abs(D[k] / (lr * c1 * (1 - b1) / (4 * eps)) - 1.0) < 1e-3
    # an entry with a steady gradient of size 1: D is of the order of lr
    g1 = np.array([1.0])
    D1 = optim.adam_adaptation(g1, (1 - b1**t) * g1, (1 - b2**t) * g1 * g1, t, lr, b1, b2, eps)
    assert D[k] / abs(D1[0]) > 1e6
