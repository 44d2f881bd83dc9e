"""GPU parity, fp32 workloads (1: logistic regression, 2: MLP 784-256-256-10): the HIP path through the C ABI
against the float64 oracle on the same seeded inputs.  Bar: relative L2 <= 1e-4 on the hypergradient and the
updated theta / lambda; integer artefacts bit-exact."""
import numpy as np
import pytest
from datagen import make_workload, init_theta, init_lambda, CounterRNG
from harness import rel_l2, make_pair, dev_batch, push_state, pull

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _batches(wl, step):
    it, im = wl.train_batch(step), wl.meta_batch_idx(step)
    return (wl.x_train[it], wl.y_train[it]), (wl.x_meta[im], wl.y_meta[im])


@pytest.mark.parametrize("cfg", [1, 2])
def test_base_step_parity(cfg):
    wl = make_workload(cfg)
    orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl))
    for s in range(3):
        (x, y), _ = _batches(wl, s)
        push_state(orc, gpu)
        lo = orc.base_step(x, y)
        gpu.base_step(dev_batch(gpu, x, y))
        assert rel_l2(pull(gpu, "G"), orc.g) < TOL
        assert rel_l2(pull(gpu, "THETA"), orc.theta) < 1e-6
        assert rel_l2(pull(gpu, "M"), orc.m) < TOL and rel_l2(pull(gpu, "V"), orc.v) < TOL
        assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 1e-5 * abs(lo)
        assert int(pull(gpu, "COUNTERS")[0]) == orc.t
    gpu.close()


@pytest.mark.parametrize("cfg", [1, 2])
def test_meta_step_parity_teacher_forced(cfg):
    wl = make_workload(cfg)
    orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl))
    for s in range(3):                      # history, so that the adaptation is not the degenerate first step
        (x, y), _ = _batches(wl, s)
        orc.base_step(x, y)
    for s in range(3, 6):
        (x, y), (xm, ym) = _batches(wl, s)
        orc.base_step(x, y)
        push_state(orc, gpu)
        tb, mb = dev_batch(gpu, x, y), dev_batch(gpu, xm, ym)
        # meta_grad is pure
        gpu.meta_grad(tb, mb)
        assert np.array_equal(pull(gpu, "THETA"), orc.theta.astype(np.float32))
        assert np.array_equal(pull(gpu, "LAMBDA"), orc.lam.astype(np.float32))
        h_pure = pull(gpu, "HYPERGRAD")
        r = orc.meta_step(x, y, xm, ym)
        gpu.meta_step(tb, mb)
        assert rel_l2(pull(gpu, "GMETA"), r["g_meta"]) < TOL
        assert rel_l2(pull(gpu, "VDIR"), r["v"]) < TOL
        sc = pull(gpu, "SCALARS")
        assert abs(sc[0] - r["eps"]) < TOL * r["eps"]
        h = pull(gpu, "HYPERGRAD")
        assert np.array_equal(h, h_pure)
        assert rel_l2(h, r["h"]) < TOL, rel_l2(h, r["h"])
        assert rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
        assert rel_l2(pull(gpu, "LAMBDA"), orc.lam) < TOL
        cnt = pull(gpu, "COUNTERS")
        assert int(cnt[1]) == orc.meta_t and int(cnt[2]) == 0
    gpu.close()


def test_free_running_trajectory_workload1():
    """20 meta steps at unroll 1, no teacher forcing (plus one warm-up base step of history)."""
    wl = make_workload(1)
    orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl))
    tb, mb = dev_batch(gpu, wl.x_train, wl.y_train), dev_batch(gpu, wl.x_meta, wl.y_meta)
    orc.base_step(wl.x_train, wl.y_train); gpu.base_step(tb)
    lam0 = orc.lam.copy()
    for s in range(wl.steps):
        orc.base_step(wl.x_train, wl.y_train); gpu.base_step(tb)
        r = orc.meta_step(wl.x_train, wl.y_train, wl.x_meta, wl.y_meta); gpu.meta_step(tb, mb)
        assert rel_l2(pull(gpu, "HYPERGRAD"), r["h"]) < 1e-3, (s, rel_l2(pull(gpu, "HYPERGRAD"), r["h"]))
    assert rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
    assert rel_l2(pull(gpu, "LAMBDA") - lam0, orc.lam - lam0) < 1e-3
    assert int(pull(gpu, "COUNTERS")[1]) == wl.steps
    gpu.close()


def test_masking_is_bit_exact_and_call_order():
    import paper_2310_05674_amd as pkg
    wl = make_workload(1)
    th0, lam0 = init_theta(wl), init_lambda(wl)
    mask = np.ones(wl.n_train, dtype=np.uint8); mask[::7] = 0
    mmask = np.ones(wl.n_meta, dtype=np.uint8); mmask[3] = 0
    outs = []
    for junk in (False, True):
        x, y, xm, ym = wl.x_train.copy(), wl.y_train.copy(), wl.x_meta.copy(), wl.y_meta.copy()
        if junk:
            x[::7] = 1e3; y[::7] = 1 - y[::7]; xm[3] = -77.0
        orc, gpu = make_pair(wl, th0, lam0)
        tb, mb = dev_batch(gpu, x, y, mask), dev_batch(gpu, xm, ym, mmask)
        with pytest.raises(pkg.SamaError) as e:
            gpu.meta_step(tb, mb)
        assert e.value.code == 2
        for _ in range(3):
            gpu.base_step(tb)
            if not junk:
                orc.base_step(x, y, mask)
        gpu.meta_step(tb, mb)
        outs.append((pull(gpu, "HYPERGRAD"), pull(gpu, "THETA"), pull(gpu, "LAMBDA")))
        if not junk:
            r = orc.meta_step(x, y, xm, ym, mask, mmask)
            assert rel_l2(outs[0][0], r["h"]) < TOL and rel_l2(outs[0][1], orc.theta) < TOL
        gpu.close()
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)


def test_degenerate_direction_is_skipped():
    """Zero history (g = m = v = 0) gives v = 0: hypergradient 0, lambda and theta untouched, status raised."""
    wl = make_workload(1)
    orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl))
    tb, mb = dev_batch(gpu, wl.x_train, wl.y_train), dev_batch(gpu, wl.x_meta, wl.y_meta)
    gpu.base_step(tb)
    z = np.zeros(gpu.n, dtype=np.float32)
    for nm in ("G", "M", "V"):
        gpu.set_state(nm, z)
    th, lam = pull(gpu, "THETA"), pull(gpu, "LAMBDA")
    gpu.meta_step(tb, mb)
    assert np.all(pull(gpu, "HYPERGRAD") == 0) and np.array_equal(pull(gpu, "THETA"), th) and np.array_equal(pull(gpu, "LAMBDA"), lam)
    cnt = pull(gpu, "COUNTERS")
    assert int(cnt[1]) == 0 and int(cnt[2]) == 1
    gpu.close()


def test_non_finite_hypergradient_is_skipped():
    """A lambda-gradient that is not finite although ||v|| is (here: a NaN planted in the weight net's output bias after
    the base steps, which the direct-gradient pass never reads): hypergradient 0, lambda, theta and the meta moments
    untouched, status raised, the meta step count not advanced -- as the oracle does."""
    wl = make_workload(1)
    orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl))
    tb, mb = dev_batch(gpu, wl.x_train, wl.y_train), dev_batch(gpu, wl.x_meta, wl.y_meta)
    for _ in range(3):
        orc.base_step(wl.x_train, wl.y_train); gpu.base_step(tb)
    lam = pull(gpu, "LAMBDA").copy(); lam[-1] = np.nan
    gpu.set_state("LAMBDA", lam); orc.lam = lam.astype(np.float64)
    th, mm = pull(gpu, "THETA"), pull(gpu, "META_M")
    r = orc.meta_step(wl.x_train, wl.y_train, wl.x_meta, wl.y_meta)
    assert orc.status == 1 and orc.meta_t == 0 and r["eps"] > 0 and not np.all(np.isfinite(r["h"]))
    gpu.meta_step(tb, mb)
    assert np.all(pull(gpu, "HYPERGRAD") == 0) and np.array_equal(pull(gpu, "THETA"), th)
    assert np.array_equal(pull(gpu, "LAMBDA"), lam, equal_nan=True) and np.array_equal(pull(gpu, "META_M"), mm)
    cnt = pull(gpu, "COUNTERS")
    assert int(cnt[1]) == 0 and int(cnt[2]) == 1 and float(pull(gpu, "SCALARS")[0]) > 0
    gpu.close()


@pytest.mark.parametrize("variant", ["sgd", "sgd_momentum", "sama_na"])
def test_sgd_and_no_adaptation_variants(variant):
    wl = make_workload(1)
    kw = {"sgd": dict(base_opt="sgd", base_lr=0.05), "sgd_momentum": dict(base_opt="sgd", base_lr=0.05, momentum=0.9),
          "sama_na": dict(adapt_mode=1)}[variant]
    orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl), **kw)
    tb, mb = dev_batch(gpu, wl.x_train, wl.y_train), dev_batch(gpu, wl.x_meta, wl.y_meta)
    for _ in range(3 if variant == "sgd_momentum" else 2):
        orc.base_step(wl.x_train, wl.y_train); gpu.base_step(tb)
    if variant == "sgd_momentum":      # free-running velocity (the M state) and weights after three steps
        assert rel_l2(pull(gpu, "M"), orc.m) < TOL and rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
        assert rel_l2(orc.m, orc.g) > 0.5
    r = orc.meta_step(wl.x_train, wl.y_train, wl.x_meta, wl.y_meta); gpu.meta_step(tb, mb)
    assert rel_l2(pull(gpu, "HYPERGRAD"), r["h"]) < TOL and rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
    gpu.close()


@pytest.mark.parametrize("base_opt", ["adam", "sgd"])
def test_weight_decay_enters_the_kept_gradient(base_opt):
    """L2 term in front of the solver (the wdecay column of App. B): the G state, and through it the adaptation of
    Eq. 4, carry g + weight_decay * theta.  The decay is large enough that dropping it anywhere breaks the bars."""
    wl = make_workload(1)
    kw = dict(base_opt=base_opt, weight_decay=0.5)
    if base_opt == "sgd":
        kw["base_lr"] = 0.05
    orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl), **kw)
    ref, _unused = make_pair(wl, init_theta(wl), init_lambda(wl), **dict(kw, weight_decay=0.0))
    _unused.close()
    tb, mb = dev_batch(gpu, wl.x_train, wl.y_train), dev_batch(gpu, wl.x_meta, wl.y_meta)
    for _ in range(3):
        orc.base_step(wl.x_train, wl.y_train); gpu.base_step(tb)
        ref.base_step(wl.x_train, wl.y_train)
        assert rel_l2(pull(gpu, "G"), orc.g) < TOL and rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
    assert rel_l2(ref.g, orc.g) > 0.1          # the term matters at this size
    r = orc.meta_step(wl.x_train, wl.y_train, wl.x_meta, wl.y_meta); gpu.meta_step(tb, mb)
    assert rel_l2(pull(gpu, "VDIR"), r["v"]) < TOL
    assert rel_l2(pull(gpu, "HYPERGRAD"), r["h"]) < TOL and rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
    gpu.close()


@pytest.mark.parametrize("base_opt", ["adam", "sgd"])
def test_scheduled_rates(base_opt):
    """lr_scheduler of App. B through sama_set_lr: every base step runs at the rate set before it, the meta update at the
    meta rate set before it, and the adaptation keeps the rate of the base step it differentiates even when the next
    value has been set already.  Rates differ by up to 4x, so a stale or early rate breaks the bars."""
    import paper_2310_05674_amd as pkg
    wl = make_workload(1)
    scale = 5.0 if base_opt == "sgd" else 1.0
    base = [wl.base_lr * scale * f for f in (1.0, 0.25, 0.6, 0.4, 1.0)]
    meta = [wl.meta_lr * f for f in (1.0, 2.0, 0.5, 1.0, 1.0)]
    orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl), base_opt=base_opt, base_lr=base[0])
    tb, mb = dev_batch(gpu, wl.x_train, wl.y_train), dev_batch(gpu, wl.x_meta, wl.y_meta)
    with pytest.raises(pkg.SamaError):
        gpu.set_lr(0.0, 1e-3)
    with pytest.raises(pkg.SamaError):
        gpu.set_lr(1e-3, float("nan"))
    for _ in range(2):                                  # history: the adaptation of the very first Adam step is zero
        orc.base_step(wl.x_train, wl.y_train); gpu.base_step(tb)
    lam0 = orc.lam.copy()
    for k in range(4):
        orc.base_lr, orc.meta_lr = base[k], meta[k]
        gpu.set_lr(base[k], meta[k])
        orc.base_step(wl.x_train, wl.y_train); gpu.base_step(tb)
        assert rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
        orc.base_lr = base[k + 1]                       # the scheduler has moved on before the meta step
        gpu.set_lr(base[k + 1], meta[k])
        r = orc.meta_step(wl.x_train, wl.y_train, wl.x_meta, wl.y_meta); gpu.meta_step(tb, mb)
        assert rel_l2(pull(gpu, "VDIR"), r["v"]) < 1e-3, (k, rel_l2(pull(gpu, "VDIR"), r["v"]))
        assert rel_l2(pull(gpu, "HYPERGRAD"), r["h"]) < 1e-3      # free running, as in the trajectory test
        assert rel_l2(pull(gpu, "LAMBDA") - lam0, orc.lam - lam0) < 1e-3 and rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
    gpu.close()


@pytest.mark.parametrize("corr", [0, 6])
def test_eval_returns_logits_losses_and_weights(corr):
    """sama_eval against the oracle's forward half of the base step, with and without label correction; it leaves every
    state vector alone, also the losses of the last step."""
    import torch
    from datagen import init_lambda_corr
    wl = make_workload(2)
    lam0 = np.concatenate([init_lambda(wl), init_lambda_corr(wl, corr)]) if corr else init_lambda(wl)
    kw = dict(corr_hidden=corr, corr_kappa=1.5) if corr else {}
    orc, gpu = make_pair(wl, init_theta(wl), lam0, **kw)
    (x, y), (xm, ym) = _batches(wl, 0)
    tb = dev_batch(gpu, x, y)
    for _ in range(2):
        orc.base_step(x, y); gpu.base_step(tb)
    before = {k: pull(gpu, k).copy() for k in ("THETA", "LAMBDA", "M", "V", "G", "LOSSES", "SCALARS", "COUNTERS")}
    n, C = len(ym), wl.dims[-1]
    zo = torch.full((n, C), -7.0, device=gpu.dev); lo = torch.full((n,), -7.0, device=gpu.dev); wo = torch.full((n,), -7.0, device=gpu.dev)
    gpu.eval(dev_batch(gpu, xm, ym), zo, lo, wo)
    z, l, w = orc.evaluate(xm, ym)
    assert rel_l2(zo.cpu().numpy(), z) < TOL and rel_l2(lo.cpu().numpy(), l) < TOL and rel_l2(wo.cpu().numpy(), w) < TOL
    for k, v in before.items():
        assert np.array_equal(pull(gpu, k), v), k
    # any subset of the outputs
    w2 = torch.zeros(n, device=gpu.dev)
    gpu.eval(dev_batch(gpu, xm, ym), weights_out=w2)
    assert torch.equal(w2, wo)
    gpu.eval(dev_batch(gpu, xm, ym))
    gpu.close()


def test_ragged_shapes():
    """Widths and batch sizes that are not multiples of any tile (67-33-5, batches 37 / 19)."""
    from datagen.workloads import Workload
    r = CounterRNG(99)
    wl = Workload(cfg=0, kind="mlp", dims=(67, 33, 5), bf16=False, H=9, batch=37, meta_batch=19, base_lr=1e-2,
                  meta_lr=1e-3, alpha=0.5, noise=0.0, n_train=37, n_meta=19, steps=1)
    x = r.normal(1, 37 * 67).reshape(37, 67).astype(np.float32); y = r.integers(2, 37, 5).astype(np.int32)
    xm = r.normal(3, 19 * 67).reshape(19, 67).astype(np.float32); ym = r.integers(4, 19, 5).astype(np.int32)
    th0 = (0.2 * r.normal(5, 67 * 33 + 33 * 5 + 33 + 5)).astype(np.float32).astype(np.float64)
    lam0 = r.normal(6, 28).astype(np.float32).astype(np.float64)
    orc, gpu = make_pair(wl, th0, lam0)
    tb, mb = dev_batch(gpu, x, y), dev_batch(gpu, xm, ym)
    for _ in range(3):
        orc.base_step(x, y); gpu.base_step(tb)
    assert rel_l2(pull(gpu, "G"), orc.g) < TOL
    rr = orc.meta_step(x, y, xm, ym); gpu.meta_step(tb, mb)
    assert rel_l2(pull(gpu, "HYPERGRAD"), rr["h"]) < TOL and rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
    gpu.close()


def test_batch_size_limits():
    """One sample, the largest batch the library takes (2048), and the sizes it must refuse."""
    import torch
    import paper_2310_05674_amd as pkg
    from datagen.workloads import Workload
    r = CounterRNG(123)
    F, C, B, Bm = 32, 3, 2048, 2048
    wl = Workload(cfg=0, kind="mlp", dims=(F, 16, C), bf16=False, H=8, batch=B, meta_batch=Bm, base_lr=1e-2, meta_lr=1e-3,
                  alpha=0.5, noise=0.0, n_train=B, n_meta=Bm, steps=1)
    x = r.normal(1, B * F).reshape(B, F).astype(np.float32); y = r.integers(2, B, C).astype(np.int32)
    xm = r.normal(3, Bm * F).reshape(Bm, F).astype(np.float32); ym = r.integers(4, Bm, C).astype(np.int32)
    th0 = (0.3 * r.normal(5, F * 16 + 16 * C + 16 + C)).astype(np.float32).astype(np.float64)
    lam0 = r.normal(6, 25).astype(np.float32).astype(np.float64)
    for n, nm in ((B, Bm), (1, 1), (1, Bm)):
        orc, gpu = make_pair(wl, th0, lam0)
        tb, mb = dev_batch(gpu, x[:n], y[:n]), dev_batch(gpu, xm[:nm], ym[:nm])
        for _ in range(3):
            orc.base_step(x[:n], y[:n]); gpu.base_step(tb)
        assert rel_l2(pull(gpu, "G"), orc.g) < TOL, (n, nm)
        rr = orc.meta_step(x[:n], y[:n], xm[:nm], ym[:nm]); gpu.meta_step(tb, mb)
        # Eq. 5 divides a difference of two fp32 passes by 2 eps: with one sample nothing averages the rounding of the two
        # losses, and 1e-7 of relative rounding on a 1e-3 relative difference is the 1e-4 bar itself
        assert rel_l2(pull(gpu, "HYPERGRAD"), rr["h"]) < (TOL if n > 1 else 1e-3), (n, nm, rel_l2(pull(gpu, "HYPERGRAD"), rr["h"]))
        assert rel_l2(pull(gpu, "THETA"), orc.theta) < TOL and rel_l2(pull(gpu, "LAMBDA"), orc.lam) < TOL
        gpu.close()
    # refused: an empty batch, a batch above max_batch, a context above the library's limit
    small = Workload(cfg=0, kind="mlp", dims=(F, 16, C), bf16=False, H=8, batch=8, meta_batch=8, base_lr=1e-2, meta_lr=1e-3,
                     alpha=0.5, noise=0.0, n_train=8, n_meta=8, steps=1)
    _, gpu = make_pair(small, th0, lam0)
    xt, yt = torch.as_tensor(x[:9], device=gpu.dev), torch.as_tensor(y[:9], device=gpu.dev)
    before = pull(gpu, "THETA").copy()
    for bad in (gpu.batch(xt, yt), gpu.batch(xt[:0].contiguous(), yt[:0].contiguous())):
        with pytest.raises(pkg.SamaError) as e:
            gpu.base_step(bad)
        assert e.value.code == 1
    assert np.array_equal(pull(gpu, "THETA"), before) and int(pull(gpu, "COUNTERS")[0]) == 0      # nothing was enqueued
    gpu.close()
    with pytest.raises(pkg.SamaError):
        pkg.Sama(pkg.SamaConfig.make("mlp", (F, 16, C), H=8, max_batch=2049, max_meta_batch=8), th0, lam0)


def test_fully_masked_batch_changes_nothing():
    """B_eff = 0: every coefficient is zero, the gradient is exactly zero and the first Adam step leaves theta alone."""
    wl = make_workload(1)
    th0, lam0 = init_theta(wl), init_lambda(wl)
    _, gpu = make_pair(wl, th0, lam0)
    gpu.base_step(dev_batch(gpu, wl.x_train, wl.y_train, np.zeros(wl.n_train, dtype=np.uint8)))
    assert np.all(pull(gpu, "G") == 0.0) and float(pull(gpu, "SCALARS")[2]) == 0.0
    assert np.array_equal(pull(gpu, "THETA"), th0.astype(np.float32))
    assert np.all(np.isfinite(pull(gpu, "M"))) and np.all(np.isfinite(pull(gpu, "V")))
    gpu.close()


@pytest.mark.parametrize("cfg,steps", [(1, 300), (2, 60)])
def test_reweighting_learns_to_down_weight_flipped_labels(cfg, steps):
    """What the method is for (Sec. 4.1): run freely on the noisy synthetic data, the learned weights w(l; lambda) end up
    lower on the samples whose labels were flipped than on the clean ones, and the base learner fits the clean labels
    better than at the start.  (Functional check of the whole loop on the GPU; the oracle only evaluates the outcome.)"""
    import torch
    from oracle import models, wnet
    wl = make_workload(cfg)
    _, gpu = make_pair(wl, init_theta(wl), init_lambda(wl))
    model = models.make_model(wl.kind, wl.dims)
    x64 = wl.x_train.astype(np.float64)

    def outcome():
        th, lam = pull(gpu, "THETA").astype(np.float64), pull(gpu, "LAMBDA").astype(np.float64)
        w = wnet.weights(model.losses(th, x64, wl.y_train), lam)
        acc = float((np.argmax(model.logits(th, x64), axis=1) == wl.y_train_clean).mean())
        return float(w[~wl.flipped].mean()), float(w[wl.flipped].mean()), acc

    wc0, wf0, acc0 = outcome()
    for k in range(steps):
        (x, y), (xm, ym) = _batches(wl, k)
        tb, mb = dev_batch(gpu, x, y), dev_batch(gpu, xm, ym)
        gpu.base_step(tb)
        if k >= 2:      # Eq. 4 vanishes identically after the very first Adam step (rounding noise, normalised to a step of
            gpu.meta_step(tb, mb)   # norm alpha, would be all the direction holds): give the moments some history first
    wc, wf, acc = outcome()
    print(f"workload {cfg}: mean weight clean / flipped {wc0:.4f} / {wf0:.4f} -> {wc:.4f} / {wf:.4f}; accuracy on the clean labels {acc0:.3f} -> {acc:.3f}")
    # workload 2 is separable: after ~90 iterations the clean data are fitted exactly and the meta gradient, with it the
    # direction v, is rounding noise that the step size alpha / ||v|| blows up to norm alpha; the run stops before that
    assert int(pull(gpu, "COUNTERS")[1]) >= steps // 2
    assert wc > 1.2 * wf and wc - wf > 10 * abs(wc0 - wf0)
    assert acc > acc0 + 0.25
    gpu.close()
