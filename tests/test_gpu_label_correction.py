"""GPU parity of label correction (Sec. 4.1: the base loss of a noisy sample is the weighted cross-entropy against
the corrected soft label; lambda = [weight net | corrector]): the HIP path through the C ABI against the float64
oracle, teacher-forced.  fp32 workloads to 1e-4, the small bf16 encoder to the kernel-arithmetic bar 1e-2."""
import numpy as np
import pytest
from datagen import make_workload, init_theta, init_lambda, init_lambda_corr
from harness import rel_l2, make_pair, dev_batch, push_state, pull

pytestmark = pytest.mark.gpu


def _batches(wl, step):
    it, im = wl.train_batch(step), wl.meta_batch_idx(step)
    return (wl.x_train[it], wl.y_train[it]), (wl.x_meta[im], wl.y_meta[im])


def _lam0(wl, Hc):
    return np.concatenate([init_lambda(wl), init_lambda_corr(wl, Hc)])


@pytest.mark.parametrize("cfg,Hc,kappa", [(1, 8, 1.5), (2, 37, 4.0), (2, 128, 0.0)])
def test_label_correction_parity_fp32(cfg, Hc, kappa):
    wl = make_workload(cfg)
    orc, gpu = make_pair(wl, init_theta(wl), _lam0(wl, Hc), corr_hidden=Hc, corr_kappa=kappa)
    nr = 3 * wl.H + 1
    assert gpu.nl == orc.lam.size
    rng = np.random.default_rng(cfg)
    for s in range(3):
        (x, y), _ = _batches(wl, s)
        mask = (rng.random(len(y)) < 0.8).astype(np.uint8) if s == 1 else None
        push_state(orc, gpu)
        l_want = orc.model.losses(orc.theta, x, orc.targets(orc.theta, x, y))
        lo = orc.base_step(x, y, mask)
        gpu.base_step(dev_batch(gpu, x, y, mask))
        assert np.max(np.abs(pull(gpu, "LOSSES")[:len(y)] - l_want)) < 1e-5 * max(1.0, np.max(l_want))
        assert rel_l2(pull(gpu, "G"), orc.g) < 1e-4
        assert rel_l2(pull(gpu, "THETA"), orc.theta) < 1e-6
        assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 1e-5 * abs(lo)
    for s in range(3, 6):
        (x, y), (xm, ym) = _batches(wl, s)
        mask = (rng.random(len(y)) < 0.8).astype(np.uint8) if s == 4 else None
        orc.base_step(x, y, mask)
        push_state(orc, gpu)
        tb, mb = dev_batch(gpu, x, y, mask), dev_batch(gpu, xm, ym)
        r = orc.meta_step(x, y, xm, ym, mask)
        gpu.meta_step(tb, mb)
        gp, gm, h = pull(gpu, "GLAM_PLUS"), pull(gpu, "GLAM_MINUS"), pull(gpu, "HYPERGRAD")
        e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), v=rel_l2(pull(gpu, "VDIR"), r["v"]),
                 glam_r=rel_l2(gp[:nr], r["glam_p"][:nr]), glam_c=rel_l2(gp[nr:], r["glam_p"][nr:]),
                 glam_m_c=rel_l2(gm[nr:], r["glam_m"][nr:]), h_r=rel_l2(h[:nr], r["h"][:nr]), h_c=rel_l2(h[nr:], r["h"][nr:]),
                 theta=rel_l2(pull(gpu, "THETA"), orc.theta), lam=rel_l2(pull(gpu, "LAMBDA"), orc.lam))
        print(f"workload {cfg} Hc {Hc} step {s}: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
        assert np.linalg.norm(r["h"][nr:]) > 0
        assert max(e["gmeta"], e["v"], e["glam_r"], e["glam_c"], e["glam_m_c"], e["theta"], e["lam"]) < 1e-4, e
        # the hypergradient is a difference of two fp32 forward passes eps apart (Eq. 5)
        assert e["h_r"] < 1e-4 and e["h_c"] < 1e-4, e
        assert int(pull(gpu, "COUNTERS")[2]) == 0
    gpu.close()


def test_dominant_prior_reduces_to_reweighting_on_the_gpu():
    """kappa large: the corrected label is the given one, so theta-side results equal those of plain reweighting
    and the corrector's hypergradient vanishes."""
    wl = make_workload(2)
    Hc = 16
    th0 = init_theta(wl)
    orc_c, gpu_c = make_pair(wl, th0, _lam0(wl, Hc), corr_hidden=Hc, corr_kappa=200.0)
    orc_r, gpu_r = make_pair(wl, th0, init_lambda(wl))
    nr = 3 * wl.H + 1
    for s in range(3):
        (x, y), _ = _batches(wl, s)
        gpu_c.base_step(dev_batch(gpu_c, x, y)); gpu_r.base_step(dev_batch(gpu_r, x, y))
    (x, y), (xm, ym) = _batches(wl, 3)
    gpu_c.meta_step(dev_batch(gpu_c, x, y), dev_batch(gpu_c, xm, ym))
    gpu_r.meta_step(dev_batch(gpu_r, x, y), dev_batch(gpu_r, xm, ym))
    assert rel_l2(pull(gpu_c, "THETA"), pull(gpu_r, "THETA")) < 1e-6
    hc, hr = pull(gpu_c, "HYPERGRAD"), pull(gpu_r, "HYPERGRAD")
    assert rel_l2(hc[:nr], hr) < 1e-5
    assert np.linalg.norm(hc[nr:]) < 1e-12 * max(np.linalg.norm(hr), 1e-30) or np.all(hc[nr:] == 0)
    gpu_c.close(); gpu_r.close()


def test_label_correction_small_encoder_bf16():
    small = dict(dims=(2, 192, 3, 320, 128, 600, 3), batch=5, meta_batch=3)
    wl = make_workload(3, n_train=40, n_meta=12, **small)
    Hc = 24
    orc, gpu = make_pair(wl, init_theta(wl, 0.02), _lam0(wl, Hc), base_lr=1e-3, corr_hidden=Hc, corr_kappa=2.0)
    nr = 3 * wl.H + 1
    for s in range(3):
        (x, y), _ = _batches(wl, s)
        orc.base_step(x, y)
    for s in range(3, 5):
        (x, y), (xm, ym) = _batches(wl, s)
        push_state(orc, gpu)
        orc.base_step(x, y)
        gpu.base_step(dev_batch(gpu, x, y))
        assert rel_l2(pull(gpu, "G"), orc.g) < 1e-2
        push_state(orc, gpu)
        r = orc.meta_step(x, y, xm, ym)
        gpu.meta_step(dev_batch(gpu, x, y), dev_batch(gpu, xm, ym))
        gp, h = pull(gpu, "GLAM_PLUS"), pull(gpu, "HYPERGRAD")
        e = dict(glam_r=rel_l2(gp[:nr], r["glam_p"][:nr]), glam_c=rel_l2(gp[nr:], r["glam_p"][nr:]),
                 h_r=rel_l2(h[:nr], r["h"][:nr]), h_c=rel_l2(h[nr:], r["h"][nr:]),
                 theta=rel_l2(pull(gpu, "THETA"), orc.theta), lam=rel_l2(pull(gpu, "LAMBDA"), orc.lam))
        print(f"small encoder Hc {Hc} step {s}: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
        assert e["glam_r"] < 1e-2 and e["glam_c"] < 1e-2, e
        assert e["h_r"] < 2e-2 and e["h_c"] < 2e-2, e
        assert e["theta"] < 2e-2 and e["lam"] < 2e-2
    gpu.close()
