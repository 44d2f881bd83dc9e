"""GPU parity, bf16 encoder workloads: the HIP path through the C ABI against the float64 oracle on the same
seeded inputs, from the oracle's unrounded state (teacher-forced) and free-running.  Bar: relative L2 <= 2e-2 on the
hypergradient and the updated theta / lambda (bf16 GEMM operands, fp32 accumulation and state).  Nothing in this file
rounds the oracle's state to what the kernels can hold, except the one test of the mixed-precision switch
(fast_base_pass = 1), which says so."""
import numpy as np
import pytest
from datagen import make_workload, init_theta, init_lambda, round_to_bf16, seq_lengths
from oracle.models import with_lengths
from harness import rel_l2, make_pair, dev_batch, push_state, pull

pytestmark = pytest.mark.gpu
TOL = 2e-2

SMALL = dict(dims=(2, 192, 3, 320, 128, 600, 3), batch=5, meta_batch=3)      # ragged N tiles, odd batch sizes
KTOL = 1e-2     # bar of the small-shape tests on single gradients: ~10 bf16 roundings (2^-9) of GEMM inputs per layer


def _well_measured(orc, tau=0.1):
    """Entries whose kept base gradient lies above the noise floor of a bf16 pass: |g_i| >= tau * rms of g over the
    entry's tensor (from the oracle alone).  A pass with bf16 GEMM operands carries an error of the order of 1e-3 of a
    tensor's rms on EVERY entry of its gradient, so the relative error of an entry grows as the entry shrinks -- and the
    adaptation of Eq. 4 is largest (by orders of magnitude) exactly on the entries with the smallest gradient history,
    which therefore hold most of ||v||^2 while being the worst measured.  With the GPU's own g, m', v' in Eq. 4 the
    perturbation vector is compared entry by entry on the well-measured entries; its norm enters through eps."""
    mask = np.zeros(orc.g.size, dtype=bool)
    for name, (off, shape) in orc.model.slices.items():
        sl = slice(off, off + int(np.prod(shape)))
        mask[sl] = np.abs(orc.g[sl]) >= tau * np.sqrt(np.mean(orc.g[sl] ** 2))
    return mask


def _gemm_block(orc):
    return sum(int(np.prod(sh)) for nm, (o, sh) in orc.model.slices.items() if nm.split(".")[-1] in ("Wqkv", "Wo", "W1", "W2"))


def _batches(wl, step):
    it, im = wl.train_batch(step), wl.meta_batch_idx(step)
    return (wl.x_train[it], wl.y_train[it]), (wl.x_meta[im], wl.y_meta[im])


def _group_errors(orc, got, want):
    out = {}
    for name, (off, shape) in orc.model.slices.items():
        sl = slice(off, off + int(np.prod(shape)))
        out[name] = rel_l2(got[sl], want[sl])
    return out


@pytest.mark.parametrize("scale", [0.02, 0.08])
def test_small_encoder_base_step(scale):
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    orc, gpu = make_pair(wl, init_theta(wl, scale), init_lambda(wl), base_lr=1e-3)
    for s in range(2):
        (x, y), _ = _batches(wl, s)
        push_state(orc, gpu)
        th_before = orc.theta.copy()
        l_before = orc.model.losses(orc.theta, x, y)
        lo = orc.base_step(x, y)
        gpu.base_step(dev_batch(gpu, x, y))
        losses = pull(gpu, "LOSSES")[:len(y)]
        # diagnostic: how much of the difference is the bf16 rounding of the GEMM weights themselves
        ng = sum(int(np.prod(sh)) for nm, (o, sh) in orc.model.slices.items() if nm.split(".")[-1] in ("Wqkv", "Wo", "W1", "W2"))
        th_r = th_before.copy(); th_r[:ng] = round_to_bf16(th_r[:ng])
        l_r = orc.model.losses(th_r, x, y)
        print(f"  losses: max|l|={np.max(l_before):.3f} gpu-oracle {np.max(np.abs(losses - l_before)):.2e} "
              f"gpu-oracle(bf16 weights) {np.max(np.abs(losses - l_r)):.2e}")
        assert np.max(np.abs(losses - l_before)) < 2e-2 * max(1.0, np.max(l_before)), np.max(np.abs(losses - l_before))
        g = pull(gpu, "G")
        errs = _group_errors(orc, g, orc.g)
        worst = max(errs, key=errs.get)
        print(f"scale {scale} step {s}: rel-L2 g {rel_l2(g, orc.g):.3e}; worst group {worst} {errs[worst]:.3e}")
        assert rel_l2(g, orc.g) < KTOL
        assert all(e < 2e-2 for e in errs.values()), errs
        assert rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
        assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 2e-2 * abs(lo)
    gpu.close()


@pytest.mark.parametrize("scale", [0.02, 0.08])
def test_small_encoder_meta_step(scale):
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    orc, gpu = make_pair(wl, init_theta(wl, scale), init_lambda(wl), base_lr=1e-3)
    for s in range(3):
        (x, y), _ = _batches(wl, s)
        orc.base_step(x, y)
    for s in range(3, 5):
        (x, y), (xm, ym) = _batches(wl, s)
        orc.base_step(x, y)
        push_state(orc, gpu)
        tb, mb = dev_batch(gpu, x, y), dev_batch(gpu, xm, ym)
        r = orc.meta_step(x, y, xm, ym)
        gpu.meta_step(tb, mb)
        h = pull(gpu, "HYPERGRAD")
        e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), v=rel_l2(pull(gpu, "VDIR"), r["v"]),
                 eps=abs(pull(gpu, "SCALARS")[0] - r["eps"]) / r["eps"], h=rel_l2(h, r["h"]),
                 glam_p=rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"]), theta=rel_l2(pull(gpu, "THETA"), orc.theta),
                 lam=rel_l2(pull(gpu, "LAMBDA"), orc.lam))
        print(f"scale {scale} step {s}: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
        assert e["gmeta"] < KTOL and e["glam_p"] < KTOL and e["eps"] < KTOL and e["v"] < TOL
        # at scale 0.08 / lr 1e-3 the map v -> h is ill-conditioned (a 1e-2 change of v moves h by 4e-2 in exact
        # arithmetic as well), so there h is printed, not asserted: its inputs (g_meta, v, eps, g_lambda^+) carry the bars
        if scale == 0.02:
            assert e["h"] < TOL, e
        assert e["theta"] < TOL and e["lam"] < TOL
        assert int(pull(gpu, "COUNTERS")[2]) == 0
    gpu.close()


def test_meta_grad_is_pure_and_matches_meta_step():
    """sama_meta_grad leaves theta, lambda and the moments untouched and returns the hypergradient that sama_meta_step
    then applies.  The two take different routes through the elementwise chain (separate low halves and nudge against
    the old bf16 copy / one fused pass against the new one), so the two hypergradients agree to rounding of the low
    halves, not bit for bit; the applied step must still land on the oracle's theta."""
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    for s in range(4):
        (x, y), _ = _batches(wl, s)
        orc.base_step(x, y)
    (x, y), (xm, ym) = _batches(wl, 4)
    push_state(orc, gpu)
    tb, mb = dev_batch(gpu, x, y), dev_batch(gpu, xm, ym)
    before = {k: pull(gpu, k).copy() for k in ("THETA", "LAMBDA", "M", "V", "META_M", "META_V")}
    gpu.meta_grad(tb, mb)
    for k, v in before.items():
        assert np.array_equal(pull(gpu, k), v), k
    h_pure = pull(gpu, "HYPERGRAD").copy()
    gpu.meta_grad(tb, mb)
    assert np.array_equal(pull(gpu, "HYPERGRAD"), h_pure)          # and is repeatable bit for bit
    r = orc.meta_step(x, y, xm, ym)
    gpu.meta_step(tb, mb)
    h = pull(gpu, "HYPERGRAD")
    assert rel_l2(h_pure, r["h"]) < TOL and rel_l2(h, r["h"]) < TOL
    assert rel_l2(h, h_pure) < 5e-3, rel_l2(h, h_pure)
    assert rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
    th = pull(gpu, "THETA")
    # the nudge itself, fused block and tail alike: theta_old - eps v with the GPU's own eps and v, one fp32 rounding
    want = before["THETA"].astype(np.float64) - float(pull(gpu, "SCALARS")[0]) * pull(gpu, "VDIR").astype(np.float64)
    assert np.max(np.abs(th - want)) <= 2.0 ** -23 * np.max(np.abs(want))
    for name, (off, shape) in orc.model.slices.items():           # every tensor moved, GEMM block and tail alike
        sl = slice(off, off + int(np.prod(shape)))
        assert not np.array_equal(th[sl], before["THETA"][sl]), name
    gpu.close()


# ------------------------------------------------------------------------------------------ full workloads 3-5
_RUNS = {}


def _run_workload(cfg, n_train, n_meta):
    """Real shapes and hyper-parameters of workload `cfg`, nothing rounded anywhere; one run per workload serves the
    tests below (the oracle takes a minute on workload 5).
      a. base step 0 from the initial theta on both sides: the gradient of one pass;
      b. one more oracle base step (history for the adaptation), its state pushed, one meta step (teacher-forced);
      c. the oracle's state after that meta step -- a general point: fp32 master weights off the bf16 grid after two
         Adam steps and a nudge -- pushed once, then ONE WHOLE ITERATION on each side from its own state: base step
         (gradient compared), then the meta step with the GPU's own g, m', v' in the adaptation of Eq. 4."""
    if cfg in _RUNS:
        return _RUNS[cfg]
    import time
    t0 = time.time()
    wl = make_workload(cfg, n_train=n_train, n_meta=n_meta)
    orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl))
    out = {}
    (x, y), _ = _batches(wl, 0)
    orc.base_step(x, y)
    gpu.base_step(dev_batch(gpu, x, y))
    g = pull(gpu, "G")
    errs = _group_errors(orc, g, orc.g)
    worst = max(errs, key=errs.get)
    out["a"] = dict(g=rel_l2(g, orc.g), worst=errs[worst], theta=rel_l2(pull(gpu, "THETA"), orc.theta))
    print(f"cfg {cfg} a: base step 0 rel-L2 g {out['a']['g']:.3e}, worst group {worst} {errs[worst]:.1e}  [{time.time() - t0:.0f}s]", flush=True)

    def meta_errors(r):
        e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), v=rel_l2(pull(gpu, "VDIR"), r["v"]),
                 eps=abs(pull(gpu, "SCALARS")[0] - r["eps"]) / r["eps"], h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
                 theta=rel_l2(pull(gpu, "THETA"), orc.theta), lam=rel_l2(pull(gpu, "LAMBDA"), orc.lam))
        e["fd_signal"] = np.linalg.norm(r["glam_p"] - r["glam_m"]) / np.linalg.norm(r["glam_p"])
        e["glam_p"] = rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"])
        e["status"] = int(pull(gpu, "COUNTERS")[2])
        return e

    (x, y), (xm, ym) = _batches(wl, 1)
    orc.base_step(x, y)
    push_state(orc, gpu)
    r = orc.meta_step(x, y, xm, ym)
    gpu.meta_step(dev_batch(gpu, x, y), dev_batch(gpu, xm, ym))
    out["b"] = meta_errors(r)
    print(f"cfg {cfg} b: " + " ".join(f"{k}={v:.2e}" for k, v in out["b"].items()) + f"  [{time.time() - t0:.0f}s]", flush=True)

    push_state(orc, gpu)
    ng = _gemm_block(orc)
    out["off_grid"] = float(np.mean(round_to_bf16(orc.theta[:ng]) != orc.theta[:ng]))
    (x, y), (xm, ym) = _batches(wl, 2)
    tb, mb = dev_batch(gpu, x, y), dev_batch(gpu, xm, ym)
    th_before = orc.theta.copy()
    orc.base_step(x, y)
    gpu.base_step(tb)
    g = pull(gpu, "G")
    errs = _group_errors(orc, g, orc.g)
    worst = max(errs, key=errs.get)
    out["c_base"] = dict(g=rel_l2(g, orc.g), worst=errs[worst], theta=rel_l2(pull(gpu, "THETA"), orc.theta),
                         step=rel_l2(pull(gpu, "THETA").astype(np.float64) - th_before, orc.theta - th_before),
                         m=rel_l2(pull(gpu, "M"), orc.m), v=rel_l2(pull(gpu, "V"), orc.v))
    print(f"cfg {cfg} c: off-grid weights {out['off_grid']:.2f}; base step rel-L2 g {out['c_base']['g']:.3e} worst group {worst} "
          f"{errs[worst]:.1e} update {out['c_base']['step']:.2e}  [{time.time() - t0:.0f}s]", flush=True)
    well = _well_measured(orc)             # from the oracle's kept gradient, before the meta step moves anything
    r = orc.meta_step(x, y, xm, ym)
    gpu.meta_step(tb, mb)
    out["c_meta"] = meta_errors(r)
    out["c_meta"]["v_well"] = rel_l2(pull(gpu, "VDIR")[well], r["v"][well])
    out["c_meta"]["well_frac"] = float(well.mean())
    out["c_meta"]["well_share"] = float(np.sum(r["v"][well] ** 2) / np.sum(r["v"] ** 2))
    print(f"cfg {cfg} c: " + " ".join(f"{k}={v:.2e}" for k, v in out["c_meta"].items()) + f"  [{time.time() - t0:.0f}s]", flush=True)
    gpu.close()
    _RUNS[cfg] = out
    return out


SIZES = {3: (128, 64), 4: (96, 64), 5: (48, 32)}


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_workload_parity(cfg):
    """Steps a and b of _run_workload: the gradient of the first base step, and a teacher-forced meta step."""
    o = _run_workload(cfg, *SIZES[cfg])
    assert o["a"]["g"] < KTOL and o["a"]["worst"] < 3e-2 and o["a"]["theta"] < TOL, o["a"]
    e = o["b"]
    assert e["h"] < TOL and e["theta"] < TOL and e["lam"] < TOL and e["eps"] < TOL and e["gmeta"] < TOL and e["v"] < TOL, e
    assert e["status"] == 0


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_workload_iteration_from_general_state(cfg):
    """Step c of _run_workload: one whole iteration (sama_base_step, then sama_meta_step with the GPU's own gradient and
    moments) from master weights that are NOT bf16-representable, against the oracle doing the same two calls."""
    o = _run_workload(cfg, *SIZES[cfg])
    assert o["off_grid"] > 0.5, o["off_grid"]            # the state really is a general one
    b = o["c_base"]
    assert b["g"] < TOL and b["worst"] < 5e-2 and b["theta"] < TOL and b["step"] < TOL and b["m"] < TOL and b["v"] < TOL, b
    e = o["c_meta"]
    assert e["h"] < TOL and e["theta"] < TOL and e["lam"] < TOL and e["eps"] < TOL and e["gmeta"] < TOL, e
    # v with the GPU's own g, m', v' in Eq. 4: asserted on the entries whose gradient is above the pass's noise floor (see
    # _well_measured: 40-60 % of the entries, which hold only a few per cent of ||v||^2); over all entries it is printed
    # (1e-2 ... 1e-1 depending on the data seed) and enters the assertions through eps, h and theta
    assert e["well_frac"] > 0.3 and e["v_well"] < TOL, e
    assert e["status"] == 0


def test_mixed_precision_switch_sees_the_rounded_weights():
    """fast_base_pass = 1 is ordinary mixed precision: the base step differentiates at bf16(theta).  From a
    bf16-representable theta it agrees with the default (split) pass and with the oracle; from a general state its
    gradient equals the oracle's gradient AT THE ROUNDED WEIGHTS (the only place in this file where oracle weights are
    rounded, to state what the switch computes), while the default pass follows the oracle at theta itself."""
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    th0 = init_theta(wl, 0.02)
    orc, fast = make_pair(wl, th0, init_lambda(wl), base_lr=1e-3, fast_base_pass=1)
    _, split = make_pair(wl, th0, init_lambda(wl), base_lr=1e-3)
    for s in range(3):
        (x, y), _ = _batches(wl, s)
        orc.base_step(x, y)
    (x, y), _ = _batches(wl, 3)
    push_state(orc, fast); push_state(orc, split)
    ng = _gemm_block(orc)
    th_r = orc.theta.copy(); th_r[:ng] = round_to_bf16(th_r[:ng])
    target = orc.targets(th_r, x, y)
    l = orc.model.losses(th_r, x, target)
    from oracle import wnet
    coef = wnet.weights(l, orc.lam) / len(y)
    _, g_rounded = orc.model.loss_grad(th_r, x, target, coef)
    orc.base_step(x, y)
    tb = dev_batch(fast, x, y)
    fast.base_step(tb); split.base_step(dev_batch(split, x, y))
    e_fast_r, e_fast, e_split = rel_l2(pull(fast, "G"), g_rounded), rel_l2(pull(fast, "G"), orc.g), rel_l2(pull(split, "G"), orc.g)
    print(f"fast vs oracle at bf16(theta) {e_fast_r:.2e}; fast vs oracle at theta {e_fast:.2e}; split vs oracle at theta {e_split:.2e}")
    assert e_fast_r < KTOL and e_split < KTOL
    fast.close(); split.close()


# ------------------------------------------------------------------------------------------ unroll > 1
@pytest.mark.parametrize("where", ["small", "workload3"])
def test_unrolled_iteration_free_running(where):
    """Unroll U = 3 (the paper runs U = 10, App. B): three free-running base steps and one meta step on each side from the
    same start, no state pushed in between; a second iteration follows on the small encoder.

    Asserted at the bars of this file: every base step's gradient, moments and weights, the direct gradient, and the
    quantities the parity target names -- hypergradient, theta, lambda.  The perturbation vector v and the step size
    eps are printed only: free-running from zero moments they are ill-conditioned in the method itself.  The adaptation
    of Eq. 4 (App. C) vanishes identically at t = 1, cancels to a tenth of its terms at t = 2, 3, and peaks at
    lr c1 (1 - beta1) / (4 eps_A) for entries with c2 sqrt(v') near eps_A = 1e-8 (pinned in closed form in
    tests/test_oracle_optim.py), i.e. on the few entries whose gradient history is far below the rounding noise of any
    finite-precision pass; in the float64 oracle itself a relative gradient noise of 1e-3 moves v by more than its norm
    there.  The small encoder therefore runs with eps_A = 1e-5, where that peak is a thousand times lower."""
    if where == "small":
        wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
        orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3, adam_eps=1e-5)
        iters = 2
    else:
        wl = make_workload(3, n_train=128, n_meta=64)
        orc, gpu = make_pair(wl, init_theta(wl), init_lambda(wl))
        iters = 1
    k = 0
    for it in range(iters):
        for u in range(3):
            (x, y), (xm, ym) = _batches(wl, k); k += 1
            tb = dev_batch(gpu, x, y)
            orc.base_step(x, y); gpu.base_step(tb)
            e = dict(g=rel_l2(pull(gpu, "G"), orc.g), theta=rel_l2(pull(gpu, "THETA"), orc.theta),
                     m=rel_l2(pull(gpu, "M"), orc.m), v=rel_l2(pull(gpu, "V"), orc.v))
            print(f"{where} it {it} base step {u}: " + " ".join(f"{kk}={vv:.2e}" for kk, vv in e.items()))
            assert e["g"] < KTOL and e["theta"] < TOL and e["m"] < KTOL and e["v"] < KTOL, e
        r = orc.meta_step(x, y, xm, ym)
        gpu.meta_step(tb, dev_batch(gpu, xm, ym))
        e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), v=rel_l2(pull(gpu, "VDIR"), r["v"]),
                 eps=abs(pull(gpu, "SCALARS")[0] - r["eps"]) / r["eps"], h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
                 theta=rel_l2(pull(gpu, "THETA"), orc.theta), lam=rel_l2(pull(gpu, "LAMBDA"), orc.lam))
        print(f"{where} it {it} meta step: " + " ".join(f"{kk}={vv:.2e}" for kk, vv in e.items()))
        assert e["gmeta"] < KTOL and e["h"] < TOL and e["theta"] < TOL and e["lam"] < TOL, e
        if where == "small":       # well-conditioned there (eps_A = 1e-5): the direction and the step size carry bars too
            assert e["v"] < TOL and e["eps"] < KTOL, e
        assert int(pull(gpu, "COUNTERS")[0]) == 3 * (it + 1) and int(pull(gpu, "COUNTERS")[1]) == it + 1
        assert int(pull(gpu, "COUNTERS")[2]) == 0
    gpu.close()


def test_second_stream_changes_no_result():
    """The backward pass runs its weight-gradient launches, and the per-layer optimizer update / adaptation behind them,
    on a second stream.  With everything on one stream instead (tuning hooks of the library) a base step must give the
    same bits, and a meta step the same numbers up to the order in which the partial sums of ||v||^2 are added."""
    import ctypes
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    res = {}
    for mode in (0, 1):
        orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
        gpu.lib.sama_dev_side_stream(ctypes.c_int32(mode)); gpu.lib.sama_dev_side_sink(ctypes.c_int32(mode))
        try:
            for s in range(3):
                (x, y), (xm, ym) = _batches(wl, s)
                gpu.base_step(dev_batch(gpu, x, y))
            after_base = {k: pull(gpu, k).copy() for k in ("G", "THETA", "M", "V")}
            gpu.meta_step(dev_batch(gpu, x, y), dev_batch(gpu, xm, ym))
            res[mode] = (after_base, {k: pull(gpu, k).copy() for k in ("GMETA", "VDIR", "HYPERGRAD", "THETA", "LAMBDA", "SCALARS")})
        finally:
            gpu.lib.sama_dev_side_stream(ctypes.c_int32(1)); gpu.lib.sama_dev_side_sink(ctypes.c_int32(1))
            gpu.close()
    for k in res[0][0]:
        assert np.array_equal(res[0][0][k], res[1][0][k]), k
    assert np.array_equal(res[0][1]["GMETA"], res[1][1]["GMETA"])
    assert np.array_equal(res[0][1]["VDIR"], res[1][1]["VDIR"])
    assert abs(res[0][1]["SCALARS"][0] - res[1][1]["SCALARS"][0]) <= 1e-6 * res[0][1]["SCALARS"][0]
    for k in ("HYPERGRAD", "THETA", "LAMBDA"):
        assert rel_l2(res[1][1][k], res[0][1][k]) < 1e-4, k


def test_single_sequence_batches():
    """One train sequence and one meta sequence (M = 128 token rows: a single partial GEMM tile row)."""
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    (x, y), (xm, ym) = _batches(wl, 0)
    x, y, xm, ym = x[:1], y[:1], xm[:1], ym[:1]
    for _ in range(2):
        orc.base_step(x, y)
    push_state(orc, gpu)
    orc.base_step(x, y); gpu.base_step(dev_batch(gpu, x, y))
    assert rel_l2(pull(gpu, "G"), orc.g) < KTOL
    push_state(orc, gpu)
    r = orc.meta_step(x, y, xm, ym)
    gpu.meta_step(dev_batch(gpu, x, y), dev_batch(gpu, xm, ym))
    e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), v=rel_l2(pull(gpu, "VDIR"), r["v"]),
             glam_p=rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"]), h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
             theta=rel_l2(pull(gpu, "THETA"), orc.theta), lam=rel_l2(pull(gpu, "LAMBDA"), orc.lam))
    print("single sequence: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
    assert e["gmeta"] < KTOL and e["glam_p"] < KTOL and e["v"] < TOL and e["theta"] < TOL and e["lam"] < TOL
    assert e["h"] < TOL, e
    gpu.close()


def test_free_running_trajectory_is_reproducible_bit_for_bit():
    """No floating-point atomics and a fixed order in every reduction, on two streams: two runs of the same 30
    iterations (unroll 2) from the same start end in the same bits."""
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    outs = []
    for rep in range(2):
        _, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
        for k in range(30):
            (x, y), (xm, ym) = _batches(wl, k)
            tb, mb = dev_batch(gpu, x, y), dev_batch(gpu, xm, ym)
            gpu.base_step(tb); gpu.base_step(tb); gpu.meta_step(tb, mb)
        outs.append({k: pull(gpu, k).copy() for k in ("THETA", "LAMBDA", "M", "V", "HYPERGRAD", "COUNTERS")})
        gpu.close()
    assert int(outs[0]["COUNTERS"][0]) == 60 and int(outs[0]["COUNTERS"][1]) == 30 and int(outs[0]["COUNTERS"][2]) == 0
    assert np.all(np.isfinite(outs[0]["THETA"]))
    for k in outs[0]:
        assert np.array_equal(outs[0][k], outs[1][k]), k


@pytest.mark.parametrize("variant", ["sgd", "sgd_momentum", "sama_na"])
def test_small_encoder_sgd_and_no_adaptation(variant):
    """The bf16 encoder with an SGD base solver (D = base lr) and with the adaptation switched off (SAMA-NA, D = 1):
    the per-layer update / adaptation slices of the two-stream backward take their other branches here."""
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    kw = {"sgd": dict(base_opt="sgd", base_lr=0.05), "sgd_momentum": dict(base_opt="sgd", base_lr=0.02, momentum=0.9),
          "sama_na": dict(adapt_mode=1, base_lr=1e-3)}[variant]
    orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), **kw)
    for s in range(2):
        (x, y), _ = _batches(wl, s)
        orc.base_step(x, y)
    (x, y), (xm, ym) = _batches(wl, 2)
    push_state(orc, gpu)
    th_before = orc.theta.copy()
    orc.base_step(x, y); gpu.base_step(dev_batch(gpu, x, y))
    assert rel_l2(pull(gpu, "G"), orc.g) < KTOL
    assert rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
    if variant != "sama_na":       # SGD's update is linear in g (Adam's divides by sqrt(v'), which magnifies the error of small entries)
        assert rel_l2(pull(gpu, "THETA").astype(np.float64) - th_before, orc.theta - th_before) < KTOL
    if variant == "sgd_momentum":
        assert rel_l2(pull(gpu, "M"), orc.m) < KTOL and rel_l2(orc.m, orc.g) > 0.5                       # the velocity, with history
    push_state(orc, gpu)
    r = orc.meta_step(x, y, xm, ym)
    gpu.meta_step(dev_batch(gpu, x, y), dev_batch(gpu, xm, ym))
    e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), v=rel_l2(pull(gpu, "VDIR"), r["v"]),
             eps=abs(pull(gpu, "SCALARS")[0] - r["eps"]) / r["eps"], h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
             theta=rel_l2(pull(gpu, "THETA"), orc.theta), lam=rel_l2(pull(gpu, "LAMBDA"), orc.lam))
    print(f"{variant}: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
    assert e["gmeta"] < KTOL and e["v"] < KTOL and e["eps"] < KTOL and e["h"] < TOL and e["theta"] < TOL and e["lam"] < TOL
    gpu.close()


def test_padded_batches_small_encoder():
    """Sequence lengths (key-padding mask): base step and meta step against the oracle on a length mix that includes a
    one-token and a full sequence; then the invariants of padding on the GPU alone: full lengths give the bits of no
    lengths, and other tokens in the padded positions change no bit of the gradient."""
    import torch
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    S, V = wl.dims[4], wl.dims[5]
    orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    lens_all = seq_lengths(wl.seed + 1, 64, S)
    for s in range(3):
        (x, y), _ = _batches(wl, s)
        orc.base_step(with_lengths(x, lens_all[5 * s:5 * s + 5]), y)
    for s in range(3, 5):
        (x, y), (xm, ym) = _batches(wl, s)
        lt = lens_all[5 * s:5 * s + 5].copy(); lm = lens_all[40 + 3 * s:43 + 3 * s].copy()
        lt[0], lt[1], lm[0] = 1, S, 2
        push_state(orc, gpu)
        tb, mb = dev_batch(gpu, x, y, lens=lt), dev_batch(gpu, xm, ym, lens=lm)
        # the mask matters on these batches
        assert np.max(np.abs(orc.model.losses(orc.theta, x, y) - orc.model.losses(orc.theta, with_lengths(x, lt), y))) > 1e-3
        lo = orc.base_step(with_lengths(x, lt), y)
        gpu.base_step(tb)
        g = pull(gpu, "G")
        errs = _group_errors(orc, g, orc.g)
        print(f"padded base step {s}: rel-L2 g {rel_l2(g, orc.g):.3e}; worst group {max(errs, key=errs.get)} {max(errs.values()):.3e}")
        assert rel_l2(g, orc.g) < KTOL and all(e < TOL for e in errs.values()), errs
        assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 2e-2 * abs(lo)
        push_state(orc, gpu)
        r = orc.meta_step(with_lengths(x, lt), y, with_lengths(xm, lm), ym)
        gpu.meta_step(tb, mb)
        e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
                 glam_p=rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"]), theta=rel_l2(pull(gpu, "THETA"), orc.theta))
        print(f"padded meta step {s}: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
        assert e["gmeta"] < KTOL and e["glam_p"] < KTOL and e["h"] < TOL and e["theta"] < TOL
    # ---- invariants, GPU against itself
    (x, y), _ = _batches(wl, 5)
    lens = np.array([S, 7, 64, 1, 100], dtype=np.int32)

    def grad_of(xx, ll):
        push_state(orc, gpu)
        gpu.base_step(dev_batch(gpu, xx, y, lens=ll))
        return pull(gpu, "G").copy(), pull(gpu, "LOSSES")[:5].copy()
    g_none, l_none = grad_of(x, None)
    g_full, l_full = grad_of(x, np.full(5, S, dtype=np.int32))
    assert np.array_equal(g_none, g_full) and np.array_equal(l_none, l_full)
    g_a, l_a = grad_of(x, lens)
    x2 = x.copy()
    for b in range(5):
        x2[b, lens[b]:] = V - 1 - b
    g_b, l_b = grad_of(x2, lens)
    tok = orc.model.slices["tok_emb"][0]
    keep = np.ones(g_a.size, dtype=bool); keep[tok:tok + V * wl.dims[1]] = False
    assert np.array_equal(l_a, l_b) and np.array_equal(g_a[keep], g_b[keep])
    tg_a, tg_b = g_a[tok:tok + V * wl.dims[1]].reshape(V, -1), g_b[tok:tok + V * wl.dims[1]].reshape(V, -1)
    real = np.unique(np.concatenate([x[b, :lens[b]] for b in range(5)]))
    assert np.array_equal(tg_a[real], tg_b[real])
    assert np.all(tg_b[[V - 1 - b for b in range(1, 5) if (V - 1 - b) not in real]] == 0.0)      # pad-only tokens: no gradient
    # out-of-range lengths are clamped, not an error
    g_c, _ = grad_of(x, np.array([S + 50, 7, 64, 0, 100], dtype=np.int32))
    assert np.array_equal(g_c, g_a)
    gpu.close()


@pytest.mark.parametrize("S,padded,B", [(64, False, 3), (64, True, 5), (256, False, 3), (256, True, 3), (256, True, 32)])
def test_other_sequence_lengths(S, padded, B):
    """Sequence lengths 64 and 256 (the attention kernels are instantiated per length; 256 walks two tiles per wave):
    one base step and one meta step against the oracle, with and without padding.  The last case fills the 8192-token
    limit of a batch (32 sequences of 256)."""
    Bm = max(2, B // 2)
    wl = make_workload(3, n_train=8 * B, n_meta=8 * Bm, dims=(2, 128, 2, 256, S, 600, 3), batch=B, meta_batch=Bm)
    orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    lens = seq_lengths(wl.seed + S, 6 * B, S)
    lens[0], lens[1] = 1, S
    inp = (lambda x, l: with_lengths(x, l)) if padded else (lambda x, l: x)
    for s in range(3):
        (x, y), _ = _batches(wl, s)
        orc.base_step(inp(x, lens[B * (s + 1):B * (s + 2)]), y)
    (x, y), (xm, ym) = _batches(wl, 3)
    lt, lm = lens[:B], lens[5 * B:5 * B + Bm]
    push_state(orc, gpu)
    tb = dev_batch(gpu, x, y, lens=lt if padded else None)
    mb = dev_batch(gpu, xm, ym, lens=lm if padded else None)
    lo = orc.base_step(inp(x, lt), y)
    gpu.base_step(tb)
    g = pull(gpu, "G")
    errs = _group_errors(orc, g, orc.g)
    print(f"S={S} padded={padded} base: rel-L2 g {rel_l2(g, orc.g):.3e}; worst group {max(errs, key=errs.get)} {max(errs.values()):.3e}")
    assert rel_l2(g, orc.g) < KTOL and all(e < TOL for e in errs.values()), errs
    assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 2e-2 * abs(lo)
    push_state(orc, gpu)
    r = orc.meta_step(inp(x, lt), y, inp(xm, lm), ym)
    gpu.meta_step(tb, mb)
    e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
             glam_p=rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"]), theta=rel_l2(pull(gpu, "THETA"), orc.theta))
    print(f"S={S} padded={padded} meta: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
    assert e["gmeta"] < KTOL and e["glam_p"] < KTOL and e["h"] < TOL and e["theta"] < TOL
    gpu.close()


def test_out_of_range_ids_and_labels_are_clamped():
    """Token ids outside [0, V) and labels outside [0, C) are clamped on the device by every kernel that indexes with
    them (embedding gather, token-gradient scatter, per-sample stage): a batch carrying such values gives the bits of
    the batch with the clamped values, for the base step and for the meta step."""
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    V, C = wl.dims[5], wl.dims[6]
    (x, y), (xm, ym) = _batches(wl, 0)
    bad_x, bad_y = x.copy(), y.copy()
    bad_x[0, 3], bad_x[1, 7], bad_x[2, 0], bad_x[4, 127] = V + 5, -3, 2 ** 30, -2 ** 31
    bad_y[0], bad_y[3] = C + 2, -1
    res = []
    for xx, yy in ((bad_x, bad_y), (np.clip(bad_x, 0, V - 1), np.clip(bad_y, 0, C - 1))):
        _, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
        tb, mb = dev_batch(gpu, xx, yy), dev_batch(gpu, xm, ym)
        gpu.base_step(tb); gpu.base_step(tb); gpu.meta_step(tb, mb)
        res.append({k: pull(gpu, k).copy() for k in ("G", "THETA", "HYPERGRAD", "LAMBDA", "LOSSES")})
        assert np.all(np.isfinite(res[-1]["THETA"])) and int(pull(gpu, "COUNTERS")[2]) == 0
        gpu.close()
    for k in res[0]:
        assert np.array_equal(res[0][k], res[1][k]), k


def test_non_finite_hypergradient_takes_back_the_early_nudge():
    """bf16 models nudge the GEMM block of theta in the pass that writes the +- halves, before the hypergradient exists.
    When the hypergradient then turns out not to be finite (a NaN planted in the weight net's output bias, which the
    direct-gradient pass never reads), the step is skipped like the oracle's: hypergradient 0, lambda and the meta
    moments untouched, the non-GEMM tail of theta untouched bit for bit, the GEMM block back at its old value up to one
    fp32 rounding -- and the working copy and its residual half follow, so the next base step gives the gradient of a
    context that never saw the skipped step."""
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    _, ref = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    for s in range(3):
        (x, y), (xm, ym) = _batches(wl, s)
        gpu.base_step(dev_batch(gpu, x, y)); ref.base_step(dev_batch(ref, x, y)); orc.base_step(x, y)
    lam = pull(gpu, "LAMBDA").copy(); lam_bad = lam.copy(); lam_bad[-1] = np.nan
    gpu.set_state("LAMBDA", lam_bad); orc.lam = lam_bad.astype(np.float64)
    th, mm = pull(gpu, "THETA").copy(), pull(gpu, "META_M").copy()
    r = orc.meta_step(x, y, xm, ym)
    assert orc.status == 1 and orc.meta_t == 0 and r["eps"] > 0
    gpu.meta_step(dev_batch(gpu, x, y), dev_batch(gpu, xm, ym))
    cnt = pull(gpu, "COUNTERS")
    assert int(cnt[1]) == 0 and int(cnt[2]) == 1 and float(pull(gpu, "SCALARS")[0]) > 0
    assert np.all(pull(gpu, "HYPERGRAD") == 0) and np.array_equal(pull(gpu, "META_M"), mm)
    assert np.array_equal(pull(gpu, "LAMBDA"), lam_bad, equal_nan=True)
    th2 = pull(gpu, "THETA")
    ng = _gemm_block(orc)
    assert np.array_equal(th2[ng:], th[ng:])
    assert np.max(np.abs(th2[:ng].astype(np.float64) - th[:ng])) <= 2.0 ** -23 * np.max(np.abs(th[:ng]))
    assert not np.array_equal(pull(gpu, "VDIR"), np.zeros_like(th))          # the direction itself was computed
    gpu.set_state("LAMBDA", lam)
    (x, y), _ = _batches(wl, 3)
    gpu.base_step(dev_batch(gpu, x, y)); ref.base_step(dev_batch(ref, x, y))
    assert rel_l2(pull(gpu, "G"), pull(ref, "G")) < 1e-4, rel_l2(pull(gpu, "G"), pull(ref, "G"))
    gpu.close(); ref.close()


def test_eval_small_encoder_with_padding():
    """sama_eval on the bf16 encoder, padded batch: logits, losses and weights against the oracle at the bf16 working
    weights (what the base step's forward sees)."""
    import torch
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    S = wl.dims[4]
    orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    (x, y), (xm, ym) = _batches(wl, 0)
    push_state(orc, gpu)
    orc.t = 1                                            # evaluate needs no history; keep the oracle's guard quiet
    lens = np.array([S, 9, 1, 77, 40], dtype=np.int32)
    zo = torch.zeros((5, wl.dims[-1]), device=gpu.dev); lo = torch.zeros(5, device=gpu.dev); wo = torch.zeros(5, device=gpu.dev)
    gpu.eval(dev_batch(gpu, x, y, lens=lens), zo, lo, wo)
    z, l, w = orc.evaluate(with_lengths(x, lens), y)
    print(f"eval: logits {rel_l2(zo.cpu().numpy(), z):.2e} losses {rel_l2(lo.cpu().numpy(), l):.2e} weights {rel_l2(wo.cpu().numpy(), w):.2e}")
    assert rel_l2(zo.cpu().numpy(), z) < KTOL and rel_l2(lo.cpu().numpy(), l) < KTOL and rel_l2(wo.cpu().numpy(), w) < KTOL
    gpu.close()


def test_checkpoint_and_resume_continue_bit_for_bit():
    """The settable state (theta, the moments, the kept gradient, lambda and its moments, the counters) is everything a
    run needs: a fresh context that is handed the state of a run after 6 iterations continues with the bits of the
    uninterrupted run (bf16 encoder, two streams, scheduled rates)."""
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    names = ("THETA", "M", "V", "G", "LAMBDA", "META_M", "META_V")
    rate = lambda k: 1e-3 * (1.0 - 0.05 * k)

    def run(gpu, k0, k1):
        for k in range(k0, k1):
            (x, y), (xm, ym) = _batches(wl, k)
            tb, mb = dev_batch(gpu, x, y), dev_batch(gpu, xm, ym)
            gpu.set_lr(rate(k), 1e-3)
            gpu.base_step(tb); gpu.meta_step(tb, mb)

    _, a = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    run(a, 0, 6)
    saved = {n: pull(a, n).copy() for n in names}
    counters = pull(a, "COUNTERS").copy()
    run(a, 6, 10)
    want = {n: pull(a, n).copy() for n in names + ("HYPERGRAD", "COUNTERS")}
    a.close()
    _, b = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    for n in names:
        b.set_state(n, saved[n])
    b.set_state("COUNTERS", counters)
    run(b, 6, 10)
    for n in want:
        assert np.array_equal(pull(b, n), want[n]), n
    b.close()


@pytest.mark.parametrize("d,heads,ffn", [(1280, 20, 1344), (2048, 32, 2048)])
def test_wide_encoder(d, heads, ffn):
    """Hidden widths above 1024 (the LayerNorm kernels then keep eight 16-byte pieces of a row per lane): one base step
    and one meta step against the oracle."""
    wl = make_workload(3, n_train=24, n_meta=8, dims=(1, d, heads, ffn, 64, 300, 3), batch=3, meta_batch=2)
    orc, gpu = make_pair(wl, init_theta(wl, 0.02), init_lambda(wl), base_lr=1e-3)
    for s in range(2):
        (x, y), _ = _batches(wl, s)
        orc.base_step(x, y)
    (x, y), (xm, ym) = _batches(wl, 2)
    push_state(orc, gpu)
    tb, mb = dev_batch(gpu, x, y), dev_batch(gpu, xm, ym)
    lo = orc.base_step(x, y)
    gpu.base_step(tb)
    g = pull(gpu, "G")
    errs = _group_errors(orc, g, orc.g)
    print(f"d={d} base: rel-L2 g {rel_l2(g, orc.g):.3e}; worst group {max(errs, key=errs.get)} {max(errs.values()):.3e}")
    assert rel_l2(g, orc.g) < KTOL and all(e < TOL for e in errs.values()), errs
    assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 2e-2 * abs(lo)
    push_state(orc, gpu)
    r = orc.meta_step(x, y, xm, ym)
    gpu.meta_step(tb, mb)
    e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
             glam_p=rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"]), theta=rel_l2(pull(gpu, "THETA"), orc.theta))
    e["glam_m"] = rel_l2(pull(gpu, "GLAM_MINUS"), r["glam_m"]); e["eps"] = abs(pull(gpu, "SCALARS")[0] - r["eps"]) / r["eps"]
    # h = -(g+ - g-) / (2 eps): with |dg+-| <= GBAR |g+-| and the relative error of eps <= EBAR, the relative error of h is
    # at most GBAR (|g+| + |g-|) / |g+ - g-| + EBAR -- a bar made of the oracle's numbers and the two fixed bars alone.
    # On this single-layer wide model at its initial point the two passes differ in the fourth digit only, so the
    # bar on h is far above the workloads' 2e-2; the inputs of the difference carry the tight bars.
    GBAR, EBAR = 2e-4, KTOL
    amplification = (np.linalg.norm(r["glam_p"]) + np.linalg.norm(r["glam_m"])) / np.linalg.norm(r["glam_p"] - r["glam_m"])
    hbar = GBAR * amplification + EBAR
    print(f"d={d} meta: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()) + f" amplification={amplification:.1e} hbar={hbar:.2e}")
    assert e["gmeta"] < KTOL and e["theta"] < TOL
    assert e["glam_p"] < GBAR and e["glam_m"] < GBAR and e["eps"] < EBAR
    assert e["h"] < hbar
    gpu.close()
