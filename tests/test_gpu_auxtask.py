"""GPU parity of auxiliary-task reweighting (Sec. 4.3: L_base = L_ft + weighted masked-token loss of the auxiliary
sequences, L_meta = L_ft): the HIP path through the C ABI against the float64 oracle on the same seeded inputs,
teacher-forced from the oracle's unrounded state, on a small encoder with a 640-token vocabulary (bf16 GEMM operands)."""
import numpy as np
import pytest
from datagen import make_workload, make_aux_batch, make_aux_workload, AUX_TASK, init_theta, init_lambda
from harness import rel_l2, make_aux_pair, dev_batch, dev_aux_batch, push_state, pull
from oracle.models import with_lengths

pytestmark = pytest.mark.gpu
KTOL, TOL = 1e-2, 2e-2
SMALL = dict(dims=(2, 192, 3, 320, 128, 640, 3), batch=5, meta_batch=3, mlm=True)


def _setup(n_pt=4, scale=0.02):
    wl = make_workload(3, n_train=40, n_meta=12, **SMALL)
    orc, gpu = make_aux_pair(wl, init_theta(wl, scale), init_lambda(wl), max_aux_batch=n_pt, max_aux_masked=n_pt * 26,
                             base_lr=1e-3)
    return wl, orc, gpu


def _ft(wl, step):
    it, im = wl.train_batch(step), wl.meta_batch_idx(step)
    return (wl.x_train[it], wl.y_train[it]), (wl.x_meta[im], wl.y_meta[im])


def _group_errors(orc, got, want):
    out = {}
    for name, (off, shape) in orc.model.slices.items():
        sl = slice(off, off + int(np.prod(shape)))
        out[name] = rel_l2(got[sl], want[sl])
    return out


def test_aux_base_step_parity():
    wl, orc, gpu = _setup()
    for s in range(2):
        ft, _ = _ft(wl, s)
        pt = make_aux_batch(wl, s, 4)
        push_state(orc, gpu)
        th = orc.theta.copy()
        l_ft = orc.model.losses(th, ft[0], ft[1])
        l_pos = orc.model.mlm_losses(th, pt[0], pt[1], pt[2], pt[3])
        l_seq = np.array([l_pos[pt[1] == i].mean() for i in range(4)])
        lo = orc.base_step(ft, pt)
        gpu.aux_base_step(dev_batch(gpu, ft[0], ft[1]), dev_aux_batch(gpu, *pt))
        losses = pull(gpu, "LOSSES")
        assert np.max(np.abs(losses[:5] - l_ft)) < 2e-2 * max(1.0, np.max(l_ft))
        assert np.max(np.abs(losses[5:9] - l_seq)) < 2e-2 * np.max(l_seq), (losses[5:9], l_seq)
        assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 1e-2 * abs(lo)
        g = pull(gpu, "G")
        errs = _group_errors(orc, g, orc.g)
        worst = max(errs, key=errs.get)
        print(f"aux base step {s}: L_base {lo:.4f} rel-L2 g {rel_l2(g, orc.g):.3e}; worst group {worst} {errs[worst]:.3e}; "
              f"Wmlm {errs['Wmlm']:.3e} bmlm {errs['bmlm']:.3e}")
        assert rel_l2(g, orc.g) < KTOL
        assert errs["Wmlm"] < KTOL and errs["bmlm"] < KTOL and errs["tok_emb"] < TOL
        assert all(e < TOL for e in errs.values()), errs
        # the first Adam steps are sign-like (|update| = lr whatever |g|), so theta carries the gradient's rounding noise
        assert rel_l2(pull(gpu, "THETA"), orc.theta) < TOL
        assert int(pull(gpu, "COUNTERS")[0]) == orc.t
    gpu.close()


def test_aux_meta_step_parity():
    wl, orc, gpu = _setup()
    nw = orc.model.slices["Wmlm"]
    for s in range(3):
        ft, _ = _ft(wl, s)
        orc.base_step(ft, make_aux_batch(wl, s, 4))
    for s in range(3, 5):
        ft, meta = _ft(wl, s)
        pt = make_aux_batch(wl, s, 4 if s == 3 else 3)          # the second round with a smaller auxiliary batch
        orc.base_step(ft, pt)
        push_state(orc, gpu)
        ptb, mb = dev_aux_batch(gpu, *pt), dev_batch(gpu, meta[0], meta[1])
        gpu.aux_meta_grad(ptb, mb)
        assert np.array_equal(pull(gpu, "THETA"), orc.theta.astype(np.float32))
        h_pure = pull(gpu, "HYPERGRAD")
        r = orc.meta_step(pt, meta)
        gpu.aux_meta_step(ptb, mb)
        gm = pull(gpu, "GMETA")
        assert np.all(gm[nw[0]:nw[0] + int(np.prod(nw[1]))] == 0)      # L_ft does not touch the masked-token head
        h = pull(gpu, "HYPERGRAD")
        e = dict(gmeta=rel_l2(gm, r["g_meta"]), v=rel_l2(pull(gpu, "VDIR"), r["v"]),
                 eps=abs(pull(gpu, "SCALARS")[0] - r["eps"]) / r["eps"], h=rel_l2(h, r["h"]),
                 glam_p=rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"]), glam_m=rel_l2(pull(gpu, "GLAM_MINUS"), r["glam_m"]),
                 theta=rel_l2(pull(gpu, "THETA"), orc.theta), lam=rel_l2(pull(gpu, "LAMBDA"), orc.lam))
        print(f"aux meta step {s}: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
        # two routes through the elementwise chain (separate low halves / one fused pass): agreement to the rounding of
        # the low halves, amplified by the difference of Eq. 5, not bit for bit
        assert rel_l2(h_pure, r["h"]) < TOL and rel_l2(h, h_pure) < TOL
        assert e["gmeta"] < KTOL and e["glam_p"] < KTOL and e["glam_m"] < KTOL and e["eps"] < KTOL and e["v"] < TOL
        assert e["h"] < TOL, e
        assert e["theta"] < TOL and e["lam"] < TOL
        assert int(pull(gpu, "COUNTERS")[2]) == 0 and int(pull(gpu, "COUNTERS")[1]) == orc.meta_t
    gpu.close()


def test_aux_padded_batches():
    """Sequence lengths on the finetuning, the auxiliary and the meta batch (key-padding mask): one base step and one
    meta step against the oracle; each auxiliary sequence is as long as its last masked position at least."""
    wl, orc, gpu = _setup()
    S = wl.dims[4]
    for s in range(3):
        ft, _ = _ft(wl, s)
        orc.base_step(ft, make_aux_batch(wl, s, 4))
    ft, meta = _ft(wl, 3)
    ids_pt, seq, pos, tgt = make_aux_batch(wl, 3, 4)
    last = np.array([pos[seq == i].max() for i in range(4)])
    l_pt = np.minimum(last + np.array([1, 9, 40, S]), S).astype(np.int32)
    l_ft = np.array([S, 1, 30, 77, 5], dtype=np.int32); l_m = np.array([12, S, 3], dtype=np.int32)
    ftl, ptl, metal = (with_lengths(ft[0], l_ft), ft[1]), (with_lengths(ids_pt, l_pt), seq, pos, tgt), (with_lengths(meta[0], l_m), meta[1])
    push_state(orc, gpu)
    ref_l = orc.model.mlm_losses(orc.theta, ids_pt, seq, pos, tgt)
    assert np.max(np.abs(ref_l - orc.model.mlm_losses(orc.theta, ptl[0], seq, pos, tgt))) > 1e-3      # the mask matters
    lo = orc.base_step(ftl, ptl)
    ftb, ptb = dev_batch(gpu, ft[0], ft[1], lens=l_ft), dev_aux_batch(gpu, ids_pt, seq, pos, tgt, lens=l_pt)
    gpu.aux_base_step(ftb, ptb)
    g = pull(gpu, "G")
    errs = _group_errors(orc, g, orc.g)
    print(f"padded aux base step: rel-L2 g {rel_l2(g, orc.g):.3e}; worst group {max(errs, key=errs.get)} {max(errs.values()):.3e}")
    assert rel_l2(g, orc.g) < KTOL and all(e < TOL for e in errs.values()), errs
    assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 1e-2 * abs(lo)
    push_state(orc, gpu)
    r = orc.meta_step(ptl, metal)
    gpu.aux_meta_step(ptb, dev_batch(gpu, meta[0], meta[1], lens=l_m))
    e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
             glam_p=rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"]), theta=rel_l2(pull(gpu, "THETA"), orc.theta))
    print("padded aux meta step: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
    assert e["gmeta"] < KTOL and e["glam_p"] < KTOL and e["h"] < TOL and e["theta"] < TOL
    # lengths on one half only: the other half counts as full
    push_state(orc, gpu)
    gpu.aux_base_step(dev_batch(gpu, ft[0], ft[1]), dev_aux_batch(gpu, ids_pt, seq, pos, tgt, lens=np.full(4, S, dtype=np.int32)))
    g_half = pull(gpu, "G").copy()
    push_state(orc, gpu)
    gpu.aux_base_step(dev_batch(gpu, ft[0], ft[1]), dev_aux_batch(gpu, ids_pt, seq, pos, tgt))
    assert np.array_equal(g_half, pull(gpu, "G"))
    gpu.close()


def test_aux_sequence_length_256():
    """The auxiliary task at the sequence length of the paper's continued-pretraining runs (256): one base step and one
    meta step against the oracle."""
    wl = make_workload(3, n_train=40, n_meta=12, **dict(SMALL, dims=(2, 192, 3, 320, 256, 640, 3)))
    n_pt = 3
    orc, gpu = make_aux_pair(wl, init_theta(wl, 0.02), init_lambda(wl), max_aux_batch=n_pt, max_aux_masked=n_pt * 52, base_lr=1e-3)
    for s in range(2):
        ft, _ = _ft(wl, s)
        orc.base_step(ft, make_aux_batch(wl, s, n_pt))
    ft, meta = _ft(wl, 2)
    pt = make_aux_batch(wl, 2, n_pt)
    push_state(orc, gpu)
    lo = orc.base_step(ft, pt)
    ftb, ptb = dev_batch(gpu, ft[0], ft[1]), dev_aux_batch(gpu, *pt)
    gpu.aux_base_step(ftb, ptb)
    g = pull(gpu, "G")
    errs = _group_errors(orc, g, orc.g)
    print(f"S=256 aux base step: rel-L2 g {rel_l2(g, orc.g):.3e}; worst group {max(errs, key=errs.get)} {max(errs.values()):.3e}")
    assert rel_l2(g, orc.g) < KTOL and all(e < TOL for e in errs.values()), errs
    assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 1e-2 * abs(lo)
    push_state(orc, gpu)
    r = orc.meta_step(pt, meta)
    gpu.aux_meta_step(ptb, dev_batch(gpu, meta[0], meta[1]))
    e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
             glam_p=rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"]), theta=rel_l2(pull(gpu, "THETA"), orc.theta))
    print("S=256 aux meta step: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()))
    assert e["gmeta"] < KTOL and e["glam_p"] < KTOL and e["h"] < TOL and e["theta"] < TOL
    gpu.close()


def test_aux_eval_returns_sequence_losses_and_weights():
    import torch
    wl, orc, gpu = _setup()
    for s in range(2):
        ft, _ = _ft(wl, s)
        orc.base_step(ft, make_aux_batch(wl, s, 4))
    push_state(orc, gpu)
    ids_pt, seq, pos, tgt = make_aux_batch(wl, 2, 3)
    lens = np.array([128, max(pos[seq == 1]) + 1, 128], dtype=np.int32)
    before = {k: pull(gpu, k).copy() for k in ("THETA", "LAMBDA", "M", "V", "G", "SCALARS", "COUNTERS")}
    lo = torch.full((3,), -1.0, device=gpu.dev); wo = torch.full((3,), -1.0, device=gpu.dev)
    gpu.aux_eval(dev_aux_batch(gpu, ids_pt, seq, pos, tgt, lens=lens), lo, wo)
    l, w = orc.evaluate_aux((with_lengths(ids_pt, lens), seq, pos, tgt))
    print(f"aux eval: losses {rel_l2(lo.cpu().numpy(), l):.2e} weights {rel_l2(wo.cpu().numpy(), w):.2e}")
    assert rel_l2(lo.cpu().numpy(), l) < KTOL and rel_l2(wo.cpu().numpy(), w) < KTOL
    for k, v in before.items():
        assert np.array_equal(pull(gpu, k), v), k
    gpu.aux_eval(dev_aux_batch(gpu, ids_pt, seq, pos, tgt, lens=lens), weights_out=wo)
    gpu.close()


def test_aux_entry_points_reject_bad_batches():
    import torch
    import paper_2310_05674_amd as pkg
    wl, orc, gpu = _setup()
    ft, meta = _ft(wl, 0)
    pt = make_aux_batch(wl, 0, 4)
    good = dev_aux_batch(gpu, *pt)
    with pytest.raises(pkg.SamaError):      # meta gradient before any base step
        gpu.aux_meta_step(good, dev_batch(gpu, meta[0], meta[1]))
    big = make_aux_batch(wl, 0, 5)
    with pytest.raises(pkg.SamaError):      # more sequences than max_aux_batch
        gpu.aux_base_step(dev_batch(gpu, ft[0], ft[1]), dev_aux_batch(gpu, *big))
    many = gpu.aux_batch(good._keep[0], torch.arange(4 * 26 + 1, dtype=torch.int32, device=gpu.dev),
                         torch.zeros(4 * 26 + 1, dtype=torch.int32, device=gpu.dev))
    with pytest.raises(pkg.SamaError):      # more masked positions than max_aux_masked
        gpu.aux_base_step(dev_batch(gpu, ft[0], ft[1]), many)
    gpu.close()
    # a context without the head refuses the auxiliary entry points
    wl2 = make_workload(3, n_train=40, n_meta=12, dims=SMALL["dims"], batch=5, meta_batch=3)
    from harness import make_pair
    _, plain = make_pair(wl2, init_theta(wl2), init_lambda(wl2))
    with pytest.raises(pkg.SamaError):
        plain.aux_base_step(dev_batch(plain, ft[0], ft[1]), dev_aux_batch(plain, *pt))
    plain.close()


def test_aux_full_size_parity():
    """The configuration `bench.py --aux` times (12 layers, d = 768, 50304-token vocabulary, 16 + 16 sequences of 256 tokens): base
    step 0 from the bf16-representable initial theta at the kernel-arithmetic bar, then one meta step from the oracle's
    state at the end-to-end bar with nothing snapped."""
    import time
    t0 = time.time()
    n_pt = AUX_TASK["n_pt"]
    wl = make_aux_workload(n_train=32, n_meta=16)
    orc, gpu = make_aux_pair(wl, init_theta(wl), init_lambda(wl), max_aux_batch=n_pt, max_aux_masked=n_pt * (wl.dims[4] // 5 + 1))
    ft, _ = _ft(wl, 0)
    pt = make_aux_batch(wl, 0, n_pt)
    lo = orc.base_step(ft, pt)
    gpu.aux_base_step(dev_batch(gpu, ft[0], ft[1]), dev_aux_batch(gpu, *pt))
    g = pull(gpu, "G")
    errs = _group_errors(orc, g, orc.g)
    worst = max(errs, key=errs.get)
    print(f"aux full size: L_base {lo:.3f} rel-L2 g {rel_l2(g, orc.g):.3e}, worst group {worst} {errs[worst]:.1e}, Wmlm "
          f"{errs['Wmlm']:.1e} bmlm {errs['bmlm']:.1e}  [{time.time() - t0:.0f}s]", flush=True)
    assert rel_l2(g, orc.g) < KTOL and errs[worst] < 3e-2
    assert abs(float(pull(gpu, "SCALARS")[2]) - lo) < 1e-2 * abs(lo)
    ft, meta = _ft(wl, 1)
    pt = make_aux_batch(wl, 1, n_pt)
    orc.base_step(ft, pt)
    push_state(orc, gpu)
    r = orc.meta_step(pt, meta)
    gpu.aux_meta_step(dev_aux_batch(gpu, *pt), dev_batch(gpu, meta[0], meta[1]))
    e = dict(gmeta=rel_l2(pull(gpu, "GMETA"), r["g_meta"]), v=rel_l2(pull(gpu, "VDIR"), r["v"]),
             eps=abs(pull(gpu, "SCALARS")[0] - r["eps"]) / r["eps"], h=rel_l2(pull(gpu, "HYPERGRAD"), r["h"]),
             glam_p=rel_l2(pull(gpu, "GLAM_PLUS"), r["glam_p"]),
             theta=rel_l2(pull(gpu, "THETA"), orc.theta), lam=rel_l2(pull(gpu, "LAMBDA"), orc.lam))
    e["fd_signal"] = np.linalg.norm(r["glam_p"] - r["glam_m"]) / np.linalg.norm(r["glam_p"])
    print("aux full size: " + " ".join(f"{k}={v:.2e}" for k, v in e.items()) + f"  [{time.time() - t0:.0f}s]", flush=True)
    assert e["h"] < TOL and e["theta"] < TOL and e["lam"] < TOL and e["eps"] < TOL and e["gmeta"] < TOL and e["v"] < TOL, e
    assert int(pull(gpu, "COUNTERS")[2]) == 0
    gpu.close()
