"""Writes tests/golden/oracle_trajectories.json: a few numbers of short oracle runs (losses, step sizes, leading
hypergradient components, parameter norms) on the seeded inputs, for every variant the oracle has.  Calls only
oracle/ and datagen/; the file freezes the oracle's arithmetic, so that a later change to it shows up as a failing
test that the change has to account for (the oracle's correctness itself rests on the pins in tests/test_oracle_*.py,
not on this file)."""
import json
import os
import sys
import numpy as np
sys.path.insert(0, os.path.join(os.path.dirname(__file__), "..", ".."))
from datagen import make_workload, make_aux_batch, init_theta, init_lambda, init_lambda_corr, seq_lengths  # noqa: E402
from oracle import models  # noqa: E402
from oracle.reweight import SamaOracle, ADAM, SGD  # noqa: E402
from oracle.auxtask import AuxTaskOracle  # noqa: E402

SMALL = dict(dims=(2, 64, 1, 128, 64, 300, 3), batch=4, meta_batch=3)


def summary(r, orc, loss):
    return dict(loss=float(loss), eps=float(r["eps"]), h_head=[float(v) for v in r["h"][:6]], h_norm=float(np.linalg.norm(r["h"])),
                v_norm=float(np.linalg.norm(r["v"])), theta_norm=float(np.linalg.norm(orc.theta)), lam_norm=float(np.linalg.norm(orc.lam)))


def run_plain(wl, steps, lam0=None, lens=None, **kw):
    orc = SamaOracle(models.make_model(wl.kind, wl.dims), init_theta(wl), init_lambda(wl) if lam0 is None else lam0,
                     base_lr=wl.base_lr, meta_lr=wl.meta_lr, alpha=wl.alpha, **kw)
    out = []
    it = wl.train_batch(steps)
    x0 = wl.x_train[it] if lens is None else models.with_lengths(wl.x_train[it], lens[0][it])
    orc.base_step(x0, wl.y_train[it])                 # history: the adaptation of the very first Adam step is zero
    for s in range(steps):
        it, im = wl.train_batch(s), wl.meta_batch_idx(s)
        x, y, xm, ym = wl.x_train[it], wl.y_train[it], wl.x_meta[im], wl.y_meta[im]
        if lens is not None:
            x, xm = models.with_lengths(x, lens[0][it]), models.with_lengths(xm, lens[1][im])
        loss = orc.base_step(x, y)
        out.append(summary(orc.meta_step(x, y, xm, ym), orc, loss))
    return out


def build():
    out = {}
    wl1, wl2 = make_workload(1), make_workload(2)
    out["workload1_adam"] = run_plain(wl1, 3)
    out["workload1_sgd_wd"] = run_plain(wl1, 3, base_opt=SGD, weight_decay=0.01)
    out["workload1_sgd_momentum"] = run_plain(wl1, 3, base_opt=SGD, momentum=0.9)
    out["workload1_no_adaptation"] = run_plain(wl1, 3, adapt_mode=1)
    out["workload2_adam_wd"] = run_plain(wl2, 2, weight_decay=0.01)
    out["workload2_label_correction"] = run_plain(wl2, 2, lam0=np.concatenate([init_lambda(wl2), init_lambda_corr(wl2, 5)]),
                                                  corr_hidden=5, corr_kappa=1.5, n_classes=wl2.dims[-1])
    enc = make_workload(3, n_train=16, n_meta=9, **SMALL)
    out["small_encoder"] = run_plain(enc, 2)
    S = enc.dims[4]
    out["small_encoder_padded"] = run_plain(enc, 2, lens=(seq_lengths(enc.seed + 1, 16, S), seq_lengths(enc.seed + 2, 9, S)))
    aux = make_workload(3, n_train=16, n_meta=9, mlm=True, **SMALL)
    orc = AuxTaskOracle(models.make_model(aux.kind, aux.dims, mlm=True), init_theta(aux), init_lambda(aux), base_lr=aux.base_lr,
                        meta_lr=aux.meta_lr, alpha=aux.alpha)
    rows = []
    it = aux.train_batch(2)
    orc.base_step((aux.x_train[it], aux.y_train[it]), make_aux_batch(aux, 2, 3))
    for s in range(2):
        it, im = aux.train_batch(s), aux.meta_batch_idx(s)
        pt = make_aux_batch(aux, s, 3)
        loss = orc.base_step((aux.x_train[it], aux.y_train[it]), pt)
        rows.append(summary(orc.meta_step(pt, (aux.x_meta[im], aux.y_meta[im])), orc, loss))
    out["small_encoder_auxiliary_task"] = rows
    return out


if __name__ == "__main__":
    json.dump(build(), open(os.path.join(os.path.dirname(__file__), "oracle_trajectories.json"), "w"), indent=1)
