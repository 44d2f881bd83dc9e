"""SAMA on auxiliary-task reweighting (Sec. 4.3, continued pretraining as a multitask problem):

    base:  theta*(lambda) = argmin  L_ft(D_ft; theta) + (1/|D_pt|) sum_{x in D_pt} w(x; lambda) L_pt(x; theta)
    meta:  lambda* = argmin L_ft(D_ft; theta*(lambda))

L_ft: mean cross-entropy of the classifier head; L_pt(x; theta): masked-token cross-entropy of sequence x, the mean
over its masked positions.  Float64.  Test infrastructure: a slow statement of the method to check the GPU path with.

reading: the paper does not say what w sees of x; here, as in the data-reweighting problem, w(x; lambda) =
w(L_pt(x; theta); lambda) is the 1 -> H -> 1 weight net on the sequence's own pretraining loss, a constant of the
theta-gradient.  reading: the meta level uses batches of the same finetuning task (the paper adds no validation data).
One base step takes one finetuning batch and one pretraining batch; the theta+- passes of Eq. 5 need the pretraining
batch only, because the finetuning term of the base loss does not depend on lambda.
"""
import numpy as np
from . import models, optim, sama_core, wnet
from .reweight import SamaOracle, ADAM


def seq_losses(l_pos, seq, n_pt):
    """L_pt of each sequence: mean of the masked-token losses of its positions (0 for a sequence without any)."""
    out = np.zeros(n_pt)
    cnt = np.zeros(n_pt)
    for j in range(len(seq)):
        out[seq[j]] += l_pos[j]
        cnt[seq[j]] += 1.0
    return out / np.maximum(cnt, 1.0), cnt


class AuxTaskOracle(SamaOracle):
    """Batches: ft = (ids_ft [n_ft, S], y_ft [n_ft]); pt = (ids_pt [n_pt, S], seq, pos, tgt) with masked position j at
    (seq[j], pos[j]) of ids_pt and target token tgt[j].  ids_ft, ids_pt and the meta batch's ids may each be a
    models.with_lengths(ids, lens) pair (padded sequences)."""

    def base_step(self, ft, pt):
        ids_ft, y_ft = ft
        ids_pt, seq, pos, tgt = pt
        n_ft, n_pt = len(models.split_lengths(ids_ft)[0]), len(models.split_lengths(ids_pt)[0])
        ids = models.cat_inputs(ids_ft, ids_pt)
        l_pos = self.model.mlm_losses(self.theta, ids_pt, seq, pos, tgt)
        l_seq, cnt = seq_losses(l_pos, seq, n_pt)
        w = wnet.weights(l_seq, self.lam)
        coef = np.concatenate([np.full(n_ft, 1.0 / n_ft), np.zeros(n_pt)])
        y = np.concatenate([np.asarray(y_ft), np.zeros(n_pt, dtype=np.asarray(y_ft).dtype)])
        coef_pos = (w / (n_pt * np.maximum(cnt, 1.0)))[seq]
        l, l_pos2, g = self.model.loss_grad_mlm(self.theta, ids, y, coef, np.asarray(seq) + n_ft, pos, tgt, coef_pos)
        g = g + self.weight_decay * self.theta
        self.g = g
        self.t += 1
        self.lr_step = self.base_lr          # a scheduler may change base_lr between steps (lr_scheduler column, App. B)
        if self.base_opt == ADAM:
            self.theta, self.m, self.v = optim.adam_update(self.theta, self.m, self.v, g, self.t, self.base_lr,
                                                           self.beta1, self.beta2, self.adam_eps)
        else:
            self.theta = optim.sgd_update(self.theta, g, self.base_lr)
        return float(np.sum(coef * l) + np.sum(coef_pos * l_pos2))

    def base_loss(self, theta, lam, ft, pt):
        """The scalar the base step descends (for checks)."""
        ids_ft, y_ft = ft
        ids_pt, seq, pos, tgt = pt
        l_seq, _ = seq_losses(self.model.mlm_losses(theta, ids_pt, seq, pos, tgt), seq, len(models.split_lengths(ids_pt)[0]))
        return float(np.mean(self.model.losses(theta, ids_ft, y_ft))) + wnet.base_loss(l_seq, lam)

    def evaluate_aux(self, pt):
        """(L_pt(x), w(L_pt(x); lambda)) of each auxiliary sequence at the current state, forward only."""
        ids_pt, seq, pos, tgt = pt
        l_seq, _ = seq_losses(self.model.mlm_losses(self.theta, ids_pt, seq, pos, tgt), seq, len(models.split_lengths(ids_pt)[0]))
        return l_seq, wnet.weights(l_seq, self.lam)

    def glam(self, theta, pt):
        """dL_base/dlambda: only the weighted pretraining term depends on lambda."""
        ids_pt, seq, pos, tgt = pt
        l_seq, _ = seq_losses(self.model.mlm_losses(theta, ids_pt, seq, pos, tgt), seq, len(models.split_lengths(ids_pt)[0]))
        return wnet.base_loss_grad_lambda(l_seq, self.lam, None)

    def meta_grad(self, pt, meta):
        """Eq. 5 on the current state; changes nothing: direct gradient of the mean finetuning loss on the meta batch
        (Eq. 1), v = D g_meta, eps = alpha / ||v||, the +- passes on the pretraining batch that produced g."""
        if self.t == 0:
            raise RuntimeError("meta_grad before any base step")
        ids_m, y_m = meta
        _, g_meta = self.model.loss_grad(self.theta, ids_m, y_m, np.full(len(y_m), 1.0 / len(y_m)))
        v = sama_core.perturbation(self.adaptation(), g_meta)
        eps = sama_core.step_size(v, self.alpha)
        h, gp, gm = sama_core.central_difference(lambda th: self.glam(th, pt), self.theta, v, eps)
        return dict(h=h, eps=eps, v=v, g_meta=g_meta, glam_p=gp, glam_m=gm)

    def meta_step(self, pt, meta):
        """meta_grad, Adam on lambda with h, theta <- theta - eps v; skipped (status raised) for a degenerate v."""
        r = self.meta_grad(pt, meta)
        if r["eps"] == 0.0 or not np.all(np.isfinite(r["h"])):
            self.status = 1
            return r
        self.meta_t += 1
        self.lam, self.meta_m, self.meta_v = optim.adam_update(self.lam, self.meta_m, self.meta_v, r["h"], self.meta_t,
                                                               self.meta_lr, self.meta_beta1, self.meta_beta2, self.meta_eps)
        self.theta = sama_core.nudge(self.theta, r["v"], r["eps"])
        return r
