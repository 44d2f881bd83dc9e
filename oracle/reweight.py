"""SAMA on the data-reweighting bilevel problem (Sec. 4.1):

    base:  theta*(lambda) = argmin (1/B_eff) sum_i mask_i w(l_i; lambda) l_i(theta)     on noisy data
    meta:  lambda* = argmin mean CE on clean data at theta*(lambda)

one `unroll` of base steps followed by one meta step (Sec. 2, Sec. 3.2).  Float64 throughout.
Readings where the paper is silent are marked "reading:" below.
"""
import numpy as np
from . import corrector, optim, sama_core, wnet

SGD, ADAM = 0, 1


class SamaOracle:
    def __init__(self, model, theta0, lambda0, *, base_opt=ADAM, base_lr=1e-3, beta1=0.9, beta2=0.999,
                 adam_eps=1e-8, meta_lr=1e-3, meta_beta1=0.9, meta_beta2=0.999, meta_eps=1e-8,
                 alpha=1.0, adapt_mode=optim.ADAPT_ADAM, corr_hidden=0, corr_kappa=4.0, n_classes=None,
                 weight_decay=0.0, momentum=0.0):
        self.model = model
        self.theta = np.array(theta0, dtype=np.float64)
        self.lam = np.array(lambda0, dtype=np.float64)
        n = self.theta.size
        self.m = np.zeros(n); self.v = np.zeros(n); self.g = np.zeros(n)
        self.t = 0
        self.meta_m = np.zeros(self.lam.size); self.meta_v = np.zeros(self.lam.size)
        self.meta_t = 0
        self.base_opt, self.base_lr, self.beta1, self.beta2, self.adam_eps = base_opt, base_lr, beta1, beta2, adam_eps
        self.meta_lr, self.meta_beta1, self.meta_beta2, self.meta_eps = meta_lr, meta_beta1, meta_beta2, meta_eps
        self.lr_step = base_lr               # the rate of the last base step
        self.alpha, self.adapt_mode = alpha, adapt_mode
        # reading: the base optimizer's weight decay (the "wdecay" column of the hyperparameter tables of App. B) is an L2
        # term, weight_decay * theta added to the gradient before the solver; g, as kept for the adaptation, includes it
        self.weight_decay = float(weight_decay)
        # reading: "SGD" in the tables of App. B may carry heavy-ball momentum; the velocity lives in self.m
        self.momentum = float(momentum)
        if self.momentum != 0.0 and base_opt != SGD:
            raise ValueError("momentum belongs to the SGD base solver")
        self.status = 0                # 1 after a meta step skipped for ||v|| = 0 / non-finite
        # label correction (Sec. 4.1): lambda = [lambda_r | lambda_c]; corr_hidden = 0 turns it off
        self.Hc, self.kappa, self.C = int(corr_hidden), float(corr_kappa), n_classes
        if self.Hc > 0:
            if n_classes is None:
                raise ValueError("label correction needs n_classes")
            self.nr = self.lam.size - corrector.size(n_classes, self.Hc)
            if self.nr < 4 or (self.nr - 1) % 3 != 0:
                raise ValueError("lambda0 must hold [weight net | corrector]")
        else:
            self.nr = self.lam.size

    # ------------------------------------------------------------------ base level
    def base_step(self, x, y, mask=None):
        """One step of the base solver u on L_base.  w_i is a constant of the backward pass
        (reading: no gradient through the weight net's input, the Meta-Weight-Net convention);
        normalisation is 1/B_eff, B_eff = sum mask (reading of 1/|D_noisy|).  Returns L_base."""
        mask = np.ones(len(y)) if mask is None else np.asarray(mask, dtype=np.float64)
        target = self.targets(self.theta, x, y)
        l = self.model.losses(self.theta, x, target)
        w = wnet.weights(l, self.lam[:self.nr])
        coef = mask * w / mask.sum()
        l, g = self.model.loss_grad(self.theta, x, target, coef)
        g = g + self.weight_decay * self.theta
        self.g = g
        self.t += 1
        self.lr_step = self.base_lr          # a scheduler may change base_lr between steps (lr_scheduler column, App. B)
        if self.base_opt == ADAM:
            self.theta, self.m, self.v = optim.adam_update(self.theta, self.m, self.v, g, self.t, self.base_lr,
                                                           self.beta1, self.beta2, self.adam_eps)
        elif self.momentum != 0.0:
            self.theta, self.m = optim.sgd_momentum_update(self.theta, self.m, g, self.base_lr, self.momentum)
        else:
            self.theta = optim.sgd_update(self.theta, g, self.base_lr)
        return float(np.sum(coef * l))

    def evaluate(self, x, y):
        """What the base step sees of a batch, forward only: (logits, l, w) with l_i the per-sample loss (against the
        corrected label when label correction is on) and w_i = w(l_i; lambda), the learned importance of sample i."""
        target = self.targets(self.theta, x, y)
        l = self.model.losses(self.theta, x, target)
        return self.model.logits(self.theta, x), l, wnet.weights(l, self.lam[:self.nr])

    # ------------------------------------------------------------------ meta level
    def adaptation(self):
        """du/dg on the diagonal from the LAST base step's gradient and its post-update moments
        (reading: no extra backward pass is spent on re-evaluating g at the updated theta, in
        keeping with the three-pass count of Sec. 3.3).  gamma is the rate that step used: under
        a schedule (lr_scheduler column, App. B) base_lr may have moved on since."""
        if self.adapt_mode == optim.ADAPT_NONE:
            return np.ones_like(self.g)
        if self.base_opt == ADAM:
            return optim.adam_adaptation(self.g, self.m, self.v, self.t, self.lr_step, self.beta1, self.beta2,
                                         self.adam_eps)
        return optim.sgd_adaptation(self.g, self.lr_step)

    def targets(self, theta, x, y):
        """What the base loss compares the prediction with: the labels themselves, or the corrected soft labels
        c(x, y; lambda_c) of the label-correction meta learner (constants of every theta-gradient)."""
        if self.Hc == 0:
            return y
        p = corrector.softmax(self.model.logits(theta, x))
        return corrector.forward(self.lam[self.nr:], np.asarray(y), p, self.Hc, self.kappa)[0]

    def glam(self, theta, x, y, mask=None):
        """dL_base(theta, lambda)/dlambda: a forward pass for l_i(theta), then the weight net's backward and, with label
        correction, the corrector's backward.  reading: the weight net's input l_i and the corrector's input
        softmax(z_i) are constants (the same stop-gradients as in the base step), so
            d/dlambda_r = (1/B_eff) sum_i mask_i l_i dw_i/dlambda_r,
            d/dlambda_c = (1/B_eff) sum_i mask_i w_i sum_k (-log p_ik) dc_ik/dlambda_c."""
        if self.Hc == 0:
            l = self.model.losses(theta, x, y)
            return wnet.base_loss_grad_lambda(l, self.lam, mask)
        mk = np.ones(len(y)) if mask is None else np.asarray(mask, dtype=np.float64)
        z = self.model.logits(theta, x)
        p = corrector.softmax(z)
        logp = z - z.max(axis=1, keepdims=True)
        logp = logp - np.log(np.exp(logp).sum(axis=1, keepdims=True))
        c, cache = corrector.forward(self.lam[self.nr:], np.asarray(y), p, self.Hc, self.kappa)
        l = -(c * logp).sum(axis=1)
        g_r = wnet.base_loss_grad_lambda(l, self.lam[:self.nr], mask)
        w = wnet.weights(l, self.lam[:self.nr])
        dc = (mk * w / mk.sum())[:, None] * (-logp)
        g_c = corrector.backward(self.lam[self.nr:], cache, dc, self.Hc)
        return np.concatenate([g_r, g_c])

    def meta_grad(self, xt, yt, xm, ym, mask_t=None, mask_m=None):
        """Eq. 5 on the current state; changes nothing.  Returns dict(h, eps, v, g_meta, glam_p, glam_m).
        reading: the theta+- passes reuse the train batch (xt, yt) that produced g."""
        if self.t == 0:
            raise RuntimeError("meta_grad before any base step")
        mm = np.ones(len(ym)) if mask_m is None else np.asarray(mask_m, dtype=np.float64)
        _, g_meta = self.model.loss_grad(self.theta, xm, ym, mm / mm.sum())        # direct gradient, Eq. 1
        v = sama_core.perturbation(self.adaptation(), g_meta)
        eps = sama_core.step_size(v, self.alpha)
        h, gp, gm = sama_core.central_difference(lambda th: self.glam(th, xt, yt, mask_t), self.theta, v, eps)
        return dict(h=h, eps=eps, v=v, g_meta=g_meta, glam_p=gp, glam_m=gm)

    def meta_step(self, xt, yt, xm, ym, mask_t=None, mask_m=None):
        """meta_grad, then Adam on lambda with h (Table 4), then theta <- theta - eps v (end of Sec. 3.2).
        reading: the nudge leaves the base moments and step count alone; a zero / non-finite ||v||
        skips both updates and raises `status`."""
        r = self.meta_grad(xt, yt, xm, ym, mask_t, mask_m)
        if r["eps"] == 0.0 or not np.all(np.isfinite(r["h"])):
            self.status = 1
            return r
        self.meta_t += 1
        self.lam, self.meta_m, self.meta_v = optim.adam_update(self.lam, self.meta_m, self.meta_v, r["h"],
                                                               self.meta_t, self.meta_lr, self.meta_beta1,
                                                               self.meta_beta2, self.meta_eps)
        self.theta = sama_core.nudge(self.theta, r["v"], r["eps"])
        return r
