"""Pins for the auxiliary-task part of the oracle (oracle/auxtask.py, the masked-token head of oracle/models.py;
Sec. 4.3): the head against a second implementation from torch library layers with autograd, the assembled base
gradient and lambda-gradient against differences of the scalar base loss, the finite-difference product of Eq. 5
against the mixed partial of that scalar, and the special case of constant weights."""
import numpy as np
import pytest
from datagen import CounterRNG, make_workload, make_aux_batch, param_layout
from oracle import models, wnet
from oracle.auxtask import AuxTaskOracle, seq_losses

torch = pytest.importorskip("torch")
from test_oracle_models import _torch_encoder_losses      # noqa: E402  (the torch.nn assembly of the same encoder)

DIMS = (2, 16, 4, 32, 8, 40, 3)


def _setup(seed=3, n_ft=3, n_pt=4):
    enc = models.Encoder(*DIMS, mlm=True)
    L, d, heads, ffn, S, V, C = DIMS
    r = CounterRNG(seed)
    th = 0.3 * r.normal(1, enc.n)
    for name in ("emb_ln_g",) + tuple(f"l{l}.ln{k}_g" for l in range(L) for k in (1, 2)):
        enc.get(th, name)[...] += 1.0
    ids_ft = r.integers(2, n_ft * S, V).reshape(n_ft, S); ids_ft[:, 0] = 0
    y_ft = r.integers(3, n_ft, C)
    ids_pt = r.integers(4, n_pt * S, V).reshape(n_pt, S); ids_pt[:, 0] = 0
    seq = np.array([0, 0, 1, 2, 2, 2, 3]); pos = np.array([1, 5, 3, 2, 4, 7, 6])
    tgt = r.integers(5, len(seq), V)
    H = 4
    lam = np.concatenate([r.normal(6, H), np.abs(r.normal(7, H)), r.normal(8, H), [0.2]])
    return enc, th, (ids_ft, y_ft), (ids_pt, seq, pos, tgt), lam


def test_layout_agrees_with_datagen():
    enc = models.Encoder(*DIMS, mlm=True)
    assert [(n, tuple(s), o) for n, s, o in param_layout("encoder", DIMS, mlm=True)] == \
        sorted([(n, tuple(s), o) for n, (o, s) in enc.slices.items()], key=lambda t: t[2])
    plain = models.Encoder(*DIMS)
    assert enc.n == plain.n + DIMS[5] * DIMS[1] + DIMS[5]


def test_masked_token_head_vs_torch_autograd():
    enc, th, (ids_ft, y_ft), (ids_pt, seq, pos, tgt), _ = _setup()
    n_ft = len(ids_ft)
    ids = np.concatenate([ids_ft, ids_pt])
    y = np.concatenate([y_ft, np.zeros(len(ids_pt), dtype=y_ft.dtype)])
    r = CounterRNG(9)
    coef = np.concatenate([r.uniform(1, n_ft), np.zeros(len(ids_pt))]); coef_pos = r.uniform(2, len(seq))
    l, l_pos, g = enc.loss_grad_mlm(th, ids, y, coef, seq + n_ft, pos, tgt, coef_pos)
    # second implementation: torch.nn layers for the trunk, F.linear + F.cross_entropy for the head
    F = torch.nn.functional
    t = torch.tensor(th, dtype=torch.float64, requires_grad=True)
    P = lambda name: t[enc.slices[name][0]:enc.slices[name][0] + int(np.prod(enc.slices[name][1]))].reshape(enc.slices[name][1])
    x = F.layer_norm(F.embedding(torch.tensor(ids, dtype=torch.long), P("tok_emb")) + P("pos_emb")[:ids.shape[1]], (enc.d,),
                     P("emb_ln_g"), P("emb_ln_b"), 1e-5)
    for k in range(enc.L):
        p = f"l{k}."
        xs = x.transpose(0, 1)
        a, _ = F.multi_head_attention_forward(xs, xs, xs, enc.d, enc.heads, P(p + "Wqkv"), P(p + "bqkv"), None, None,
                                              False, 0.0, P(p + "Wo"), P(p + "bo"), training=False, need_weights=False)
        x = F.layer_norm(x + a.transpose(0, 1), (enc.d,), P(p + "ln1_g"), P(p + "ln1_b"), 1e-5)
        f = F.linear(F.gelu(F.linear(x, P(p + "W1"), P(p + "b1"))), P(p + "W2"), P(p + "b2"))
        x = F.layer_norm(x + f, (enc.d,), P(p + "ln2_g"), P(p + "ln2_b"), 1e-5)
    lc = F.cross_entropy(F.linear(x[:, 0, :], P("Wc"), P("bc")), torch.tensor(y, dtype=torch.long), reduction="none")
    lt = F.cross_entropy(F.linear(x[torch.tensor(seq + n_ft), torch.tensor(pos)], P("Wmlm"), P("bmlm")),
                         torch.tensor(tgt, dtype=torch.long), reduction="none")
    ((lc * torch.tensor(coef)).sum() + (lt * torch.tensor(coef_pos)).sum()).backward()
    assert np.allclose(l, lc.detach().numpy(), rtol=1e-11) and np.allclose(l_pos, lt.detach().numpy(), rtol=1e-11)
    assert np.allclose(enc.mlm_losses(th, ids_pt, seq, pos, tgt), l_pos, rtol=1e-12)     # sequences are independent
    gt = t.grad.numpy()
    for name, (off, shape) in enc.slices.items():
        sl = slice(off, off + int(np.prod(shape)))
        assert np.max(np.abs(g[sl] - gt[sl])) <= 1e-9 * (np.max(np.abs(gt[sl])) + 1e-12), name
    assert np.linalg.norm(g[slice(*[enc.slices["Wmlm"][0], enc.slices["Wmlm"][0] + 10])]) > 0
    # without masked positions the function is the plain classifier gradient
    l0, g0 = enc.loss_grad(th, ids, y, coef)
    _, _, g1 = enc.loss_grad_mlm(th, ids, y, coef, seq + n_ft, pos, tgt, np.zeros(len(seq)))
    assert np.allclose(g0, g1, rtol=0, atol=1e-15) and np.allclose(l0, l)


def test_sequence_loss_is_the_mean_over_its_positions():
    l_pos = np.array([1.0, 3.0, 5.0, 2.0, 4.0, 6.0, 7.0])
    l, cnt = seq_losses(l_pos, np.array([0, 0, 1, 2, 2, 2, 4]), 5)
    assert np.array_equal(l, [2.0, 5.0, 4.0, 0.0, 7.0]) and np.array_equal(cnt, [2, 1, 3, 0, 1])


def test_base_gradient_and_glam_are_gradients_of_the_scalar_base_loss():
    enc, th, ft, pt, lam = _setup()
    orc = AuxTaskOracle(enc, th, lam, base_lr=1e-2)
    L0 = orc.base_loss(th, lam, ft, pt)
    Lb = orc.base_step(ft, pt)
    assert abs(Lb - L0) < 1e-12 * abs(L0)
    # d/dlambda by differences
    gl = orc.glam(th, pt)
    for k in range(len(lam)):
        e = np.zeros(len(lam)); e[k] = 1e-6
        fd = (orc.base_loss(th, lam + e, ft, pt) - orc.base_loss(th, lam - e, ft, pt)) / 2e-6
        assert abs(fd - gl[k]) < 1e-8 * (1 + abs(gl[k])), k
    # d/dtheta by differences, with the weights held constant (the stop-gradient of the base step)
    ids_pt, seq, pos, tgt = pt
    l_seq, cnt = seq_losses(enc.mlm_losses(th, ids_pt, seq, pos, tgt), seq, len(ids_pt))
    w = wnet.weights(l_seq, lam)

    def S(t):
        ls, _ = seq_losses(enc.mlm_losses(t, ids_pt, seq, pos, tgt), seq, len(ids_pt))
        return float(np.mean(enc.losses(t, ft[0], ft[1])) + np.mean(w * ls))
    r = CounterRNG(21)
    for k in list(r.integers(1, 12, enc.n)) + [enc.slices["Wmlm"][0] + int(tgt[0]) * enc.d + 1, enc.slices["bmlm"][0] + int(tgt[3]),
                                               enc.slices["Wc"][0], enc.slices["tok_emb"][0]]:
        e = np.zeros(enc.n); e[k] = 1e-6
        fd = (S(th + e) - S(th - e)) / 2e-6
        assert abs(fd - orc.g[k]) < 2e-7 * (1 + abs(orc.g[k])), (k, fd, orc.g[k])


def test_padded_batches_in_the_assembled_base_step():
    """Sequence lengths on both halves of the stacked batch: the base gradient is still the gradient of the scalar base
    loss (directional differences), and it differs from the unpadded one."""
    enc, th, ft, pt, lam = _setup()
    ids_pt, seq, pos, tgt = pt
    ftl = (models.with_lengths(ft[0], np.array([8, 3, 6])), ft[1])
    ptl = (models.with_lengths(ids_pt, np.array([6, 8, 8, 7])), seq, pos, tgt)     # every masked position is a real token
    orc = AuxTaskOracle(enc, th, lam, base_lr=1e-2)
    ref = AuxTaskOracle(enc, th, lam, base_lr=1e-2)
    Lb = orc.base_step(ftl, ptl); ref.base_step(ft, pt)
    assert abs(Lb - orc.base_loss(th, lam, ftl, ptl)) < 1e-12 * abs(Lb)
    assert np.linalg.norm(orc.g - ref.g) > 1e-2 * np.linalg.norm(ref.g)
    l_seq, _ = seq_losses(enc.mlm_losses(th, ptl[0], seq, pos, tgt), seq, 4)
    w = wnet.weights(l_seq, lam)

    def S(t):
        ls, _ = seq_losses(enc.mlm_losses(t, ptl[0], seq, pos, tgt), seq, 4)
        return float(np.mean(enc.losses(t, ftl[0], ftl[1])) + np.mean(w * ls))
    r = CounterRNG(31)
    for k in range(4):
        u = r.normal(k, enc.n); u /= np.linalg.norm(u)
        fd = (S(th + 1e-6 * u) - S(th - 1e-6 * u)) / 2e-6
        assert abs(fd - orc.g @ u) < 1e-7 * (1 + abs(fd)), (k, fd, orc.g @ u)
    # the +- passes see the lengths too
    r1 = orc.meta_grad(ptl, ftl); r0 = orc.meta_grad(pt, ftl)
    assert np.linalg.norm(r1["h"] - r0["h"]) > 1e-3 * np.linalg.norm(r0["h"])


def test_evaluate_aux_is_the_weighted_term_of_the_base_loss():
    enc, th, ft, pt, lam = _setup()
    orc = AuxTaskOracle(enc, th, lam, base_lr=1e-2)
    l_seq, w = orc.evaluate_aux(pt)
    assert abs(orc.base_loss(th, lam, ft, pt) - (np.mean(enc.losses(th, ft[0], ft[1])) + np.mean(w * l_seq))) < 1e-13
    ids_pt, seq, pos, tgt = pt
    l_pos = enc.mlm_losses(th, ids_pt, seq, pos, tgt)
    assert np.allclose(l_seq, [l_pos[seq == i].mean() for i in range(len(ids_pt))], rtol=1e-13)
    assert np.all((w > 0) & (w < 1))


def test_constant_weights_give_plain_multitask_gradient_and_zero_hypergradient_rows():
    """W2 = 0: w = sigmoid(b2) for every sequence, so the base gradient is that of L_ft + sigmoid(b2) mean L_pt, and only
    the rows of dL_base/dlambda that do not vanish with W2 = 0 (W2 itself and b2) are non-zero."""
    enc, th, ft, pt, lam = _setup()
    H = (len(lam) - 1) // 3
    lam[2 * H:3 * H] = 0.0
    orc = AuxTaskOracle(enc, th, lam)
    orc.base_step(ft, pt)
    ids_pt, seq, pos, tgt = pt
    c = 1.0 / (1.0 + np.exp(-lam[-1]))
    cnt = np.bincount(seq, minlength=len(ids_pt)).astype(float)
    n_ft = len(ft[0])
    ids = np.concatenate([ft[0], ids_pt])
    y = np.concatenate([ft[1], np.zeros(len(ids_pt), dtype=ft[1].dtype)])
    _, _, g = enc.loss_grad_mlm(th, ids, y, np.concatenate([np.full(n_ft, 1 / n_ft), np.zeros(len(ids_pt))]), seq + n_ft, pos, tgt,
                                (c / (len(ids_pt) * cnt))[seq])
    assert np.allclose(orc.g, g, rtol=1e-13, atol=1e-16)
    gl = orc.glam(th, pt)
    assert np.all(gl[:2 * H] == 0.0) and np.linalg.norm(gl[2 * H:]) > 0


def test_fd_product_is_the_mixed_partial_times_v_and_meta_step_bookkeeping():
    enc, th, ft, pt, lam = _setup()
    orc = AuxTaskOracle(enc, th, lam, base_lr=1e-2, meta_lr=1e-2, alpha=0.05)
    for _ in range(3):
        orc.base_step(ft, pt)
    meta = (ft[0][:2], ft[1][:2])
    r = orc.meta_grad(pt, meta)
    th0, lam0 = orc.theta.copy(), orc.lam.copy()
    # h = -(d^2 L_base / dlambda dtheta) v: four-point difference of the scalar base loss
    v, eps = r["v"], r["eps"]
    d = 1e-5
    for k in range(0, len(lam), 3):
        e = np.zeros(len(lam)); e[k] = d
        mixed = (orc.base_loss(th0 + eps * v, lam0 + e, ft, pt) - orc.base_loss(th0 + eps * v, lam0 - e, ft, pt)
                 - orc.base_loss(th0 - eps * v, lam0 + e, ft, pt) + orc.base_loss(th0 - eps * v, lam0 - e, ft, pt)) / (4 * d * eps)
        assert abs(-mixed - r["h"][k]) < 1e-5 * (1e-12 + np.max(np.abs(r["h"]))), (k, -mixed, r["h"][k])
    # the direct gradient is that of the mean finetuning loss on the meta batch
    _, gm = enc.loss_grad(th0, meta[0], meta[1], np.full(2, 0.5))
    assert np.allclose(r["g_meta"], gm, rtol=1e-13, atol=1e-18)
    r2 = orc.meta_step(pt, meta)
    assert np.allclose(r2["h"], r["h"]) and orc.meta_t == 1
    assert np.allclose(orc.theta, th0 - eps * v) and not np.array_equal(orc.lam, lam0)
