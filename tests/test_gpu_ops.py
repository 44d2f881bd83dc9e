"""Per-kernel parity through the op-level C ABI (include/sama_ops.h): the elementwise chain against the oracle's
formulas on random arrays with ragged lengths, the bf16 GEMM in its three operand storages against a float64
matmul, and run-to-run bit stability."""
import numpy as np
import pytest
import torch
from datagen import CounterRNG, round_to_bf16
from harness import rel_l2
from oracle import optim, sama_core

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a, dtype=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(a), device=DEV).to(dtype).contiguous()


def _bf16_bits_to_f64(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("wd", [0.0, 0.25])
@pytest.mark.parametrize("n,n16", [(1, 1), (7, 5), (4096 * 1024 + 3, 4096 * 1024 - 6), (1000003, 0)])
def test_adam_kernel(n, n16, wd):
    from paper_2310_05674_amd import binding as B
    r = CounterRNG(100 + n % 97)
    g = r.normal(1, n); m = 0.1 * r.normal(2, n); v = (0.3 * r.normal(3, n)) ** 2; th = 0.05 * r.normal(4, n)
    g32, m32, v32, th32 = (x.astype(np.float32) for x in (g, m, v, th))
    tg, tm, tv, tt = _dev(g32), _dev(m32), _dev(v32), _dev(th32)
    t16 = torch.zeros(max(n16, 1), dtype=torch.bfloat16, device=DEV)
    B.op_adam(tg, tm, tv, tt, t16 if n16 else None, n16, 7, 1e-3, 0.9, 0.999, 1e-8, wd)
    ge = g32.astype(np.float64) + wd * th32.astype(np.float64)   # the L2 term goes in front of the solver
    th2, m2, v2 = optim.adam_update(th32.astype(np.float64), m32.astype(np.float64), v32.astype(np.float64),
                                    ge, 7, 1e-3, 0.9, 0.999, 1e-8)
    if wd == 0.0:
        assert np.array_equal(tg.cpu().numpy(), g32)              # only read
    else:
        assert rel_l2(tg.cpu().numpy(), ge) < 1e-6                # kept for the adaptation
    assert rel_l2(tm.cpu().numpy(), m2) < 1e-6 and rel_l2(tv.cpu().numpy(), v2) < 1e-6
    upd = np.abs(th2 - th32.astype(np.float64))
    assert np.all(np.abs(tt.cpu().numpy() - th2) <= 1e-5 * (upd + np.abs(th2)) + 1e-9)
    # the step itself: 1e-5 for the kernel's fp32 arithmetic plus what storing theta in fp32 costs (half an ulp per element,
    # which on a single element is already 5e-6 of a step of lr = 1e-3)
    half_ulp = 0.5 * np.spacing(np.abs(th2).astype(np.float32)).astype(np.float64)
    assert rel_l2(tt.cpu().numpy() - th32, th2 - th32) < 1e-5 + np.linalg.norm(half_ulp) / np.linalg.norm(th2 - th32)
    if n16:
        # bit-exact: the working copy is the round-to-nearest-even of the fp32 master the kernel just wrote
        want = round_to_bf16(tt.cpu().numpy()[:n16].astype(np.float64))
        assert np.array_equal(_bf16_bits_to_f64(t16[:n16]), want)


@pytest.mark.parametrize("n", [5, 2 ** 20 + 1, 7 * 2 ** 20 + 13])
def test_adapt_norm_kernel(n):
    from paper_2310_05674_amd import binding as B
    r = CounterRNG(200 + n % 89)
    g = r.normal(1, n); gm = r.normal(4, n)
    m0 = 0.2 * r.normal(2, n); v0 = (0.4 * r.normal(3, n)) ** 2
    m = 0.9 * m0 + 0.1 * g; v = 0.999 * v0 + 0.001 * g * g
    v[::11] = 0.0; m[::11] = 0.0; g[::11] = 0.0                        # zero-history elements
    g32, m32, v32, gm32 = (x.astype(np.float32) for x in (g, m, v, gm))
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    partial = torch.zeros(65536, dtype=torch.float64, device=DEV)
    scal = torch.zeros(4, dtype=torch.float32, device=DEV); status = torch.full((1,), 7, dtype=torch.int64, device=DEV)
    B.op_adapt_norm(_dev(g32), _dev(m32), _dev(v32), _dev(gm32), out, partial, 5, 1e-3, 0.9, 0.999, 1e-8, 0.5, scal, status)
    D = optim.adam_adaptation(g32.astype(np.float64), m32.astype(np.float64), v32.astype(np.float64), 5, 1e-3, 0.9, 0.999, 1e-8)
    want = sama_core.perturbation(D, gm32.astype(np.float64))
    got = out.cpu().numpy()
    assert np.all(got[::11] == 0.0)
    assert rel_l2(got, want) < 5e-5          # fp32 cancellation in (1-b1) v' - (1-b2) m' g; the workload bar is 1e-4
    eps = sama_core.step_size(want, 0.5)
    s = scal.cpu().numpy()
    assert abs(s[0] - eps) < 5e-5 * eps and abs(s[1] - np.linalg.norm(want)) < 5e-5 * np.linalg.norm(want)
    assert int(status.item()) == 0
    # run-to-run bit stability of the norm (fixed-order reduction)
    scal2 = torch.zeros(4, dtype=torch.float32, device=DEV)
    B.op_adapt_norm(_dev(g32), _dev(m32), _dev(v32), _dev(gm32), out, partial, 5, 1e-3, 0.9, 0.999, 1e-8, 0.5, scal2, status)
    assert torch.equal(scal, scal2)


def test_adapt_norm_degenerate():
    from paper_2310_05674_amd import binding as B
    n = 1000
    z = torch.zeros(n, dtype=torch.float32, device=DEV)
    out = torch.empty(n, dtype=torch.float32, device=DEV); partial = torch.zeros(65536, dtype=torch.float64, device=DEV)
    scal = torch.ones(4, dtype=torch.float32, device=DEV); status = torch.zeros(1, dtype=torch.int64, device=DEV)
    B.op_adapt_norm(z, z, z, torch.ones_like(z), out, partial, 3, 1e-3, 0.9, 0.999, 1e-8, 1.0, scal, status)
    assert float(scal[0]) == 0.0 and int(status.item()) == 1


@pytest.mark.parametrize("n16", [3, 4096 * 1024 + 5])
def test_perturb_and_nudge_kernels(n16):
    from paper_2310_05674_amd import binding as B
    n = n16 + 9
    r = CounterRNG(300 + n16 % 83)
    th = (0.02 * r.normal(1, n)).astype(np.float32); v = r.normal(2, n).astype(np.float32)
    eps = np.float32(3.1e-6)
    tth, tv, te = _dev(th), _dev(v), _dev(np.array([eps], dtype=np.float32))
    lp = torch.zeros(n16, dtype=torch.bfloat16, device=DEV); lm = torch.zeros(n16, dtype=torch.bfloat16, device=DEV)
    B.op_perturb_lo(tth, tv, te, lp, lm, n16)
    hi = round_to_bf16(th[:n16].astype(np.float64))
    th64, v64 = th.astype(np.float64), v.astype(np.float64)
    rec = {}
    for lo, sgn in ((lp, 1.0), (lm, -1.0)):
        want = th64[:n16] + sgn * float(eps) * v64[:n16]                  # theta +- eps v (Eq. 5)
        got = hi + _bf16_bits_to_f64(lo)
        rec[sgn] = got
        # lo is the bf16 rounding of (theta +- eps v) - hi: hi + lo is off by at most 2^-8 of that residual, i.e.
        # about 2^-17 of theta, far below the perturbation itself
        assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want - hi) + 2.0 ** -22 * np.abs(want) + 1e-30)
    assert rel_l2(rec[1.0] - rec[-1.0], 2.0 * float(eps) * v64[:n16]) < 2e-2
    t16 = torch.zeros(n16, dtype=torch.bfloat16, device=DEV)
    B.op_nudge(tth, tv, te, t16, n16)
    want = sama_core.nudge(th64, v64, float(eps))
    got = tth.cpu().numpy()
    assert np.max(np.abs(got - want)) < 1e-7 * np.max(np.abs(want))
    assert np.array_equal(_bf16_bits_to_f64(t16), round_to_bf16(got[:n16].astype(np.float64)))


CASES = [  # M, N, K, a_trans, b_trans, split
    (256, 128, 64, False, True, False), (136, 200, 192, False, True, True), (640, 328, 128, False, False, False),
    (264, 136, 320, False, False, True), (200, 392, 256, True, False, False), (2048, 3072, 1024, False, True, False),
    (1024, 4096, 2048, True, False, False), (2048, 1024, 3072, False, False, True)]


@pytest.mark.parametrize("M,N,K,a_trans,b_trans,split", CASES)
def test_gemm_bf16(M, N, K, a_trans, b_trans, split):
    """Every block tile (forced in turn; the hi + lo tiles fall back to the heuristic on single-term problems) and the heuristic against numpy float64 on bf16-representable operands;
    several tiles and ragged edges in M and N."""
    import ctypes
    from paper_2310_05674_amd import binding as B
    r = CounterRNG(400 + M + N + K)
    A = round_to_bf16(r.normal(1, M * K)).reshape((K, M) if a_trans else (M, K))
    Bm = round_to_bf16(r.normal(2, N * K)).reshape((N, K) if b_trans else (K, N))
    B2 = round_to_bf16(0.004 * r.normal(3, N * K)).reshape(Bm.shape) if split else None
    bias = r.normal(4, N).astype(np.float32)
    Af = A.T if a_trans else A
    Bf = (Bm + (B2 if split else 0.0)); Bf = Bf.T if b_trans else Bf
    want = Af @ Bf + bias.astype(np.float64)
    tA, tB = _dev(A, torch.bfloat16), _dev(Bm, torch.bfloat16)
    tB2 = _dev(B2, torch.bfloat16) if split else None
    tbias = _dev(bias)
    L = B.load_library()
    outs = []
    for shape in (1, 2, 3, 4, 5, 6, 7, 11, 12, 13, 14, 15, 0):
        L.sama_dev_gemm_shape(ctypes.c_int32(shape))
        o32 = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        o16 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        B.op_gemm_bf16(tA, tB, a_trans=a_trans, b_trans=b_trans, B2=tB2, bias=tbias, out32=o32, out16=o16)
        got = o32.cpu().numpy()
        assert np.all(np.isfinite(got))
        assert np.max(np.abs(got - want)) < 2e-5 * np.sqrt(K) * (1 + np.max(np.abs(want))), shape
        assert rel_l2(got, want) < 1e-5
        assert np.array_equal(_bf16_bits_to_f64(o16), round_to_bf16(got.astype(np.float64)))
        outs.append(got)
    # every tile of a class (single-term / hi + lo) accumulates an output element in the same order: same bits
    classes = ((1, 2, 3, 4, 5, 6, 7, 0), ()) if not split else ((11, 12, 13, 14, 15, 0), (1, 2, 3, 4, 5, 6, 7))
    order = (1, 2, 3, 4, 5, 6, 7, 11, 12, 13, 14, 15, 0)
    for cls in classes:
        ref = [outs[order.index(sid)] for sid in cls]
        for o in ref[1:]:
            assert np.array_equal(o, ref[0])
    L.sama_dev_gemm_shape(ctypes.c_int32(0))
    o32b = torch.empty((M, N), dtype=torch.float32, device=DEV)
    B.op_gemm_bf16(tA, tB, a_trans=a_trans, b_trans=b_trans, B2=tB2, bias=tbias, out32=o32b)
    assert np.array_equal(o32b.cpu().numpy(), outs[-1])                    # bit-stable from run to run


def test_gemm_rejects_unsupported_shapes():
    from paper_2310_05674_amd import binding as B
    A = torch.zeros((64, 96), dtype=torch.bfloat16, device=DEV); Bm = torch.zeros((64, 96), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((64, 64), dtype=torch.float32, device=DEV)
    with pytest.raises(B.SamaError):
        B.op_gemm_bf16(A, Bm, out32=out)                                   # K = 96 is not a multiple of 64
    A = torch.zeros((60, 64), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.SamaError):
        B.op_gemm_bf16(A, torch.zeros((64, 64), dtype=torch.bfloat16, device=DEV), out32=torch.zeros((60, 64), device=DEV))


@pytest.mark.parametrize("a_trans,b_trans,split", [(False, True, True), (False, True, False), (True, False, False), (False, False, True)])
def test_gemm_bf16_batch(a_trans, b_trans, split):
    """Several problems of different shapes in one launch (the stacked +- passes, a layer's weight gradients): every
    problem against numpy float64, and bit-identical to the same problem launched alone."""
    from paper_2310_05674_amd import binding as B
    shapes = [(264, 136, 128), (520, 392, 192), (128, 1024, 64), (1032, 72, 256)]
    As, Bs, B2s, outs, wants = [], [], [], [], []
    for i, (M, N, K) in enumerate(shapes):
        r = CounterRNG(900 + 7 * i + M)
        A = round_to_bf16(r.normal(1, M * K)).reshape((K, M) if a_trans else (M, K))
        Bm = round_to_bf16(r.normal(2, N * K)).reshape((N, K) if b_trans else (K, N))
        B2 = round_to_bf16(0.004 * r.normal(3, N * K)).reshape(Bm.shape) if split else None
        Af = A.T if a_trans else A
        Bf = Bm + (B2 if split else 0.0); Bf = Bf.T if b_trans else Bf
        wants.append(Af @ Bf)
        As.append(_dev(A, torch.bfloat16)); Bs.append(_dev(Bm, torch.bfloat16))
        if split:
            B2s.append(_dev(B2, torch.bfloat16))
        outs.append(torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV))
    B.op_gemm_bf16_batch(As, Bs, outs, a_trans=a_trans, b_trans=b_trans, B2s=B2s if split else None)
    for i, (M, N, K) in enumerate(shapes):
        got = outs[i].cpu().numpy()
        assert np.all(np.isfinite(got)), i
        assert rel_l2(got, wants[i]) < 1e-5, i
    # the same problems as single launches with the batch's tile forced: identical bits (same tile => same summation order)
    alone = []
    for i in range(len(shapes)):
        o = torch.empty_like(outs[i])
        B.op_gemm_bf16_batch([As[i]], [Bs[i]], [o], a_trans=a_trans, b_trans=b_trans, B2s=[B2s[i]] if split else None)
        alone.append(o)
    again = [torch.empty_like(o) for o in outs]
    B.op_gemm_bf16_batch(As, Bs, again, a_trans=a_trans, b_trans=b_trans, B2s=B2s if split else None)
    for i in range(len(shapes)):
        assert torch.equal(again[i], outs[i]), i          # bit-stable from launch to launch
        assert rel_l2(alone[i].cpu().numpy(), wants[i]) < 1e-5, i


def test_gemm_bf16_batch_rejects_mixed():
    from paper_2310_05674_amd import binding as B
    a = torch.zeros((64, 64), dtype=torch.bfloat16, device=DEV)
    o = torch.zeros((64, 64), dtype=torch.float32, device=DEV)
    with pytest.raises(B.SamaError):
        B.op_gemm_bf16_batch([a] * 5, [a] * 5, [o] * 5)                 # more than four problems
    bad = torch.zeros((64, 72), dtype=torch.bfloat16, device=DEV)       # K = 72 is not a multiple of 64
    with pytest.raises(B.SamaError):
        B.op_gemm_bf16_batch([bad], [bad], [o])
