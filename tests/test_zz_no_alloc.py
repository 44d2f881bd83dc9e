"""The allocation-free form of the adaptation + step-size op (sama_op_adapt_norm_static, for callers that cannot
allocate or pass device scratch) against sama_op_adapt_norm with a caller-owned scratch buffer, through the C ABI:
two calls in a row on one GPU, the second on a smaller input, so that what the first call left in the library's
static scratch must not leak into the second.  Bit-exact: both forms run the same kernels in the same launch shape.
The oracle's formula is checked too (the bar of the op test: 5e-5)."""
import numpy as np
import pytest
import torch
from datagen import CounterRNG
from harness import rel_l2
from oracle import optim, sama_core

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(n, seed):
    r = CounterRNG(seed)
    g = r.normal(1, n); gm = r.normal(4, n)
    m = 0.9 * 0.2 * r.normal(2, n) + 0.1 * g
    v = 0.999 * (0.4 * r.normal(3, n)) ** 2 + 0.001 * g * g
    v[::13] = 0.0; m[::13] = 0.0; g[::13] = 0.0                        # zero-history elements
    return tuple(torch.as_tensor(x.astype(np.float32), device=DEV) for x in (g, m, v, gm))


def test_static_scratch_matches_caller_scratch_on_two_calls_in_a_row():
    from paper_2310_05674_amd import binding as B
    hyp = (5, 1e-3, 0.9, 0.999, 1e-8, 0.5)
    for n, seed in ((9 * 2 ** 20 + 7, 401), (3 * 4096 + 5, 402)):       # 2305 partials, then 4: the second call is smaller
        g, m, v, gm = _inputs(n, seed)
        ref = torch.empty(n, dtype=torch.float32, device=DEV); got = torch.empty_like(ref)
        partial = torch.zeros(65536, dtype=torch.float64, device=DEV)
        s_ref = torch.zeros(4, dtype=torch.float32, device=DEV); s_got = torch.zeros_like(s_ref)
        st_ref = torch.full((1,), 7, dtype=torch.int64, device=DEV); st_got = torch.full((1,), 9, dtype=torch.int64, device=DEV)
        B.op_adapt_norm(g, m, v, gm, ref, partial, *hyp, s_ref, st_ref)
        B.op_adapt_norm_static(g, m, v, gm, got, *hyp, s_got, st_got)
        torch.cuda.synchronize()
        assert torch.equal(got, ref), n
        assert torch.equal(s_got, s_ref) and int(st_got.item()) == int(st_ref.item()) == 0, n
        D = optim.adam_adaptation(*(x.cpu().numpy().astype(np.float64) for x in (g, m, v)), *hyp[:-1])
        want = sama_core.perturbation(D, gm.cpu().numpy().astype(np.float64))
        assert rel_l2(got.cpu().numpy(), want) < 5e-5
        eps = sama_core.step_size(want, hyp[-1])
        assert abs(float(s_got[0]) - eps) < 5e-5 * eps


def test_static_scratch_rejects_sizes_beyond_its_maximum():
    from paper_2310_05674_amd import binding as B
    z = torch.zeros(8, dtype=torch.float32, device=DEV)
    s = torch.zeros(4, dtype=torch.float32, device=DEV); st = torch.zeros(1, dtype=torch.int64, device=DEV)
    with pytest.raises(B.SamaError) as e:       # the size check comes first: nothing is launched, nothing is read
        B.op_adapt_norm_static(z, z, z, z, z, 5, 1e-3, 0.9, 0.999, 1e-8, 0.5, s, st, n=(1 << 29) + 1)
    assert e.value.code == 1 and "SAMA_OP_STATIC_MAX_N" in str(e.value)
