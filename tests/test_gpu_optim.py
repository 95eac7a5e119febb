"""GPU parity of roast_optim_step against the numpy float64 oracle, through the C-ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2207_10702_amd import workloads as wl  # noqa: F401  (same import set as the other GPU tests)
from tests.util import rel_err, to_dev

pytestmark = pytest.mark.gpu
TOL = 2e-6     # a handful of fp32 operations per element


def _run(roast, kind, n, steps, wd, shadow):
    rng = np.random.default_rng(n + kind)
    M0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    grads = [(rng.standard_normal(n) * s).astype(np.float32) for s in (1.0, 0.3, 2.0, 1e-3)][:steps]
    M = to_dev(M0.copy())
    s1 = torch.zeros(n, dtype=torch.float32, device="cuda")
    s2 = torch.zeros(n, dtype=torch.float32, device="cuda")
    Mb = torch.zeros(roast.roast_m_shadow_bytes(n) // 2, dtype=torch.bfloat16, device="cuda") if shadow else None
    Mo = M0.astype(np.float64)
    o1, o2 = np.zeros(n), np.zeros(n)
    # the descriptor carries fp32 hyper-parameters: the oracle gets exactly those values
    f32 = lambda v: float(np.float32(v))
    lr, b1, b2, wd = f32(0.05), f32(0.9), f32(0.999), f32(wd)
    eps = f32(1e-10 if kind == roast.ROAST_OPT_ADAGRAD else 1e-8)
    for t, g in enumerate(grads, start=1):
        dM = to_dev(g.copy())
        d = roast.optim_desc(kind, lr, wd, b1, b2, eps, step=t, zero_grad=(t % 2 == 1))
        roast.roast_optim_step(d, M, dM, s1, s2, Mb)
        if kind == roast.ROAST_OPT_SGD:
            Mo = oracle.optim.sgd(Mo, g, lr, wd)
        elif kind == roast.ROAST_OPT_ADAGRAD:
            Mo, o1 = oracle.optim.adagrad(Mo, g, o1, lr, wd, eps)
        else:
            Mo, o1, o2 = oracle.optim.adam(Mo, g, o1, o2, t, lr, b1, b2, eps, wd)
        torch.cuda.synchronize()
        # the gradient is cleared exactly when asked to
        if t % 2 == 1:
            assert not bool(dM.any())
        else:
            assert np.array_equal(dM.cpu().numpy(), g)
    got = M.cpu().numpy()
    assert rel_err(got.astype(np.float64), Mo) <= TOL
    if kind != roast.ROAST_OPT_SGD:
        assert rel_err(s1.cpu().numpy().astype(np.float64), o1) <= TOL
    if kind == roast.ROAST_OPT_ADAM:
        assert rel_err(s2.cpu().numpy().astype(np.float64), o2) <= TOL
    if shadow:
        # the refreshed shadow is bit-identical to a shadow made from the new M
        assert torch.equal(Mb, roast.roast_m_shadow_bf16(M))


@pytest.mark.parametrize("n", [1, 3, 4, 1023, 1024, 47185, 1_280_000])
@pytest.mark.parametrize("kind", [0, 1, 2])
def test_optim_step_matches_oracle(roast, kind, n):
    _run(roast, kind, n, steps=4, wd=0.01 if n % 2 else 0.0, shadow=(n != 3))


def test_optim_step_then_mm_uses_the_refreshed_shadow(roast):
    """After a step that refreshes the shadow, the bf16 forward must equal the one from a fresh shadow."""
    rng = np.random.default_rng(8)
    I, H, O, Z, m = 256, 128, 256, 64, 20000
    h = wl.draw_hash(rng)
    d = roast.mm_desc(H, O, Z, Z, m, 1, 1.0, h)
    M = to_dev(wl.draw_m(rng, m, ("normal", 0.02)))
    X = to_dev(wl.draw_act(rng, I, H, "bf16"))
    dM = to_dev(rng.standard_normal(m).astype(np.float32))
    Mb = roast.roast_m_shadow_bf16(M)
    roast.roast_optim_step(roast.optim_desc(roast.ROAST_OPT_SGD, 0.1), M, dM, M_bf16=Mb)
    Y1 = roast.roast_mm_fwd(d, X, M, M_bf16=Mb)
    Y2 = roast.roast_mm_fwd(d, X, M)
    assert torch.equal(Y1, Y2)
