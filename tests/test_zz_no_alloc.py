"""The allocation-free lookup gradient (roast_embed_bwd_noalloc: workspace in the library's static
device array) against roast_embed_bwd with a caller workspace, through the C-ABI: two calls in a row
that share the array, the second with a smaller batch (a different list layout over the first call's
leftovers), in both reduce modes; and the size limit."""
import numpy as np
import pytest

from paper_2207_10702_amd import workloads as wl
from tests.util import F32_TOL, rel_err, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

LIMIT = 64 << 20


def draw(rng, N, D):
    rows = rng.integers(0, 1 << 33, N).astype(np.int64)
    hot = rng.integers(0, 200, N).astype(np.int64)
    rows = np.where(rng.random(N) < 0.4, hot, rows)          # repeated ids: slots with many addends
    tables = rng.integers(0, 26, N).astype(np.uint32)
    dOut = rng.standard_normal((N, D)).astype(np.float32)
    return to_dev(rows), to_dev(tables), to_dev(dOut)


@pytest.mark.parametrize("mode_name", ["atomic", "deterministic"])
def test_noalloc_gradient_matches_workspace_gradient_on_two_calls_in_a_row(roast, mode_name):
    mode = roast.ROAST_REDUCE_ATOMIC if mode_name == "atomic" else roast.ROAST_REDUCE_DETERMINISTIC
    rng = np.random.default_rng(64)
    D, Z, m_size = 128, 32, 1_280_000
    d = roast.embed_desc(D, Z, m_size, np.float32(0.8), wl.draw_hash(rng, use_sign=True, align=1))
    for N in (120_000, 30_011):                               # the second call is smaller and ragged
        need = roast.roast_embed_bwd_workspace(d, N, mode)
        assert 0 < need <= LIMIT                              # the scratch path, not the direct atomics
        rows, tables, dOut = draw(rng, N, D)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        ref = torch.zeros(m_size, dtype=torch.float32, device="cuda")
        roast.roast_embed_bwd(d, rows, tables, dOut, ref, mode, ws)
        got = torch.zeros(m_size, dtype=torch.float32, device="cuda")
        roast.roast_embed_bwd_noalloc(d, rows, tables, dOut, got, mode)
        torch.cuda.synchronize()
        assert float(ref.abs().sum().item()) > 0
        if mode == roast.ROAST_REDUCE_DETERMINISTIC:
            assert torch.equal(got, ref)                      # order-independent sums: the same bits
        else:
            assert rel_err(to_host_f64(got), to_host_f64(ref)) <= F32_TOL


def test_noalloc_gradient_refuses_what_does_not_fit(roast):
    rng = np.random.default_rng(65)
    D, Z, m_size, N = 128, 32, 1_280_000, 2_000_000
    d = roast.embed_desc(D, Z, m_size, 1.0, wl.draw_hash(rng))
    assert roast.roast_embed_bwd_workspace(d, N, roast.ROAST_REDUCE_ATOMIC) > LIMIT
    rows = torch.zeros(N, dtype=torch.int64, device="cuda")
    tables = torch.zeros(N, dtype=torch.int32, device="cuda")
    dOut = torch.zeros((N, D), dtype=torch.float32, device="cuda")
    dM = torch.zeros(m_size, dtype=torch.float32, device="cuda")
    with pytest.raises(roast.RoastError) as e:
        roast.roast_embed_bwd_noalloc(d, rows, tables, dOut, dM)
    assert e.value.status == roast.ROAST_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert not dM.any()                                        # nothing was launched
    # a small batch needs no scratch at all (direct atomics) and is served like roast_embed_bwd serves it
    n = 500
    r, t, g = draw(rng, n, D)
    a = torch.zeros(m_size, dtype=torch.float32, device="cuda")
    b = torch.zeros(m_size, dtype=torch.float32, device="cuda")
    roast.roast_embed_bwd_noalloc(d, r, t, g, a)
    roast.roast_embed_bwd(d, r, t, g, b)
    torch.cuda.synchronize()
    assert rel_err(to_host_f64(a), to_host_f64(b)) <= F32_TOL
