"""GPU parity of the per-element sign variant (use_sign = 2) against the oracle: ROAST-MM forward,
dX, dM (atomic and deterministic) in fp32 and bf16 -- on shapes the tiled matrix-core kernels would
otherwise take (bf16: their element-wise instantiations run instead; fp32: the vector-ALU kernels)
and on shapes only the generic kernels take -- and the lookup, its gradient and the pooled lookup."""
import numpy as np
import pytest

import oracle
from paper_2207_10702_amd import workloads as wl
from tests.util import BF16_TOL, F32_TOL, rel_err, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def hash2(rng):
    h = wl.draw_hash(rng, use_sign=True, align=1)
    h["use_sign"] = 2
    return h


@pytest.mark.parametrize("dtype,tol", [("f32", F32_TOL), ("bf16", BF16_TOL)])
@pytest.mark.parametrize("shape", [(70, 100, 130, 7, 5, 900), (300, 128, 320, 64, 64, 20000), (64, 256, 256, 32, 32, 4096),
                                   (37, 50, 41, 1, 1, 300)])
def test_mm_per_element_sign(roast, shape, dtype, tol):
    I, H, O, Z1, Z2, m = shape
    rng = np.random.default_rng(500 + I)
    h = hash2(rng)
    M = wl.draw_m(rng, m, ("normal", 0.05))
    X, dY = wl.draw_act(rng, I, H, dtype), wl.draw_act(rng, I, O, dtype)
    lam = np.float32(0.6)
    d = roast.mm_desc(H, O, Z1, Z2, m, 4, lam, h)
    Md, Xd, dYd = to_dev(M), to_dev(X), to_dev(dY)
    wsz = max(roast.roast_mm_fwd_workspace(d, Xd.dtype, I), roast.roast_mm_bwd_dx_workspace(d, Xd.dtype, I),
              roast.roast_mm_bwd_dM_workspace(d, I, roast.ROAST_REDUCE_ATOMIC), roast.roast_mm_bwd_dM_workspace_f32(d, I))
    assert wsz == 0                                        # no workspace helps these sizes in this variant
    shadow = roast.roast_m_shadow_bf16(Md) if dtype == "bf16" else None
    Y = roast.roast_mm_fwd(d, Xd, Md, M_bf16=shadow)
    dX = roast.roast_mm_bwd_dx(d, dYd, Md, M_bf16=shadow)
    dM = torch.zeros(m, dtype=torch.float32, device="cuda")
    roast.roast_mm_bwd_dM(d, Xd, dYd, dM)
    det = roast.ROAST_REDUCE_DETERMINISTIC
    ws = torch.empty(max(roast.roast_mm_bwd_dM_workspace(d, I, det), 1), dtype=torch.uint8, device="cuda")
    dM_det = torch.zeros(m, dtype=torch.float32, device="cuda")
    roast.roast_mm_bwd_dM(d, Xd, dYd, dM_det, det, ws)
    W = oracle.materialize_w(h, 4, H, O, Z1, Z2, float(lam), M)
    assert np.mean(np.sign(W) != np.sign(oracle.materialize_w(dict(h, use_sign=0), 4, H, O, Z1, Z2, float(lam), M))) > 0.3
    Xo, dYo = wl.act_as_f64(X), wl.act_as_f64(dY)
    assert rel_err(to_host_f64(Y), oracle.mm_fwd(Xo, W)) <= tol
    assert rel_err(to_host_f64(dX), oracle.mm_bwd_dx(dYo, W)) <= tol
    ref = oracle.mm_bwd_dm(h, 4, Z1, Z2, m, float(lam), Xo, dYo)
    assert rel_err(to_host_f64(dM), ref) <= tol
    assert rel_err(to_host_f64(dM_det), ref) <= tol
    off, sgn = roast.roast_tile_index_device(d)
    eoff, esgn = oracle.tile_index(h, 4, H, O, Z1, Z2, m)
    assert np.array_equal(off.cpu().numpy(), eoff) and np.array_equal(sgn.cpu().numpy(), esgn) and np.all(esgn == 1)


@pytest.mark.parametrize("D,Z,m,N", [(128, 32, 20000, 3000), (10, 4, 60, 333), (128, 32, 300000, 40000)])
def test_lookup_per_element_sign(roast, D, Z, m, N):
    rng = np.random.default_rng(D + N + 2)
    h = hash2(rng)
    M = wl.draw_m(rng, m, ("normal", 0.02))
    rows = rng.integers(0, 50, size=N)
    rows[::3] = rng.integers(0, 1 << 33, size=rows[::3].size)
    tables = rng.integers(0, 4, size=N).astype(np.uint32)
    dOut = rng.standard_normal((N, D), dtype=np.float32)
    lam = np.float32(0.8)
    d = roast.embed_desc(D, Z, m, lam, h)
    rd, td = to_dev(rows), to_dev(tables)
    out = roast.roast_embed_fwd(d, rd, td, to_dev(M))
    ref_out = oracle.embed_fwd(h, D, Z, float(lam), rows, tables, M)
    assert rel_err(to_host_f64(out), ref_out) <= 1e-7
    assert np.mean(np.sign(ref_out) != np.sign(oracle.embed_fwd(dict(h, use_sign=0), D, Z, float(lam), rows, tables, M))) > 0.3
    ref_dM = oracle.embed_bwd(h, D, Z, m, float(lam), rows, tables, dOut)
    for mode in (roast.ROAST_REDUCE_ATOMIC, roast.ROAST_REDUCE_DETERMINISTIC):
        ws = torch.empty(max(roast.roast_embed_bwd_workspace(d, N, mode), 1), dtype=torch.uint8, device="cuda")
        dM = torch.zeros(m, dtype=torch.float32, device="cuda")
        roast.roast_embed_bwd(d, rd, td, to_dev(dOut), dM, mode, ws)
        assert rel_err(to_host_f64(dM), ref_dM) <= F32_TOL, mode
    bag_off = np.arange(0, N + 1, 3 if N % 3 == 0 else 1, dtype=np.int64)
    pooled = roast.roast_embed_bag_fwd(d, rd, td, to_dev(bag_off), to_dev(M))
    assert rel_err(to_host_f64(pooled), oracle.embed_bag_fwd(h, D, Z, float(lam), rows, tables, bag_off, M)) <= F32_TOL


def test_unknown_sign_mode_is_rejected(roast):
    h = wl.draw_hash(np.random.default_rng(1))
    h["use_sign"] = 3
    d = roast.mm_desc(64, 64, 8, 8, 1000, 0, 1.0, h)
    with pytest.raises(roast.RoastError) as e:
        roast.roast_tile_index(d)
    assert e.value.status == roast.ROAST_ERR_RANGE
