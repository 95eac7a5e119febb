"""GPU parity of the fp32 products run on the bf16 matrix cores (three bfloat16 planes per operand,
six plane products): same oracle and the same fp32 bar (1e-5 max relative error per tensor) as the
vector-ALU fp32 kernels, on shapes that span several workgroup tiles with ragged edges, small and
large batches (split contraction), strided rows, and values across many binades."""
import numpy as np
import pytest

import oracle
from paper_2207_10702_amd import workloads as wl
from tests.util import F32_TOL, rel_err, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

# (I, H, O, Z1, Z2, |M|)
SHAPES = [
    (300, 128, 320, 64, 64, 20000),
    (513, 256, 128, 128, 128, 40000),      # one row past two 256-row blocks
    (1000, 64, 576, 64, 64, 4096),         # |M| == one tile
    (700, 640, 72, 64, 8, 5000),           # narrow hash tiles, ragged columns; dX contracts over 72 = 64 + 8
    (300, 256, 256, 32, 32, 4096),         # hash tiles half the 64-deep step (config 1's tiling)
    (260, 128, 192, 16, 8, 9000),          # 16 x 8 tiles, several per 32 x 32 accumulator block
    (64, 2048, 256, 64, 64, 50000),        # small batch: split contraction, fp32 partial sums
    (2100, 256, 128, 64, 64, 30000),       # long batch: dM contraction split over workgroups
]


def ws_tensor(nbytes):
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("pad", [0, 4, 3])      # 3: rows not 16-byte aligned (scalar pre-pass; forward / dX fall back)
def test_f32_plane_products_match_oracle(roast, shape, pad):
    I, H, O, Z1, Z2, m = shape
    rng = np.random.default_rng(4000 + I + pad)
    M = wl.draw_m(rng, m, ("normal", 0.05))
    # activations over ~12 binades, so that the low planes matter
    X = (rng.standard_normal((I, H)) * np.exp2(rng.integers(-6, 6, size=(I, H)))).astype(np.float32)
    dY = (rng.standard_normal((I, O)) * np.exp2(rng.integers(-6, 6, size=(I, O)))).astype(np.float32)
    h = wl.draw_hash(rng, use_sign=True, align=1)
    lam = np.float32(0.37)
    d = roast.mm_desc(H, O, Z1, Z2, m, 2, lam, h)
    Md = to_dev(M)
    Xd = torch.zeros((I, H + pad), dtype=torch.float32, device="cuda")[:, :H]
    Xd.copy_(to_dev(X))
    dYd = torch.zeros((I, O + pad), dtype=torch.float32, device="cuda")[:, :O]
    dYd.copy_(to_dev(dY))
    nf = roast.roast_mm_fwd_workspace(d, torch.float32, I)
    nx = roast.roast_mm_bwd_dx_workspace(d, torch.float32, I)
    nm = roast.roast_mm_bwd_dM_workspace_f32(d, I)
    assert nf > 0                                    # every shape here is covered by the forward kernel
    assert (nx > 0) == (Z2 % 8 == 0) and (nm > 0) == (Z1 % 4 == 0)
    wf, wx, wm = ws_tensor(nf), ws_tensor(nx), ws_tensor(nm)
    outs = []
    planes = roast.roast_m_planes_bf16(Md)             # made once, or rebuilt per call in the workspace: same bits
    for rep in range(2):
        for w in (wf, wx, wm):
            w.fill_(0xFF)
        Y = torch.full((I, O + pad), 7.0, dtype=torch.float32, device="cuda")[:, :O]
        dX = torch.full((I, H + pad), 7.0, dtype=torch.float32, device="cuda")[:, :H]
        roast.roast_mm_fwd(d, Xd, Md, Y, ws=wf, M_bf16=planes if rep == 0 else None)
        roast.roast_mm_bwd_dx(d, dYd, Md, dX, ws=wx, M_bf16=planes if rep == 0 else None)
        outs.append((Y, dX))
    dM = torch.zeros(m, dtype=torch.float32, device="cuda")
    roast.roast_mm_bwd_dM(d, Xd, dYd, dM, roast.ROAST_REDUCE_ATOMIC, wm)
    torch.cuda.synchronize()
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    if pad:
        assert torch.all(outs[0][0]._base[:, O:] == 7.0) and torch.all(outs[0][1]._base[:, H:] == 7.0)

    W = oracle.materialize_w(h, 2, H, O, Z1, Z2, float(lam), M)
    Xo, dYo = X.astype(np.float64), dY.astype(np.float64)
    assert rel_err(to_host_f64(outs[0][0]), oracle.mm_fwd(Xo, W)) <= F32_TOL
    assert rel_err(to_host_f64(outs[0][1]), oracle.mm_bwd_dx(dYo, W)) <= F32_TOL
    assert rel_err(to_host_f64(dM), oracle.mm_bwd_dm(h, 2, Z1, Z2, m, float(lam), Xo, dYo)) <= F32_TOL


@pytest.mark.parametrize("same_sign", [True, False])
def test_f32_plane_products_worst_case_mantissas(roast, same_sign):
    """The three dropped plane products are largest when an operand's leading plane is minimal and its
    two lower planes are all ones: significand 1.0000000 11111111 11111111b = 1 + 2^-7 - 2^-23.  Every
    activation and every entry of M carries that significand (random exponents; with `same_sign` all
    values positive, so the dropped terms add up instead of cancelling).  The bound is then
    ~2^-20 of sum |x||w| per output, still inside the fp32 bar."""
    I, H, O, Z1, Z2, m = 300, 512, 320, 64, 64, 30000
    rng = np.random.default_rng(99)
    worst = np.float32(1.0 + 2.0 ** -7 - 2.0 ** -23)
    assert int(worst.view(np.uint32)) & 0x7fffff == 0xffff

    def draw(shape, spread):
        v = worst * np.exp2(rng.integers(-spread, spread + 1, size=shape)).astype(np.float32)
        return v if same_sign else v * rng.choice(np.float32([-1.0, 1.0]), size=shape)

    M, X, dY = draw(m, 2) * np.float32(0.05), draw((I, H), 3), draw((I, O), 3)
    h = wl.draw_hash(rng, use_sign=not same_sign, align=1)
    d = roast.mm_desc(H, O, Z1, Z2, m, 1, 1.0, h)
    Md, Xd, dYd = to_dev(M), to_dev(X), to_dev(dY)
    Y = roast.roast_mm_fwd(d, Xd, Md, ws=ws_tensor(roast.roast_mm_fwd_workspace(d, torch.float32, I)))
    dX = roast.roast_mm_bwd_dx(d, dYd, Md, ws=ws_tensor(roast.roast_mm_bwd_dx_workspace(d, torch.float32, I)))
    dM = torch.zeros(m, dtype=torch.float32, device="cuda")
    roast.roast_mm_bwd_dM(d, Xd, dYd, dM, roast.ROAST_REDUCE_ATOMIC, ws_tensor(roast.roast_mm_bwd_dM_workspace_f32(d, I)))
    torch.cuda.synchronize()
    W = oracle.materialize_w(h, 1, H, O, Z1, Z2, 1.0, M)
    Xo, dYo = X.astype(np.float64), dY.astype(np.float64)
    assert rel_err(to_host_f64(Y), oracle.mm_fwd(Xo, W)) <= F32_TOL
    assert rel_err(to_host_f64(dX), oracle.mm_bwd_dx(dYo, W)) <= F32_TOL
    assert rel_err(to_host_f64(dM), oracle.mm_bwd_dm(h, 1, Z1, Z2, m, 1.0, Xo, dYo)) <= F32_TOL


def test_plane_split_is_exact_on_awkward_values(roast):
    """With |M| one tile holding a single 1.0, one output column reproduces one input column: exactly
    for every value of magnitude >= 2^-100 (largest finite, just below a power of two, 24 significant
    bits, ...), to within 2^-126 below that (subnormal residuals), and non-finite stays non-finite."""
    H, O, Z, m, I = 64, 64, 64, 64 * 64, 256
    rng = np.random.default_rng(8)
    hp = wl.draw_hash(rng, use_sign=False, align=1)
    M = np.zeros(m, dtype=np.float32)
    M[5 * 64 + 9] = 1.0                              # W[5, 9] = 1 (single tile at offset 0, no sign)
    exact = np.array([3.4028235e38, -3.4028235e38, 3.3895314e38, 0.99999994, 1.9999999, 16777215.0, 1.0000001,
                      65504.0, 1e-30, -7.7e-31, 0.0], dtype=np.float32)
    tiny = np.array([1.1754944e-38, 1e-40, -1e-45, 3e-36], dtype=np.float32)
    nonfinite = np.array([np.inf, -np.inf, np.nan], dtype=np.float32)
    X = np.zeros((I, H), dtype=np.float32)
    col = np.concatenate([exact, tiny, nonfinite, rng.standard_normal(I - 18).astype(np.float32)])
    X[:, 5] = col
    d = roast.mm_desc(H, O, Z, Z, m, 0, 1.0, hp)
    need = roast.roast_mm_fwd_workspace(d, torch.float32, I)
    assert need > 0
    Y = roast.roast_mm_fwd(d, to_dev(X), to_dev(M), ws=ws_tensor(need))
    got = Y[:, 9].cpu().numpy()
    fin = np.isfinite(col)
    big = fin & ((np.abs(col) >= 2.0 ** -100) | (col == 0))
    np.testing.assert_array_equal(got[big], col[big])
    assert np.all(np.abs(got[fin].astype(np.float64) - col[fin].astype(np.float64)) <= 2.0 ** -126)
    assert not np.isfinite(got[~fin]).any()
    others = torch.cat([Y[:, :9], Y[:, 10:]], dim=1)[torch.from_numpy(fin).cuda()]
    assert not others.any()                          # finite rows: every other column is exactly zero


def test_f32_workspace_contract(roast):
    I, H, O, Z, m = 300, 128, 320, 64, 20000
    rng = np.random.default_rng(1)
    d = roast.mm_desc(H, O, Z, Z, m, 0, 1.0, wl.draw_hash(rng))
    X = torch.randn((I, H), device="cuda")
    M = torch.randn(m, device="cuda")
    need = roast.roast_mm_fwd_workspace(d, torch.float32, I)
    with pytest.raises(roast.RoastError) as e:
        roast.roast_mm_fwd(d, X, M, ws=ws_tensor(need - 256))
    assert e.value.status == roast.ROAST_ERR_WORKSPACE
    # a shape the matrix-core kernels do not take: no workspace asked for, the call still works
    d2 = roast.mm_desc(100, 130, 7, 5, 900, 0, 1.0, wl.draw_hash(rng))
    assert roast.roast_mm_fwd_workspace(d2, torch.float32, 70) == 0
    assert roast.roast_mm_bwd_dM_workspace_f32(d2, 70) == 0
    X2, M2 = torch.randn((70, 100), device="cuda"), torch.randn(900, device="cuda")
    Y1 = roast.roast_mm_fwd(d2, X2, M2, ws=ws_tensor(16))
    Y2 = roast.roast_mm_fwd(d2, X2, M2)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)
