"""GPU parity of the strip launches of the bf16 forward and dX products: where short blocks would
queue for the CUs, one workgroup computes several consecutive 128-column blocks as one run of
contraction steps and stores the inner ones through a small staging area.  Same oracle, same bf16 bar
as the plain calls; the shapes are chosen so that strips of 2, 3 and 4 blocks form (checked through the
library's diagnostic), with ragged row counts, padded leading dimensions, tile shapes from 8 to 128
and both weight sources (bf16 shadow, fp32 M)."""
import numpy as np
import pytest

import oracle
from paper_2207_10702_amd import workloads as wl
from tests.util import BF16_TOL, rel_err, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

# (I, H, O, Z1, Z2, |M|, blocks per strip forward, dX)
SHAPES = [
    (2048, 128, 16384, 64, 64, 60000, 4, 1),     # 1024 forward blocks of 2 steps -> strips of 4
    (2048, 16384, 128, 64, 64, 60000, 1, 4),     # the same for dX
    (2000, 192, 12288, 32, 128, 50000, 3, 1),    # 768 blocks -> strips of 3; last row block ragged
    (2000, 12288, 192, 128, 32, 50000, 1, 3),
    (2048, 256, 8192, 16, 8, 9000, 2, 1),        # 512 blocks -> strips of 2; 16 hash tiles per block
    (2048, 8192, 256, 8, 16, 9000, 1, 2),
    (1800, 64, 24576, 64, 128, 70000, 3, 1),     # one contraction step per block, 1536 blocks -> 512 strips of 3
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("pad", [0, 8])
def test_strip_launches_match_oracle(roast, shape, pad):
    I, H, O, Z1, Z2, m, tf, tx = shape
    rng = np.random.default_rng(31 * I + H + O)
    M = wl.draw_m(rng, m, ("normal", 0.05))
    X = wl.draw_act(rng, I, H, "bf16")
    dY = wl.draw_act(rng, I, O, "bf16")
    h = wl.draw_hash(rng, use_sign=True, align=1)
    lam = np.float32(0.37)
    d = roast.mm_desc(H, O, Z1, Z2, m, 5, lam, h)
    assert roast.roast_mm_strip_blocks(d, I, 0) == tf and roast.roast_mm_strip_blocks(d, I, 1) == tx
    Md = to_dev(M)
    Mb = roast.roast_m_shadow_bf16(Md)
    Xd = torch.zeros((I, H + pad), dtype=torch.bfloat16, device="cuda")[:, :H]
    Xd.copy_(to_dev(X))
    dYd = torch.zeros((I, O + pad), dtype=torch.bfloat16, device="cuda")[:, :O]
    dYd.copy_(to_dev(dY))
    W = oracle.materialize_w(h, 5, H, O, Z1, Z2, float(lam), M)
    Yr = oracle.mm_fwd(wl.act_as_f64(X), W)
    dXr = oracle.mm_bwd_dx(wl.act_as_f64(dY), W)
    outs = []
    for shadow in (True, False):
        Y = torch.full((I, O + pad), 7.0, dtype=torch.bfloat16, device="cuda")[:, :O]
        dX = torch.full((I, H + pad), 7.0, dtype=torch.bfloat16, device="cuda")[:, :H]
        roast.roast_mm_fwd(d, Xd, Md, Y, M_bf16=Mb if shadow else None)
        roast.roast_mm_bwd_dx(d, dYd, Md, dX, M_bf16=Mb if shadow else None)
        torch.cuda.synchronize()
        if pad:   # nothing is written between the rows
            assert torch.all(Y._base[:, O:] == 7.0) and torch.all(dX._base[:, H:] == 7.0)
        assert rel_err(to_host_f64(Y), Yr) <= BF16_TOL
        assert rel_err(to_host_f64(dX), dXr) <= BF16_TOL
        outs.append((Y, dX))
    # the shadow holds exactly the bf16 roundings the fp32 path makes on the fly
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
