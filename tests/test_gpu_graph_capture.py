"""The library only launches kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a sequence of calls can be captured in a HIP graph once each kernel has run once.  A
captured step (forward, dX, zeroing of dM, dM, lookup forward and gradient) is replayed several
times with eager work in between; every replay must reproduce the eager results."""
import numpy as np
import pytest

import oracle
from paper_2207_10702_amd import workloads as wl
from tests.util import BF16_TOL, F32_TOL, rel_err, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_captured_step_replays_like_eager(roast, dtype):
    I, H, O, Z1, Z2, m = 320, 256, 192, 32, 32, 9000
    rng = np.random.default_rng(77)
    M = wl.draw_m(rng, m, ("normal", 0.05))
    X = wl.draw_act(rng, I, H, dtype)
    dY = wl.draw_act(rng, I, O, dtype)
    h = wl.draw_hash(rng, use_sign=True, align=1)
    lam = np.float32(0.7)
    d = roast.mm_desc(H, O, Z1, Z2, m, 2, lam, h)
    N, D, Z = 3000, 64, 16
    rows = torch.from_numpy(rng.integers(0, 50000, N).astype(np.int64)).cuda()
    tables = torch.from_numpy(rng.integers(0, 5, N).astype(np.int32)).cuda()
    dOut = torch.from_numpy(rng.standard_normal((N, D)).astype(np.float32)).cuda()
    de = roast.embed_desc(D, Z, m, lam, h)

    Md, Xd, dYd = to_dev(M), to_dev(X), to_dev(dY)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    Y = torch.empty((I, O), dtype=tdt, device="cuda")
    dX = torch.empty((I, H), dtype=tdt, device="cuda")
    dM = torch.empty(m, dtype=torch.float32, device="cuda")
    out = torch.empty((N, D), dtype=torch.float32, device="cuda")
    dMe = torch.empty(m, dtype=torch.float32, device="cuda")
    Mb = roast.roast_m_shadow_bf16(Md) if dtype == "bf16" else None
    ws = torch.empty(max(roast.roast_embed_bwd_workspace(de, N), 16), dtype=torch.uint8, device="cuda")

    def step():
        if Mb is not None:
            roast.roast_m_shadow_bf16(Md, Mb)
        roast.roast_mm_fwd(d, Xd, Md, Y, M_bf16=Mb)
        roast.roast_mm_bwd_dx(d, dYd, Md, dX, M_bf16=Mb)
        dM.zero_()                                   # a fill kernel, not a memset node
        roast.roast_mm_bwd_dM(d, Xd, dYd, dM)
        roast.roast_embed_fwd(de, rows, tables, Md, out)
        dMe.zero_()
        roast.roast_embed_bwd(de, rows, tables, dOut, dMe, roast.ROAST_REDUCE_ATOMIC, ws)

    step()                                           # eager: configures every kernel, gives the reference
    torch.cuda.synchronize()
    eager = [t.clone() for t in (Y, dX, dM, out, dMe)]

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    for rep in range(3):
        for t in (Y, dX, dM, out, dMe):
            t.fill_(float("nan"))                    # eager work between replays; stale results cannot pass
        Xd.add_(0)                                   # an unrelated eager kernel on the same stream
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, eager[0]) and torch.equal(dX, eager[1]) and torch.equal(out, eager[3]), rep
        # the two gradients are sums of atomic adds: same values up to the order of the adds
        assert rel_err(to_host_f64(dM), to_host_f64(eager[2])) <= 1e-5, rep
        assert rel_err(to_host_f64(dMe), to_host_f64(eager[4])) <= 1e-5, rep

    # and the replayed results are the oracle's
    Xo, dYo = wl.act_as_f64(X), wl.act_as_f64(dY)
    W = oracle.materialize_w(h, 2, H, O, Z1, Z2, float(lam), M)
    assert rel_err(to_host_f64(Y), oracle.mm_fwd(Xo, W)) <= tol
    assert rel_err(to_host_f64(dX), oracle.mm_bwd_dx(dYo, W)) <= tol
    assert rel_err(to_host_f64(dM), oracle.mm_bwd_dm(h, 2, Z1, Z2, m, float(lam), Xo, dYo)) <= tol
