"""GPU parity on the five benchmark configurations at their full sizes, in the launch configuration
bench.py times.  Where the oracle cannot produce every output in seconds, it is asked for sampled
outputs it can compute one by one (full rows of Y / dX, windows of dM summed over every virtual
weight that lands in them), and the adjoint identities <dY,Y> = <dX,X> = <dM,M> are checked on the
complete GPU outputs in float64.

Every reference value comes from the oracle fed with the exact tensors the GPU call received (for
the chained configuration that includes intermediate activations produced on the GPU, so that each
call is checked on its own and rounding does not compound).
"""
import numpy as np
import pytest

import oracle
from paper_2207_10702_amd import workloads as wl
from tests.util import BF16_TOL, F32_TOL, rel_err, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def sample_rows(rng, I, k):
    # always include the first and last row and a row next to a 256-row workgroup boundary
    fixed = np.array([0, 255, 256, I - 1])
    return np.unique(np.concatenate([fixed[fixed < I], rng.choice(I, size=k, replace=False)]))


AS_COMPUTED = {}   # reported, not gated: error against the reference that rounds sign*M to bf16 as the kernels do


def check_layer_sampled(roast, cfg, layer, h, M, Md, Xd, dYd, Y, dX, rng, n_rows, tol, report=None):
    """Y and dX of one call on sampled rows against the oracle's materialised W (the ideal reference:
    M not rounded).  For bf16 calls the error against the "as-computed" reference -- sign*M rounded
    to bfloat16 before the products, accumulation in double -- is recorded under `report` and printed;
    what is left there is the fp32 accumulation order and the one bf16 rounding of the output."""
    lam = float(np.float32(cfg.lam))
    W = oracle.materialize_w(h, layer.layer_id, layer.H, layer.O, cfg.Z1, cfg.Z2, lam, M)
    r = sample_rows(rng, Xd.shape[0], n_rows)
    rt = torch.from_numpy(r).cuda()
    Xs, dYs = to_host_f64(Xd[rt]), to_host_f64(dYd[rt])
    gotY, gotdX = to_host_f64(Y[rt]), to_host_f64(dX[rt])
    errs = dict(Y=rel_err(gotY, oracle.mm_fwd(Xs, W)), dX=rel_err(gotdX, oracle.mm_bwd_dx(dYs, W)))
    for k, e in errs.items():
        assert e <= tol, (layer.name, k, e)
    if report is not None and Y.dtype == torch.bfloat16:
        Wr = oracle.materialize_w(h, layer.layer_id, layer.H, layer.O, cfg.Z1, cfg.Z2, lam, M, round_bf16=True)
        ac = dict(Y=rel_err(gotY, oracle.mm_fwd(Xs, Wr)), dX=rel_err(gotdX, oracle.mm_bwd_dx(dYs, Wr)))
        worst = AS_COMPUTED.setdefault(report, dict(Y=0.0, dX=0.0, Y_ideal=0.0, dX_ideal=0.0))
        for k in ("Y", "dX"):
            worst[k] = max(worst[k], ac[k])
            worst[k + "_ideal"] = max(worst[k + "_ideal"], errs[k])
    return W


def print_as_computed(report):
    w = AS_COMPUTED.get(report)
    if w:
        print(f"\n[{report}] max rel err vs ideal reference: Y {w['Y_ideal']:.2e} dX {w['dX_ideal']:.2e}; "
              f"vs as-computed (sign*M rounded to bf16) reference: Y {w['Y']:.2e} dX {w['dX']:.2e}", flush=True)


def window_err(got_win, ref, rms):
    return float(np.max(np.abs(got_win - ref) / np.maximum(np.abs(ref), rms)))


def dot64(a, b):
    return float((a.double() * b.double()).sum().item())


def dot_scale(a, b):
    """Inner product in float64 and the size of its rounding noise: sqrt(sum (a_i b_i)^2)."""
    p = a.double() * b.double()
    return float(p.sum().item()), float(torch.sqrt((p * p).sum()).item())


def assert_adjoint(pair1, pair2, what):
    """<a1,b1> == <a2,b2> up to bf16 rounding of the stored tensors (each term off by ~2^-8 at random)."""
    s1, n1 = dot_scale(*pair1)
    s2, n2 = dot_scale(*pair2)
    assert abs(s1 - s2) <= 0.05 * (n1 + n2), (what, s1, s2, n1, n2)


# ------------------------------------------------------------------ config 1 (complete, fp32)
def test_cfg1_single_layer_fp32_complete(roast):
    cfg = wl.CONFIGS["cfg1_single_f32"]
    inp = wl.make_mm_inputs(cfg)
    l = cfg.layers[0]
    d = roast.mm_desc(l.H, l.O, cfg.Z1, cfg.Z2, cfg.m_size, l.layer_id, cfg.lam, inp.hash)
    Md, Xd, dYd = to_dev(inp.M), to_dev(inp.X[l.name]), to_dev(inp.dY[l.name])
    Y = roast.roast_mm_fwd(d, Xd, Md)
    dX = roast.roast_mm_bwd_dx(d, dYd, Md)
    dM = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
    roast.roast_mm_bwd_dM(d, Xd, dYd, dM)
    off, sgn = roast.roast_tile_index_device(d)
    eoff, esgn = oracle.tile_index(inp.hash, l.layer_id, l.H, l.O, cfg.Z1, cfg.Z2, cfg.m_size)
    assert np.array_equal(off.cpu().numpy(), eoff) and np.array_equal(sgn.cpu().numpy(), esgn)
    W = oracle.materialize_w(inp.hash, l.layer_id, l.H, l.O, cfg.Z1, cfg.Z2, cfg.lam, inp.M)
    X, dY = inp.X[l.name].astype(np.float64), inp.dY[l.name].astype(np.float64)
    assert rel_err(to_host_f64(Y), oracle.mm_fwd(X, W)) <= F32_TOL
    assert rel_err(to_host_f64(dX), oracle.mm_bwd_dx(dY, W)) <= F32_TOL
    ref_dM = oracle.mm_bwd_dm(inp.hash, l.layer_id, cfg.Z1, cfg.Z2, cfg.m_size, cfg.lam, X, dY)
    assert rel_err(to_host_f64(dM), ref_dM) <= F32_TOL
    # the configuration bench.py --workload cfg1_single_f32 times: the same calls with their workspaces
    # (fp32 on the matrix cores; the 32x32 hash tiles are half the kernel's contraction step)
    sizes = (roast.roast_mm_fwd_workspace(d, torch.float32, cfg.I), roast.roast_mm_bwd_dx_workspace(d, torch.float32, cfg.I),
             roast.roast_mm_bwd_dM_workspace_f32(d, cfg.I))
    assert min(sizes) > 0
    ws = torch.empty(max(sizes), dtype=torch.uint8, device="cuda")
    planes = roast.roast_m_planes_bf16(Md)
    Yw = roast.roast_mm_fwd(d, Xd, Md, M_bf16=planes, ws=ws)
    dXw = roast.roast_mm_bwd_dx(d, dYd, Md, M_bf16=planes, ws=ws)
    dMw = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
    roast.roast_mm_bwd_dM(d, Xd, dYd, dMw, roast.ROAST_REDUCE_ATOMIC, ws)
    assert rel_err(to_host_f64(Yw), oracle.mm_fwd(X, W)) <= F32_TOL
    assert rel_err(to_host_f64(dXw), oracle.mm_bwd_dx(dY, W)) <= F32_TOL
    assert rel_err(to_host_f64(dMw), ref_dM) <= F32_TOL


# ------------------------------------------------------------------ config 2 (chained FFN pair, bf16)
def test_cfg2_bert_ffn_bf16_full_size(roast):
    cfg = wl.CONFIGS["cfg2_bert_ffn_bf16"]
    inp = wl.make_mm_inputs(cfg)
    rng = np.random.default_rng(2)
    l1, l2 = cfg.layers
    h, lam = inp.hash, float(np.float32(cfg.lam))
    d1 = roast.mm_desc(l1.H, l1.O, cfg.Z1, cfg.Z2, cfg.m_size, l1.layer_id, cfg.lam, h)
    d2 = roast.mm_desc(l2.H, l2.O, cfg.Z1, cfg.Z2, cfg.m_size, l2.layer_id, cfg.lam, h)
    Md, Xd, dYd = to_dev(inp.M), to_dev(inp.X[l1.name]), to_dev(inp.dY[l2.name])
    # the launch configuration bench.py times: weights read from the bf16 shadow of M, dM without workspace
    Mb = roast.roast_m_shadow_bf16(Md)
    H1 = roast.roast_mm_fwd(d1, Xd, Md, M_bf16=Mb)
    Y = roast.roast_mm_fwd(d2, H1, Md, M_bf16=Mb)
    dH1 = roast.roast_mm_bwd_dx(d2, dYd, Md, M_bf16=Mb)
    dX = roast.roast_mm_bwd_dx(d1, dH1, Md, M_bf16=Mb)
    # ... and the shadow must not change a bit
    assert torch.equal(H1, roast.roast_mm_fwd(d1, Xd, Md)) and torch.equal(dX, roast.roast_mm_bwd_dx(d1, dH1, Md))
    dM2 = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
    dM1 = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
    roast.roast_mm_bwd_dM(d2, H1, dYd, dM2)
    roast.roast_mm_bwd_dM(d1, Xd, dH1, dM1)
    torch.cuda.synchronize()
    # index maps of both layers
    for d, l in ((d1, l1), (d2, l2)):
        off, sgn = roast.roast_tile_index_device(d)
        eoff, esgn = oracle.tile_index(h, l.layer_id, l.H, l.O, cfg.Z1, cfg.Z2, cfg.m_size)
        assert np.array_equal(off.cpu().numpy(), eoff) and np.array_equal(sgn.cpu().numpy(), esgn)
    # each call on sampled rows, fed with the tensors that call actually received
    check_layer_sampled(roast, cfg, l1, h, inp.M, Md, Xd, dH1, H1, dX, rng, 96, BF16_TOL, report="cfg2")
    check_layer_sampled(roast, cfg, l2, h, inp.M, Md, H1, dYd, Y, dH1, rng, 96, BF16_TOL, report="cfg2")
    print_as_computed("cfg2")
    # dM of each layer on windows of slots, summed over every virtual weight hashed into them
    Xo, dH1o, H1o, dYo = (to_host_f64(t) for t in (Xd, dH1, H1, dYd))
    for (d, l, A, G, dM) in ((d1, l1, Xo, dH1o, dM1), (d2, l2, H1o, dYo, dM2)):
        got = to_host_f64(dM)
        rms = float(np.sqrt(np.mean(got * got)))
        starts = np.concatenate([[0, cfg.m_size - 48], rng.choice(cfg.m_size - 48, size=6, replace=False)])
        for j0 in starts:
            ref = oracle.dm_window(h, l.layer_id, cfg.Z1, cfg.Z2, cfg.m_size, lam, A, G, int(j0), int(j0) + 48)
            err = np.max(np.abs(got[j0:j0 + 48] - ref) / np.maximum(np.abs(ref), rms))
            assert err <= BF16_TOL, (l.name, int(j0), err)
    # adjoint identities on the complete outputs (bf16 outputs: rounding of Y / dX limits them)
    assert_adjoint((dYd, Y), (dH1, H1), "layer 2: <dY,Y> vs <dX,X>")
    assert_adjoint((dYd, Y), (dM2, Md), "layer 2: <dY,Y> vs <dM,M>")
    assert_adjoint((dH1, H1), (dX, Xd), "layer 1: <dY,Y> vs <dX,X>")
    assert_adjoint((dH1, H1), (dM1, Md), "layer 1: <dY,Y> vs <dM,M>")


# ------------------------------------------------------------------ config 3 (48 layers, one M)
def test_cfg3_bert_stack_bf16_full_size(roast):
    cfg = wl.CONFIGS["cfg3_bert_stack_bf16"]
    inp = wl.make_mm_inputs(cfg)
    rng = np.random.default_rng(3)
    h, lam = inp.hash, float(np.float32(cfg.lam))
    Md = to_dev(inp.M)
    Mb = roast.roast_m_shadow_bf16(Md)
    dev = {}
    for l in cfg.layers[:4]:          # one X / dY per distinct shape, shared by the 12 transformer layers
        dev[(l.H, l.O)] = (to_dev(inp.X[l.name]), to_dev(inp.dY[l.name]))
    dM = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
    adj_y, adj_n = 0.0, 0.0
    for idx, l in enumerate(cfg.layers):
        d = roast.mm_desc(l.H, l.O, cfg.Z1, cfg.Z2, cfg.m_size, l.layer_id, cfg.lam, h)
        Xd, dYd = dev[(l.H, l.O)]
        Y = roast.roast_mm_fwd(d, Xd, Md, M_bf16=Mb)
        dX = roast.roast_mm_bwd_dx(d, dYd, Md, M_bf16=Mb)
        roast.roast_mm_bwd_dM(d, Xd, dYd, dM)
        off, sgn = roast.roast_tile_index_device(d)
        eoff, esgn = oracle.tile_index(h, l.layer_id, l.H, l.O, cfg.Z1, cfg.Z2, cfg.m_size)
        assert np.array_equal(off.cpu().numpy(), eoff) and np.array_equal(sgn.cpu().numpy(), esgn)
        # Y / dX rows of every one of the 48 calls (16 random rows + the fixed boundary rows)
        check_layer_sampled(roast, cfg, l, h, inp.M, Md, Xd, dYd, Y, dX, rng, 16, BF16_TOL, report="cfg3")
        a, n = dot_scale(dYd, Y)
        adj_y += a
        adj_n += n * n
        assert_adjoint((dYd, Y), (dX, Xd), l.name)
    torch.cuda.synchronize()
    print_as_computed("cfg3")
    # the shared gradient: <dM, M> = sum over layers of <dY, Y>
    adj_m, n_m = dot_scale(dM, Md)
    assert abs(adj_m - adj_y) <= 0.05 * (np.sqrt(adj_n) + n_m)
    # windows of the shared gradient, every one of the 48 layers contributing to every slot sampled:
    # 16 windows of 128 slots = 2048 slots (first and last window of M, 14 random ones), each slot the
    # sum of about a thousand virtual weights
    got = to_host_f64(dM)
    rms = float(np.sqrt(np.mean(got * got)))
    host = {k: (to_host_f64(v[0]), to_host_f64(v[1])) for k, v in dev.items()}
    WIN = 128
    starts = [0, cfg.m_size - WIN] + [int(v) for v in rng.choice(cfg.m_size - WIN, size=14, replace=False)]
    for j0 in starts:
        ref = np.zeros(WIN)
        for l in cfg.layers:
            A, G = host[(l.H, l.O)]
            ref += oracle.dm_window(h, l.layer_id, cfg.Z1, cfg.Z2, cfg.m_size, lam, A, G, j0, j0 + WIN)
        err = window_err(got[j0:j0 + WIN], ref, rms)
        assert err <= BF16_TOL, (j0, err)


# ------------------------------------------------------------------ config 4 (lookup)
def test_cfg4_dlrm_lookup_full_size(roast):
    cfg = wl.CONFIGS["cfg4_dlrm_embed_f32"]
    ei = wl.make_embed_inputs(cfg)
    rng = np.random.default_rng(4)
    d = roast.embed_desc(cfg.D, cfg.Z, cfg.m_size, cfg.lam, ei.hash)
    rows, tables, Md, dOut = to_dev(ei.rows), to_dev(ei.tables), to_dev(ei.M), to_dev(ei.dOut)
    out = roast.roast_embed_fwd(d, rows, tables, Md)
    ws = torch.empty(max(roast.roast_embed_bwd_workspace(d, cfg.N), 1), dtype=torch.uint8, device="cuda")
    dM = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
    roast.roast_embed_bwd(d, rows, tables, dOut, dM, ws=ws)
    torch.cuda.synchronize()
    # chunk map, bit-exact on sampled lookups
    off, sgn = roast.roast_chunk_index_device(d, rows, tables)
    off, sgn = off.cpu().numpy(), sgn.cpu().numpy()
    C = cfg.D // cfg.Z
    for n in rng.choice(cfg.N, size=2000, replace=False):
        for c in range(C):
            assert (off[n * C + c], sgn[n * C + c]) == oracle.locate(ei.hash, int(ei.tables[n]), int(ei.rows[n]), c,
                                                                     cfg.m_size, cfg.Z)
    # forward on sampled lookups (first, last and random ones)
    pick = np.unique(np.concatenate([[0, cfg.N - 1], rng.choice(cfg.N, size=20000, replace=False)]))
    ref = oracle.embed_fwd(ei.hash, cfg.D, cfg.Z, float(cfg.lam), ei.rows[pick], ei.tables[pick], ei.M)
    assert rel_err(to_host_f64(out[torch.from_numpy(pick).cuda()]), ref) <= 1e-7
    # gradient: every slot of M, from the oracle run over the whole batch
    ref_dM = oracle.embed_bwd(ei.hash, cfg.D, cfg.Z, cfg.m_size, float(cfg.lam), ei.rows, ei.tables, ei.dOut)
    assert rel_err(to_host_f64(dM), ref_dM) <= F32_TOL
    assert abs(dot64(dOut, out) - dot64(dM, Md)) <= 1e-4 * abs(dot64(dM, Md))
    # deterministic mode at full size: parity, and the same bits on a second run
    det = roast.ROAST_REDUCE_DETERMINISTIC
    ws_det = torch.empty(roast.roast_embed_bwd_workspace(d, cfg.N, det), dtype=torch.uint8, device="cuda")
    runs = []
    for _ in range(2):
        dM_det = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
        roast.roast_embed_bwd(d, rows, tables, dOut, dM_det, det, ws_det)
        runs.append(dM_det.cpu().numpy())
    assert rel_err(runs[0].astype(np.float64), ref_dM) <= F32_TOL
    assert np.array_equal(runs[0].view(np.uint32), runs[1].view(np.uint32))


# ------------------------------------------------------------------ config 5 (large layer, large M)
def test_cfg5_large_bf16_full_size(roast):
    cfg = wl.CONFIGS["cfg5_large_bf16"]
    inp = wl.make_mm_inputs(cfg)
    rng = np.random.default_rng(5)
    l = cfg.layers[0]
    h, lam = inp.hash, float(np.float32(cfg.lam))
    d = roast.mm_desc(l.H, l.O, cfg.Z1, cfg.Z2, cfg.m_size, l.layer_id, cfg.lam, h)
    Md, Xd, dYd = to_dev(inp.M), to_dev(inp.X[l.name]), to_dev(inp.dY[l.name])
    Mb = roast.roast_m_shadow_bf16(Md)
    Y = roast.roast_mm_fwd(d, Xd, Md, M_bf16=Mb)
    dX = roast.roast_mm_bwd_dx(d, dYd, Md, M_bf16=Mb)
    dM = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
    roast.roast_mm_bwd_dM(d, Xd, dYd, dM)
    torch.cuda.synchronize()
    off, sgn = roast.roast_tile_index_device(d)
    eoff, esgn = oracle.tile_index(h, l.layer_id, l.H, l.O, cfg.Z1, cfg.Z2, cfg.m_size)
    assert np.array_equal(off.cpu().numpy(), eoff) and np.array_equal(sgn.cpu().numpy(), esgn)
    check_layer_sampled(roast, cfg, l, h, inp.M, Md, Xd, dYd, Y, dX, rng, 60, BF16_TOL, report="cfg5")
    print_as_computed("cfg5")
    assert_adjoint((dYd, Y), (dX, Xd), "<dY,Y> vs <dX,X>")
    assert_adjoint((dYd, Y), (dM, Md), "<dY,Y> vs <dM,M>")
    # Slots that no tile covers must still be exactly zero (4096 tiles of 16384 slots in 64 Mi slots:
    # about a fifth of M is uncovered).  Coverage from the oracle's tile map, as a difference array.
    L = cfg.Z1 * cfg.Z2
    diff = np.zeros(cfg.m_size + 1, dtype=np.int32)
    np.add.at(diff, eoff, 1)
    np.add.at(diff, eoff + L, -1)
    covered = np.cumsum(diff[:-1]) > 0
    del diff
    assert 0 < covered.sum() < cfg.m_size
    uncovered = torch.from_numpy(~covered).cuda()
    assert int((dM[uncovered] != 0).sum().item()) == 0, "a slot outside every tile was written"
    # every covered slot received something (a sum of 16384 products of N(0,1) values is never exactly 0)
    assert int((dM[torch.from_numpy(covered).cuda()] == 0).sum().item()) == 0
    del uncovered
    # 32 windows of 4096 slots of dM: 8 that start at a tile's first slot, 8 that end at a tile's last
    # slot, 8 in the middle of a tile, 8 anywhere (they may be partly or wholly uncovered: expected 0)
    Xo, dYo = to_host_f64(Xd), to_host_f64(dYd)
    rms = float(torch.sqrt((dM.double() ** 2).mean()).item())
    WIN = 4096
    tiles = rng.choice(len(eoff), size=24, replace=False)
    starts = [int(eoff[t]) for t in tiles[:8]]
    starts += [int(eoff[t]) + L - WIN for t in tiles[8:16]]
    starts += [int(eoff[t]) + int(rng.integers(1, L - WIN)) for t in tiles[16:24]]
    starts += [int(v) for v in rng.integers(0, cfg.m_size - WIN, size=8)]
    starts[0], starts[8] = int(eoff[0]), int(eoff[-1]) + L - WIN          # first and last tile of the grid
    starts += [0, cfg.m_size - WIN]                                        # both ends of M
    n_nonzero = 0
    for j0 in starts:
        j0 = max(0, min(j0, cfg.m_size - WIN))
        ref = oracle.dm_window(h, l.layer_id, cfg.Z1, cfg.Z2, cfg.m_size, lam, Xo, dYo, j0, j0 + WIN)
        got = to_host_f64(dM[j0:j0 + WIN])
        assert np.array_equal(ref == 0.0, ~covered[j0:j0 + WIN])
        n_nonzero += int((ref != 0.0).sum())
        err = window_err(got, ref, rms)
        assert err <= BF16_TOL, (j0, err)
    assert n_nonzero >= 24 * WIN        # the tile-anchored windows are fully covered


# ------------------------------------------------------------------ config 2's shapes in fp32 (matrix-core plane kernels)
def test_cfg2_shapes_fp32_on_matrix_cores_full_size(roast):
    import dataclasses
    cfg = dataclasses.replace(wl.CONFIGS["cfg2_bert_ffn_bf16"], dtype="f32", chained=False)
    inp = wl.make_mm_inputs(cfg)
    rng = np.random.default_rng(22)
    h, lam = inp.hash, float(np.float32(cfg.lam))
    Md = to_dev(inp.M)
    for l in cfg.layers:
        d = roast.mm_desc(l.H, l.O, cfg.Z1, cfg.Z2, cfg.m_size, l.layer_id, cfg.lam, h)
        Xd, dYd = to_dev(inp.X[l.name]), to_dev(inp.dY[l.name])
        sizes = (roast.roast_mm_fwd_workspace(d, torch.float32, cfg.I), roast.roast_mm_bwd_dx_workspace(d, torch.float32, cfg.I),
                 roast.roast_mm_bwd_dM_workspace_f32(d, cfg.I))
        assert min(sizes) > 0
        ws = torch.empty(max(sizes), dtype=torch.uint8, device="cuda")
        Y = roast.roast_mm_fwd(d, Xd, Md, ws=ws)
        dX = roast.roast_mm_bwd_dx(d, dYd, Md, ws=ws)
        dM = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
        roast.roast_mm_bwd_dM(d, Xd, dYd, dM, roast.ROAST_REDUCE_ATOMIC, ws)
        torch.cuda.synchronize()
        check_layer_sampled(roast, cfg, l, h, inp.M, Md, Xd, dYd, Y, dX, rng, 64, F32_TOL)
        Xo, dYo = to_host_f64(Xd), to_host_f64(dYd)
        got = to_host_f64(dM)
        rms = float(np.sqrt(np.mean(got * got)))
        for j0 in np.concatenate([[0, cfg.m_size - 48], rng.choice(cfg.m_size - 48, size=4, replace=False)]):
            ref = oracle.dm_window(h, l.layer_id, cfg.Z1, cfg.Z2, cfg.m_size, lam, Xo, dYo, int(j0), int(j0) + 48)
            err = np.max(np.abs(got[j0:j0 + 48] - ref) / np.maximum(np.abs(ref), rms))
            assert err <= F32_TOL, (l.name, int(j0), err)
        # fp32 outputs: the adjoint identities hold to fp32 accuracy on the complete tensors
        s_y, n_y = dot_scale(dYd, Y)
        s_x, _ = dot_scale(dX, Xd)
        s_m, _ = dot_scale(dM, Md)
        assert abs(s_y - s_x) <= 1e-4 * n_y and abs(s_y - s_m) <= 1e-4 * n_y, (l.name, s_y, s_x, s_m, n_y)
