"""Maximum sizes: an array M of 2.5 * 2^30 entries (10.7 GB) and a 32-bit prime, so that block
offsets pass 2^31 -- the 64-bit offset paths of every kernel family (tile table of the MFMA kernels,
generic kernels, shadow of M, one-thread-per-element lookup kernels) against the oracle."""
import numpy as np
import pytest

import oracle
from paper_2207_10702_amd import workloads as wl
from tests.util import BF16_TOL, F32_TOL, rel_err, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

M_SIZE = 5 << 29
P32 = 4294967291          # largest prime below 2^32


@pytest.fixture(scope="module")
def big_m():
    g = torch.Generator(device="cuda").manual_seed(31)
    Md = torch.empty(M_SIZE, dtype=torch.float32, device="cuda").normal_(0.0, 0.05, generator=g)
    Mh = Md.cpu().numpy()
    yield Md, Mh
    del Md
    torch.cuda.empty_cache()


@pytest.mark.timeout(600)
def test_mm_with_offsets_beyond_31_bits(roast, big_m):
    Md, Mh = big_m
    rng = np.random.default_rng(77)
    I, H, O, Z = 300, 256, 384, 64
    h = wl.draw_hash(rng, use_sign=True, align=1, P=P32)
    layer = next(l for l in range(64)
                 if (oracle.tile_index(h, l, H, O, Z, Z, M_SIZE)[0] >= (1 << 31)).sum() >= 2)
    eoff, esgn = oracle.tile_index(h, layer, H, O, Z, Z, M_SIZE)
    lam = np.float32(0.7)
    d = roast.mm_desc(H, O, Z, Z, M_SIZE, layer, lam, h)
    off, sgn = roast.roast_tile_index_device(d)
    assert np.array_equal(off.cpu().numpy(), eoff) and np.array_equal(sgn.cpu().numpy(), esgn)
    W = oracle.materialize_w(h, layer, H, O, Z, Z, float(lam), Mh)
    Mb = roast.roast_m_shadow_bf16(Md)
    for dtype, tol in (("bf16", BF16_TOL), ("f32", F32_TOL)):
        X, dY = wl.draw_act(rng, I, H, dtype), wl.draw_act(rng, I, O, dtype)
        Xd, dYd = to_dev(X), to_dev(dY)
        shadow = Mb if dtype == "bf16" else None
        Y = roast.roast_mm_fwd(d, Xd, Md, M_bf16=shadow)
        dX = roast.roast_mm_bwd_dx(d, dYd, Md, M_bf16=shadow)
        if dtype == "bf16":
            assert torch.equal(Y, roast.roast_mm_fwd(d, Xd, Md)) and torch.equal(dX, roast.roast_mm_bwd_dx(d, dYd, Md))
        Xo, dYo = wl.act_as_f64(X), wl.act_as_f64(dY)
        assert rel_err(to_host_f64(Y), oracle.mm_fwd(Xo, W)) <= tol, dtype
        assert rel_err(to_host_f64(dX), oracle.mm_bwd_dx(dYo, W)) <= tol, dtype
        dM = torch.zeros(M_SIZE, dtype=torch.float32, device="cuda")
        roast.roast_mm_bwd_dM(d, Xd, dYd, dM)
        # windows at the start of tiles on both sides of 2^31, and one across the end of a tile
        starts = [int(eoff.max()), int(eoff.min()), int(np.sort(eoff)[len(eoff) // 2]) + Z * Z - 24]
        scale = None
        for j0 in starts:
            ref = oracle.dm_window(h, layer, Z, Z, M_SIZE, float(lam), Xo, dYo, j0, j0 + 48)
            got = to_host_f64(dM[j0:j0 + 48])
            scale = scale or float(np.sqrt(np.mean(ref * ref)))
            assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), scale)) <= tol, (dtype, j0)
        touched = int(torch.count_nonzero(dM).item())
        assert 0 < touched <= eoff.size * Z * Z          # nothing outside the tiles' images
        del dM
    del Mb


@pytest.mark.timeout(600)
def test_lookup_with_offsets_beyond_31_bits(roast, big_m):
    Md, Mh = big_m
    rng = np.random.default_rng(78)
    D, Z, N = 64, 16, 3000
    C = D // Z
    h = wl.draw_hash(rng, use_sign=True, align=1, P=P32)
    lam = np.float32(1.3)
    rows = rng.integers(0, 1 << 40, size=N)
    tables = rng.integers(0, 26, size=N).astype(np.uint32)
    d = roast.embed_desc(D, Z, M_SIZE, lam, h)
    out = roast.roast_embed_fwd(d, to_dev(rows), to_dev(tables), Md)
    assert rel_err(to_host_f64(out), oracle.embed_fwd(h, D, Z, float(lam), rows, tables, Mh)) <= 1e-7
    off_d, sgn_d = roast.roast_chunk_index_device(d, to_dev(rows), to_dev(tables))
    loc = [oracle.locate(h, int(tables[n]), int(rows[n]), c, M_SIZE, Z) for n in range(N) for c in range(C)]
    offs = np.array([o for o, _ in loc], dtype=np.int64)
    sgns = np.array([s for _, s in loc], dtype=np.int8)
    assert np.array_equal(off_d.cpu().numpy().reshape(-1), offs) and np.array_equal(sgn_d.cpu().numpy().reshape(-1), sgns)
    assert (offs >= (1 << 31)).sum() > 100
    # gradient: expected values at the touched slots from the scalar map; nothing else is touched
    dOut = rng.standard_normal((N, D), dtype=np.float32)
    dM = torch.zeros(M_SIZE, dtype=torch.float32, device="cuda")
    roast.roast_embed_bwd(d, to_dev(rows), to_dev(tables), to_dev(dOut), dM)
    expect = {}
    flat = dOut.reshape(N * C, Z).astype(np.float64)
    for k in range(N * C):
        for o in range(Z):
            expect[int(offs[k]) + o] = expect.get(int(offs[k]) + o, 0.0) + float(lam) * int(sgns[k]) * flat[k, o]
    idx = np.fromiter(expect.keys(), dtype=np.int64)
    ref = np.fromiter(expect.values(), dtype=np.float64)
    got = to_host_f64(dM[torch.from_numpy(idx).cuda()])
    assert rel_err(got, ref) <= F32_TOL
    assert int(torch.count_nonzero(dM).item()) <= idx.size
    # pooled variant over the same lookups (bags of 3)
    bag_off = np.arange(0, N + 1, 3, dtype=np.int64)
    pooled = roast.roast_embed_bag_fwd(d, to_dev(rows), to_dev(tables), to_dev(bag_off), Md)
    assert rel_err(to_host_f64(pooled), oracle.embed_bag_fwd(h, D, Z, float(lam), rows, tables, bag_off, Mh)) <= F32_TOL
