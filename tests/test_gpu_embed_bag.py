"""GPU parity of the pooled (bag-sum) lookup and its gradient against the CPU oracle: fp32 <= 1e-5
max relative error per tensor; empty bags, bags longer than a hashing window, rows wider than a
workgroup pass, short last chunks, both gradient paths (direct atomics / routed) and the
deterministic mode (bit-identical from run to run)."""
import numpy as np
import pytest

import oracle
from paper_2207_10702_amd import workloads as wl
from tests.util import F32_TOL, rel_err, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def bag_sizes(rng, kind, B):
    if kind == "mixed":          # empty bags at both ends and in the middle, a few long ones
        s = rng.integers(0, 9, size=B)
        s[0] = s[-1] = s[B // 2] = 0
        s[B // 3] = 70
        return s
    if kind == "fixed26":        # one id per table and sample, summed per sample
        return np.full(B, 26)
    if kind == "one_long":       # a bag longer than one hashing window (8192 / C lookups)
        s = rng.integers(0, 4, size=B)
        s[1] = 5000
        return s
    raise ValueError(kind)


CASES = [  # D, Z, m, B, bag sizes
    (128, 32, 20000, 900, "mixed"),       # 16-byte pieces, direct-atomic gradient
    (128, 32, 300000, 1500, "fixed26"),   # 39000 lookups x 4 chunks: routed gradient
    (64, 16, 5000, 40, "one_long"),
    (10, 4, 60, 120, "mixed"),            # D % 4 != 0: one element per thread, short last chunk
    (64, 64, 64, 50, "mixed"),            # |M| == chunk
    (33, 1, 500, 30, "mixed"),            # chunk size 1
    (2048, 128, 40000, 9, "mixed"),       # 512 pieces per row: two passes of the workgroup
    (96, 4, 3000, 25, "mixed"),           # 24 chunks per row: one-thread-per-element fallback
]


@pytest.mark.parametrize("D,Z,m,B,kind", CASES)
def test_bag_lookup_matches_oracle(roast, D, Z, m, B, kind):
    rng = np.random.default_rng(D * 7 + B)
    sizes = bag_sizes(rng, kind, B)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    N = int(offsets[-1])
    M = wl.draw_m(rng, m, ("normal", 0.02))
    rows = rng.integers(0, 50, size=N)
    rows[::3] = rng.integers(0, 1 << 33, size=rows[::3].size)
    tables = rng.integers(0, 4, size=N).astype(np.uint32)
    dOut = rng.standard_normal((B, D), dtype=np.float32)
    h = wl.draw_hash(rng)
    lam = np.float32(0.8)
    d = roast.embed_desc(D, Z, m, lam, h)
    rd, td, od, Md, gd = to_dev(rows), to_dev(tables), to_dev(offsets), to_dev(M), to_dev(dOut)

    out = torch.full((B, D), 5.0, dtype=torch.float32, device="cuda")
    roast.roast_embed_bag_fwd(d, rd, td, od, Md, out)
    out2 = roast.roast_embed_bag_fwd(d, rd, td, od, Md)
    ref_out = oracle.embed_bag_fwd(h, D, Z, float(lam), rows, tables, offsets, M)
    assert rel_err(to_host_f64(out), ref_out) <= F32_TOL
    assert torch.equal(out, out2)
    assert not out[torch.from_numpy(sizes == 0).cuda()].any()          # empty bags are zero rows

    ref_dM = oracle.embed_bag_bwd(h, D, Z, m, float(lam), rows, tables, offsets, dOut)
    dM = torch.zeros(m, dtype=torch.float32, device="cuda")
    roast.roast_embed_bag_bwd(d, rd, td, od, gd, dM)
    assert rel_err(to_host_f64(dM), ref_dM) <= F32_TOL
    ws = torch.empty(max(roast.roast_embed_bag_bwd_workspace(d, N, B), 1), dtype=torch.uint8, device="cuda")
    dM_ws = torch.zeros(m, dtype=torch.float32, device="cuda")
    roast.roast_embed_bag_bwd(d, rd, td, od, gd, dM_ws, ws=ws)
    assert rel_err(to_host_f64(dM_ws), ref_dM) <= F32_TOL

    det = roast.ROAST_REDUCE_DETERMINISTIC
    ws_det = torch.empty(max(roast.roast_embed_bag_bwd_workspace(d, N, B, det), 1), dtype=torch.uint8, device="cuda")
    start = rng.standard_normal(m).astype(np.float32)
    runs = []
    for _ in range(2):
        dM_det = to_dev(start.copy())
        roast.roast_embed_bag_bwd(d, rd, td, od, gd, dM_det, det, ws_det)
        runs.append(dM_det.cpu().numpy())
    assert rel_err(runs[0].astype(np.float64) - start.astype(np.float64), ref_dM) <= F32_TOL
    assert np.array_equal(runs[0].view(np.uint32), runs[1].view(np.uint32))


def test_bags_of_one_equal_the_plain_lookup_bit_for_bit(roast):
    rng = np.random.default_rng(77)
    D, Z, m, N = 128, 32, 50000, 3000
    M = wl.draw_m(rng, m, ("normal", 0.02))
    rows, tables = rng.integers(0, 1 << 30, size=N), rng.integers(0, 26, size=N).astype(np.uint32)
    d = roast.embed_desc(D, Z, m, np.float32(1.0), wl.draw_hash(rng))
    off = to_dev(np.arange(N + 1, dtype=np.int64))
    a = roast.roast_embed_bag_fwd(d, to_dev(rows), to_dev(tables), off, to_dev(M))
    b = roast.roast_embed_fwd(d, to_dev(rows), to_dev(tables), to_dev(M))
    assert torch.equal(a, b)


def test_no_lookups_and_no_bags(roast):
    d = roast.embed_desc(16, 4, 100, 1.0, wl.draw_hash(np.random.default_rng(3)))
    M = torch.ones(100, dtype=torch.float32, device="cuda")
    none_i64 = torch.empty(0, dtype=torch.int64, device="cuda")
    none_i32 = torch.empty(0, dtype=torch.int32, device="cuda")
    out = roast.roast_embed_bag_fwd(d, none_i64, none_i32, torch.zeros(6, dtype=torch.int64, device="cuda"), M,
                                    torch.full((5, 16), 3.0, device="cuda"))
    assert not out.any()                                           # five empty bags: five zero rows
    dM = torch.zeros(100, dtype=torch.float32, device="cuda")
    roast.roast_embed_bag_bwd(d, none_i64, none_i32, torch.zeros(6, dtype=torch.int64, device="cuda"),
                              torch.ones((5, 16), device="cuda"), dM)
    assert not dM.any()
    out0 = roast.roast_embed_bag_fwd(d, none_i64, none_i32, torch.zeros(1, dtype=torch.int64, device="cuda"), M)
    assert tuple(out0.shape) == (0, 16)
