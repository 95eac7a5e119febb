"""Pins for the pooled (bag-sum) lookup oracle: the stock CPU embedding-bag operator on a
materialised virtual table (forward), automatic differentiation through that operator (gradient
w.r.t. M), and the adjoint identity.  The per-lookup oracle these build on is pinned in
test_oracle_pins.py."""
import numpy as np
import pytest

import oracle
from paper_2207_10702_amd import workloads as wl

torch = pytest.importorskip("torch")


def setup(seed, D, Z, m, T, R, sizes):
    rng = np.random.default_rng(seed)
    h = wl.draw_hash(rng, use_sign=True, align=1)
    M = rng.standard_normal(m).astype(np.float32)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    N = int(offsets[-1])
    rows = rng.integers(0, R, size=N)
    tables = rng.integers(0, T, size=N).astype(np.uint32)
    if N >= 4:
        rows[1], tables[1] = rows[0], tables[0]          # a repeated id inside the first non-empty bag
    return rng, h, M, offsets, rows, tables


def position_table(h, D, Z, m, T, R):
    """(slot of M, sign) of every element of every row of the virtual tables, from the scalar map."""
    idx = np.empty((T * R, D), dtype=np.int64)
    sgn = np.empty((T * R, D), dtype=np.float64)
    for t in range(T):
        for r in range(R):
            for c in range((D + Z - 1) // Z):
                off, s = oracle.locate(h, t, r, c, m, Z)
                for o in range(min(Z, D - c * Z)):
                    idx[t * R + r, c * Z + o] = off + o
                    sgn[t * R + r, c * Z + o] = s
    return idx, sgn


@pytest.mark.parametrize("D,Z,sizes", [(12, 4, [0, 3, 1, 0, 0, 7, 2, 0]), (10, 4, [5, 0, 1]), (8, 8, [1, 1, 1, 4])])
def test_bag_sum_matches_stock_embedding_bag_and_autograd(D, Z, sizes):
    m, T, R, lam = 97, 3, 11, 0.6
    rng, h, M, offsets, rows, tables = setup(31 + D, D, Z, m, T, R, sizes)
    idx, sgn = position_table(h, D, Z, m, T, R)
    Mt = torch.tensor(M.astype(np.float64), requires_grad=True)
    E = lam * torch.from_numpy(sgn) * Mt[torch.from_numpy(idx)]                # the virtual tables, materialised
    flat = torch.from_numpy(tables.astype(np.int64) * R + rows)
    out_t = torch.nn.functional.embedding_bag(flat, E, torch.from_numpy(offsets), mode="sum",
                                              include_last_offset=True)
    out = oracle.embed_bag_fwd(h, D, Z, lam, rows, tables, offsets, M)
    assert out.shape == (len(sizes), D)
    np.testing.assert_allclose(out, out_t.detach().numpy(), rtol=1e-13, atol=1e-13)
    for b, sz in enumerate(sizes):
        if sz == 0:
            assert not out[b].any()

    dOut = rng.standard_normal(out.shape)
    (out_t * torch.from_numpy(dOut)).sum().backward()
    dM = oracle.embed_bag_bwd(h, D, Z, m, lam, rows, tables, offsets, dOut)
    np.testing.assert_allclose(dM, Mt.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(np.sum(dM * M), np.sum(dOut * out), rtol=1e-12)
    # accumulates into an existing gradient
    base = rng.standard_normal(m)
    dM2 = oracle.embed_bag_bwd(h, D, Z, m, lam, rows, tables, offsets, dOut, base.copy())
    np.testing.assert_allclose(dM2, base + dM, rtol=1e-12, atol=1e-12)


def test_bags_of_one_are_the_plain_lookup():
    D, Z, m = 16, 4, 200
    rng, h, M, offsets, rows, tables = setup(5, D, Z, m, 4, 1 << 30, [1] * 9)
    out = oracle.embed_bag_fwd(h, D, Z, 1.3, rows, tables, offsets, M)
    np.testing.assert_array_equal(out, oracle.embed_fwd(h, D, Z, 1.3, rows, tables, M))
    dOut = rng.standard_normal(out.shape)
    np.testing.assert_array_equal(oracle.embed_bag_bwd(h, D, Z, m, 1.3, rows, tables, offsets, dOut),
                                  oracle.embed_bwd(h, D, Z, m, 1.3, rows, tables, dOut))
