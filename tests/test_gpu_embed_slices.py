"""Lookup forward when M is larger than one XCD's L2: the kernel then works in slices of M (each
block of lookups is hashed by one workgroup per slice, and every workgroup writes the chunks whose
offset lies in its slice).  Element-exact against the oracle for one, four and eight slices, ragged
lookup counts, several chunks per row, and a call that is too small to be sliced."""
import numpy as np
import pytest

import oracle
from paper_2207_10702_amd import workloads as wl
from tests.util import to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.mark.parametrize("m_size,N,D,Z", [
    (2_500_000, 20_011, 128, 32),    # 10 MB: four slices; N not a multiple of 64 or 256
    (5_000_003, 16_385, 128, 32),    # 20 MB: eight slices; one lookup past a block of 256
    (1_280_000, 70_000, 64, 16),     # 5 MB (config 4's array): four slices, 4 chunks of 16
    (2_500_000, 33_000, 32, 32),     # one chunk per row
    (2_500_000, 5_000, 128, 32),     # too few chunks to slice: the plain kernel
    (800_000, 30_000, 128, 32),      # 3.2 MB: fits, one slice
    (9_000_000, 17_000, 128, 32),    # 36 MB: even an eighth does not fit, one slice
])
def test_sliced_lookup_is_exact(roast, m_size, N, D, Z):
    rng = np.random.default_rng(m_size % 1000 + N)
    h = wl.draw_hash(rng, use_sign=True, align=1)
    lam = np.float32(1.5)
    M = rng.standard_normal(m_size).astype(np.float32)
    rows = rng.integers(0, 1 << 33, N).astype(np.int64)
    tables = rng.integers(0, 26, N).astype(np.uint32)
    d = roast.embed_desc(D, Z, m_size, lam, h)
    out = roast.roast_embed_fwd(d, to_dev(rows), torch.from_numpy(tables.view(np.int32)).cuda(), to_dev(M))
    ref = oracle.embed_fwd(h, D, Z, float(lam), rows, tables, M)
    got = out.cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape
    # one fp32 multiply by +-lambda: exact in fp32, compare as such
    assert np.array_equal(got.astype(np.float32), ref.astype(np.float32))
    # and the device's own chunk map says the same
    off, sgn = roast.roast_chunk_index_device(d, to_dev(rows), torch.from_numpy(tables.view(np.int32)).cuda())
    C = D // Z
    k = int(rng.integers(0, N * C))
    o0, s0 = int(off[k].item()), int(sgn[k].item())
    assert np.array_equal(got[k // C, (k % C) * Z:(k % C + 1) * Z].astype(np.float32),
                          (np.float32(s0) * lam * M[o0:o0 + Z]).astype(np.float32))
