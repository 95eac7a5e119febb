"""CPU oracle for the pooled (bag-sum) ROAST lookup -- TEST INFRASTRUCTURE ONLY.

The lookup operation L of Section 4.1 of arXiv 2207.10702 recovers one row per id; a pooled lookup
returns, per bag, the sum of the rows of the bag's ids (the multi-hot / "gather-sum" use of an
embedding table).  Nothing new is hashed: both functions are the plain definition on top of the
per-lookup oracle, in float64, with no blocking or reordering.

  forward : out[b, :] = sum over n in [bag_offsets[b], bag_offsets[b+1]) of L(rows[n], tables[n])
  backward: the gradient of a sum hands every term the gradient of the sum, so lookup n of bag b
            scatters dOut[b, :] exactly as the per-lookup gradient of Section 4.3 would scatter its
            own row.

bag_offsets has B + 1 entries, starts at 0, is non-decreasing and ends at N (an empty bag yields a
zero row and no gradient).  Pinned in tests/test_bag_oracle_pins.py against the stock CPU
embedding-bag operator applied to a materialised table, and against automatic differentiation.
"""
import numpy as np

from . import roast_oracle as _ro


def _offsets(bag_offsets, N):
    off = np.ascontiguousarray(bag_offsets, dtype=np.int64)
    assert off.ndim == 1 and off.size >= 1 and off[0] == 0 and off[-1] == N and np.all(np.diff(off) >= 0)
    return off


def embed_bag_fwd(h, D, Z, lam, rows, tables, bag_offsets, M) -> np.ndarray:
    rows = np.asarray(rows)
    off = _offsets(bag_offsets, rows.size)
    per_lookup = _ro.embed_fwd(h, D, Z, lam, rows, tables, M)          # N x D, float64
    out = np.zeros((off.size - 1, D), dtype=np.float64)
    for b in range(off.size - 1):
        for n in range(off[b], off[b + 1]):
            out[b] += per_lookup[n]
    return out


def embed_bag_bwd(h, D, Z, m_size, lam, rows, tables, bag_offsets, dOut, dM=None) -> np.ndarray:
    rows = np.asarray(rows)
    off = _offsets(bag_offsets, rows.size)
    dOut = np.asarray(dOut, dtype=np.float64)
    assert dOut.shape == (off.size - 1, D)
    per_lookup = np.empty((rows.size, D), dtype=np.float64)
    for b in range(off.size - 1):
        per_lookup[off[b]:off[b + 1]] = dOut[b]
    return _ro.embed_bwd(h, D, Z, m_size, lam, rows, tables, per_lookup, dM)
