"""Writes the stored index maps under tests/golden/.  Calls only the CPU oracle and the seeded input
generators: no value here comes from the HIP library.  The paper prints no worked numeric example of
its maps (its Figure 1 is a drawing), so these files are not the paper's numbers; they freeze what the
oracle -- pinned elsewhere against unbounded-integer arithmetic, closed forms and library routines --
computes for the mapping of Section 4.1 ("Matrix multiplication": tile (x, y) of layer l starts at
h2(l, x, y); "Lookup": chunk c of row r of table t starts at h1(t, r, c); the sign g is described at
the end of Section 4.1), so that a later change to the oracle's arithmetic cannot go unnoticed.

Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle                                       # noqa: E402
from paper_2207_10702_amd import workloads as wl    # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def hash_line(h):
    return " ".join(f"{k}={int(h[k])}" for k in ("P", "a0", "a1", "a2", "a3", "s0", "s1", "s2", "s3", "use_sign", "align"))


def tile_file(name):
    cfg = wl.CONFIGS[name]
    h = wl.draw_hash(np.random.default_rng(cfg.seed + 1))
    layer = cfg.layers[0]
    off, sgn = oracle.tile_index(h, layer.layer_id, layer.H, layer.O, cfg.Z1, cfg.Z2, cfg.m_size)
    nty = -(-layer.O // cfg.Z2)
    with open(os.path.join(HERE, f"{name}_tile_index.txt"), "w") as f:
        f.write("# tile map of Section 4.1 (offset h2(l,x,y) in {0..|M|-Z1*Z2}, sign g(l,x,y)), from oracle.tile_index\n")
        f.write(f"# config {name}: H={layer.H} O={layer.O} Z1={cfg.Z1} Z2={cfg.Z2} |M|={cfg.m_size} layer={layer.layer_id}\n")
        f.write(f"# hash {hash_line(h)}\n# x y offset sign\n")
        for e in range(off.size):
            f.write(f"{e // nty} {e % nty} {int(off[e])} {int(sgn[e])}\n")


def chunk_file():
    # the chunk map seen through the lookup itself: with M[i] = i + 1 the forward output is
    # sign * (offset + o + 1), which shows offset and sign of every chunk
    rng = np.random.default_rng(20220710)
    h = wl.draw_hash(rng)
    D, Z, m = 16, 4, 1000
    rows = rng.integers(0, 1 << 40, 12).astype(np.int64)
    tables = rng.integers(0, 26, 12).astype(np.uint32)
    M = np.arange(1, m + 1, dtype=np.float32)
    out = oracle.embed_fwd(h, D, Z, 1.0, rows, tables, M)
    with open(os.path.join(HERE, "lookup_chunk_index.txt"), "w") as f:
        f.write("# chunk map of Section 4.1 (\"Lookup\"): offset h1(t,r,c) in {0..|M|-Z} and sign, read off oracle.embed_fwd\n")
        f.write(f"# D={D} Z={Z} |M|={m} lambda=1, M[i] = i + 1\n# hash {hash_line(h)}\n# table row chunk offset sign\n")
        for n in range(rows.size):
            for c in range(D // Z):
                v = out[n, c * Z]
                sign = 1 if v > 0 else -1
                f.write(f"{int(tables[n])} {int(rows[n])} {c} {int(round(abs(v))) - 1} {sign}\n")


if __name__ == "__main__":
    tile_file("cfg1_single_f32")
    chunk_file()
    print("wrote", sorted(p for p in os.listdir(HERE) if p.endswith(".txt")))
