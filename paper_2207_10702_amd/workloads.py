"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random tensors, ids and hash coefficients and converts
dtypes.  It contains none of ROAST's arithmetic (no hashing, no tile lookup, no
products): the HIP library and the CPU oracle each implement those on their own,
and both are fed from here so that they see identical inputs.

All draws come from numpy's PCG64 generator (`numpy.random.default_rng(seed)`);
tensors are drawn first, hash coefficients last.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

MERSENNE31 = (1 << 31) - 1


# ----------------------------------------------------------------------------- dtypes
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array rounded to bfloat16 precision, returned as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# ----------------------------------------------------------------------------- hash coefficients
def draw_hash(rng: np.random.Generator, use_sign: bool = True, align: int = 1,
              P: int = MERSENNE31) -> Dict[str, int]:
    """Coefficients of the offset and sign hashes: multipliers in [1, P), addends in [0, P)."""
    mult = rng.integers(1, P, size=6, dtype=np.int64)
    add = rng.integers(0, P, size=2, dtype=np.int64)
    return dict(P=int(P), a0=int(mult[0]), a1=int(mult[1]), a2=int(mult[2]), a3=int(add[0]),
                s0=int(mult[3]), s1=int(mult[4]), s2=int(mult[5]), s3=int(add[1]),
                use_sign=int(bool(use_sign)), align=int(align))


def identity_hash(n_inner: int, block_len: int, P: int = MERSENNE31) -> Dict[str, int]:
    """Coefficients under which block (k1, k2) lands at (k1*n_inner + k2)*block_len with sign +1.

    Valid (no wrap-around) as long as the largest such offset is below P and M has exactly
    n_outer*n_inner*block_len entries.  For ROAST-MM, n_inner is the number of tile columns and
    block_len = Z1*Z2; for the lookup, n_inner is the chunks per row and block_len = Z."""
    return dict(P=int(P), a0=0, a1=int(n_inner * block_len), a2=int(block_len), a3=0,
                s0=0, s1=0, s2=0, s3=0, use_sign=0, align=1)


# ----------------------------------------------------------------------------- configurations
@dataclass
class MMLayer:
    name: str
    H: int
    O: int
    layer_id: int


@dataclass
class MMConfig:
    name: str
    I: int
    layers: List[MMLayer]
    Z1: int
    Z2: int
    m_size: int
    dtype: str                      # "f32" or "bf16": dtype of X / Y / dY / dX (M is always fp32)
    m_dist: Tuple[str, float]       # ("uniform", bound) or ("normal", std)
    lam: float = 1.0
    chained: bool = False           # layer k's input is layer k-1's output
    seed: int = 0

    @property
    def flop_per_pass(self) -> int:
        """FLOPs of one of fwd / dX / dM summed over the layers (2*I*H*O each)."""
        return sum(2 * self.I * l.H * l.O for l in self.layers)


@dataclass
class EmbedConfig:
    name: str
    n_tables: int
    total_rows: int
    D: int
    Z: int
    m_size: int
    batch: int
    zipf_s: float = 1.05
    table_decay: float = 0.75
    m_dist: Tuple[str, float] = ("normal", 0.02)
    lam: float = 1.0
    seed: int = 0

    @property
    def N(self) -> int:
        return self.batch * self.n_tables


def _bert_layers() -> List[MMLayer]:
    out = []
    for l in range(12):
        out += [MMLayer(f"l{l}.qkv", 768, 2304, 4 * l + 0), MMLayer(f"l{l}.out", 768, 768, 4 * l + 1),
                MMLayer(f"l{l}.ffn1", 768, 3072, 4 * l + 2), MMLayer(f"l{l}.ffn2", 3072, 768, 4 * l + 3)]
    return out


CONFIGS = {
    # 1: one fp32 layer, 16x compression, lambda = C/sqrt(n) = 16/sqrt(256) = 1
    "cfg1_single_f32": MMConfig("cfg1_single_f32", I=64, layers=[MMLayer("mm", 256, 256, 0)], Z1=32, Z2=32,
                                m_size=4096, dtype="f32", m_dist=("uniform", 1.0 / 16.0), lam=1.0),
    # 2: BERT-base FFN pair, one shared M holding 1/100 of the 4 718 592 virtual parameters
    "cfg2_bert_ffn_bf16": MMConfig("cfg2_bert_ffn_bf16", I=8192,
                                   layers=[MMLayer("ffn1", 768, 3072, 0), MMLayer("ffn2", 3072, 768, 1)],
                                   Z1=64, Z2=64, m_size=4718592 // 100, dtype="bf16",
                                   m_dist=("normal", 0.02), chained=True),
    # 3: all 48 linear layers of BERT-base hashed into one M of 85 000 entries
    "cfg3_bert_stack_bf16": MMConfig("cfg3_bert_stack_bf16", I=16 * 512, layers=_bert_layers(), Z1=128, Z2=128,
                                     m_size=85000, dtype="bf16", m_dist=("normal", 0.02)),
    # 4: DLRM-shaped embedding
    "cfg4_dlrm_embed_f32": EmbedConfig("cfg4_dlrm_embed_f32", n_tables=26, total_rows=10_000_000, D=128, Z=32,
                                       m_size=1_280_000, batch=65536),
    # 5: large layer, |M| = 64 Mi entries (about 1x compression)
    "cfg5_large_bf16": MMConfig("cfg5_large_bf16", I=16384, layers=[MMLayer("mm", 4096, 16384, 0)], Z1=128,
                                Z2=128, m_size=64 * (1 << 20), dtype="bf16", m_dist=("normal", 0.02)),
}


# ----------------------------------------------------------------------------- tensors
def draw_m(rng: np.random.Generator, m_size: int, dist: Tuple[str, float]) -> np.ndarray:
    kind, p = dist
    if kind == "uniform":
        return rng.uniform(-p, p, size=m_size).astype(np.float32)
    if kind == "normal":
        return (rng.standard_normal(m_size, dtype=np.float32) * np.float32(p)).astype(np.float32)
    raise ValueError(kind)


def draw_act(rng: np.random.Generator, rows: int, cols: int, dtype: str, block_rows: int = 2048):
    """N(0,1) activations.  Returns float32 [rows, cols] for "f32", bfloat16 bit patterns (uint16) for
    "bf16".  Drawn in row blocks so that large tensors never need a float64 or second float32 copy."""
    out = np.empty((rows, cols), dtype=np.float32 if dtype == "f32" else np.uint16)
    for r0 in range(0, rows, block_rows):
        r1 = min(rows, r0 + block_rows)
        blk = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
        out[r0:r1] = blk if dtype == "f32" else f32_to_bf16_bits(blk)
    return out


def act_as_f64(a: np.ndarray) -> np.ndarray:
    """What the oracle is fed: the exact value of every stored activation, as float64."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


@dataclass
class MMInputs:
    cfg: MMConfig
    M: np.ndarray                                   # float32 [m_size]
    X: Dict[str, np.ndarray] = field(default_factory=dict)    # per layer name: [I, H]
    dY: Dict[str, np.ndarray] = field(default_factory=dict)   # per layer name: [I, O]
    hash: Optional[Dict[str, int]] = None


def make_mm_inputs(cfg: MMConfig, seed: Optional[int] = None) -> MMInputs:
    """Tensors of an MM configuration.

    One X and one dY is drawn per distinct layer shape and shared by every layer of that shape
    (this bounds memory for the 48-layer stack).  For a chained configuration only the first
    layer's X and the last layer's dY are drawn; the tensors in between are produced by the path
    under test and are not inputs."""
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    M = draw_m(rng, cfg.m_size, cfg.m_dist)
    inp = MMInputs(cfg=cfg, M=M)
    by_shape: Dict[Tuple[int, int], Tuple[np.ndarray, np.ndarray]] = {}
    if cfg.chained:
        first, last = cfg.layers[0], cfg.layers[-1]
        inp.X[first.name] = draw_act(rng, cfg.I, first.H, cfg.dtype)
        inp.dY[last.name] = draw_act(rng, cfg.I, last.O, cfg.dtype)
    else:
        for l in cfg.layers:
            if (l.H, l.O) not in by_shape:
                by_shape[(l.H, l.O)] = (draw_act(rng, cfg.I, l.H, cfg.dtype), draw_act(rng, cfg.I, l.O, cfg.dtype))
            inp.X[l.name], inp.dY[l.name] = by_shape[(l.H, l.O)]
    inp.hash = draw_hash(rng)
    return inp


@dataclass
class EmbedInputs:
    cfg: EmbedConfig
    table_rows: np.ndarray      # int64 [n_tables]: rows per table
    rows: np.ndarray            # int64 [N]: row id inside its table, lookup n = b*n_tables + t
    tables: np.ndarray          # uint32 [N]: table id of each lookup (the hash's first key)
    M: np.ndarray               # float32 [m_size]
    dOut: Optional[np.ndarray]  # float32 [N, D] or None
    hash: Dict[str, int]


def table_sizes(cfg: EmbedConfig) -> np.ndarray:
    """Rows per table proportional to decay**t, floored, remainder given to table 0."""
    w = cfg.table_decay ** np.arange(cfg.n_tables, dtype=np.float64)
    n = np.floor(cfg.total_rows * w / w.sum()).astype(np.int64)
    n = np.maximum(n, 1)
    n[0] += cfg.total_rows - n.sum()
    return n


def zipf_rows(rng: np.random.Generator, n_rows: int, s: float, count: int) -> np.ndarray:
    """`count` draws from the bounded Zipf law P(rank r) ~ r**-s over ranks 1..n_rows, by inverting
    the float64 cumulative; rank r is row r-1."""
    cdf = np.cumsum(np.arange(1, n_rows + 1, dtype=np.float64) ** (-s))
    cdf /= cdf[-1]
    r = np.searchsorted(cdf, rng.random(count), side="left")
    return np.minimum(r, n_rows - 1).astype(np.int64)


def make_embed_inputs(cfg: EmbedConfig, seed: Optional[int] = None, with_dout: bool = True,
                      batch: Optional[int] = None) -> EmbedInputs:
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    B = cfg.batch if batch is None else batch
    sizes = table_sizes(cfg)
    M = draw_m(rng, cfg.m_size, cfg.m_dist)
    rows = np.empty((B, cfg.n_tables), dtype=np.int64)
    for t in range(cfg.n_tables):
        rows[:, t] = zipf_rows(rng, int(sizes[t]), cfg.zipf_s, B)
    tables = np.tile(np.arange(cfg.n_tables, dtype=np.uint32), B)
    dOut = None
    if with_dout:
        dOut = np.empty((B * cfg.n_tables, cfg.D), dtype=np.float32)
        step = 1 << 16
        for r0 in range(0, dOut.shape[0], step):
            r1 = min(dOut.shape[0], r0 + step)
            dOut[r0:r1] = rng.standard_normal((r1 - r0, cfg.D), dtype=np.float32)
    h = draw_hash(rng)
    return EmbedInputs(cfg=cfg, table_rows=sizes, rows=rows.reshape(-1), tables=tables, M=M, dOut=dOut, hash=h)
