"""ROAST CPU oracle -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to oracle/roast_oracle.c (plain C, double precision).  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product path never does.  See the header of roast_oracle.c for the
passage of the paper each function follows.
"""
from .roast_oracle import (  # noqa: F401
    OracleHash,
    locate,
    tile_index,
    element_index,
    round_bf16,
    materialize_w,
    mm_fwd,
    mm_bwd_dx,
    mm_bwd_dw,
    scatter_dm,
    mm_bwd_dm,
    dm_window,
    embed_fwd,
    embed_bwd,
    num_threads,
)
from . import optim_oracle as optim  # noqa: F401,E402
from .bag_oracle import embed_bag_fwd, embed_bag_bwd  # noqa: F401,E402
