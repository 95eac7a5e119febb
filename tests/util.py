"""Helpers shared by the GPU parity tests: re-exported from the package (bench.py and the smoke check
use the same error metric and host <-> device conversions, and must not depend on this folder)."""
from paper_2207_10702_amd.checks import BF16_TOL, F32_TOL, rel_err, to_dev, to_host_f64  # noqa: F401
