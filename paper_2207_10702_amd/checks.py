"""Error metric, tolerances and host <-> device conversions used by the parity tests, the smoke check
and bench.py (no ROAST arithmetic here)."""
import numpy as np

F32_TOL = 1e-5     # fp32 path: max relative error per output tensor
BF16_TOL = 2e-2    # bf16 activations, fp32 accumulation


def rel_err(got, ref) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, rms(ref)): relative error with a floor at the tensor's rms,
    so that entries that happen to be near zero do not blow the ratio up."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))


def to_dev(a: np.ndarray):
    """numpy -> device tensor; uint16 arrays are bfloat16 bit patterns."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    return torch.from_numpy(a).cuda()


def to_host_f64(t) -> np.ndarray:
    """device tensor -> float64 numpy (exact for fp32 and bf16)."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    return t.cpu().numpy().astype(np.float64)
