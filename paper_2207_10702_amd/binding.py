"""Python names for the C-ABI of libroast_hip.so (see include/roast.h).

Argument marshalling only: every function checks dtypes / contiguity, passes raw device pointers
and the current HIP stream to the library, and raises RoastError on a non-zero status.  There is no
fallback: if the library has not been built, loading fails.
"""
import ctypes as C
import os
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libroast_hip.so")

ROAST_F32, ROAST_BF16 = 0, 1
ROAST_OK, ROAST_ERR_ARG, ROAST_ERR_SHAPE, ROAST_ERR_RANGE, ROAST_ERR_WORKSPACE, ROAST_ERR_HIP, ROAST_ERR_UNSUPPORTED = range(7)
ROAST_REDUCE_ATOMIC, ROAST_REDUCE_DETERMINISTIC = 0, 1

EXPORTS = ["roast_status_string", "roast_tile_index", "roast_tile_index_device", "roast_chunk_index_device",
           "roast_m_shadow_bytes", "roast_m_shadow_bf16", "roast_m_planes_bytes", "roast_m_planes_bf16",
           "roast_mm_fwd", "roast_mm_bwd_dx",
           "roast_mm_fwd_workspace", "roast_mm_bwd_dx_workspace", "roast_mm_fwd_ws", "roast_mm_bwd_dx_ws",
           "roast_mm_strip_blocks", "roast_mm_bwd_dM_workspace", "roast_mm_bwd_dM_workspace_f32", "roast_mm_bwd_dM",
           "roast_embed_fwd", "roast_embed_bwd_workspace", "roast_embed_bwd", "roast_embed_bwd_noalloc",
           "roast_embed_bag_fwd", "roast_embed_bag_bwd_workspace", "roast_embed_bag_bwd", "roast_optim_step"]


class RoastError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({status_string(status)})")


class RoastHash(C.Structure):
    _fields_ = [("P", C.c_uint64),
                ("a0", C.c_uint64), ("a1", C.c_uint64), ("a2", C.c_uint64), ("a3", C.c_uint64),
                ("s0", C.c_uint64), ("s1", C.c_uint64), ("s2", C.c_uint64), ("s3", C.c_uint64),
                ("use_sign", C.c_uint32), ("align", C.c_uint32)]


class RoastMMDesc(C.Structure):
    _fields_ = [("H", C.c_int64), ("O", C.c_int64), ("Z1", C.c_int32), ("Z2", C.c_int32),
                ("m_size", C.c_int64), ("layer_id", C.c_uint32), ("lam", C.c_float), ("hash", RoastHash)]


class RoastEmbedDesc(C.Structure):
    _fields_ = [("D", C.c_int64), ("Z", C.c_int32), ("m_size", C.c_int64), ("lam", C.c_float),
                ("hash", RoastHash)]


class RoastOptimDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("weight_decay", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float), ("step", C.c_int64), ("zero_grad", C.c_uint32)]


ROAST_OPT_SGD, ROAST_OPT_ADAGRAD, ROAST_OPT_ADAM = 0, 1, 2

_lib = None


def load() -> C.CDLL:
    """Load the in-tree library (building it first only if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("ROAST_HIP_LIB", LIB_PATH)     # override: point at another build of the same library
    # PyTorch-ROCm ships its own HIP runtime.  If this library were loaded first it would bring in the
    # system's copy, and the process would hold two runtimes: kernels launched through one on
    # streams and pointers of the other fail.  Importing torch first makes its runtime the one both use.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if path == LIB_PATH and not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = C.CDLL(path)
    vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
    MP, EP = C.POINTER(RoastMMDesc), C.POINTER(RoastEmbedDesc)
    lib.roast_status_string.argtypes = [i32]
    lib.roast_status_string.restype = C.c_char_p
    lib.roast_tile_index.argtypes = [MP, vp, vp]
    lib.roast_tile_index_device.argtypes = [MP, vp, vp, vp]
    lib.roast_chunk_index_device.argtypes = [EP, i64, vp, vp, vp, vp, vp]
    lib.roast_m_shadow_bytes.argtypes = [i64]
    lib.roast_m_shadow_bytes.restype = C.c_size_t
    lib.roast_m_shadow_bf16.argtypes = [vp, i64, vp, vp]
    lib.roast_m_planes_bytes.argtypes = [i64]
    lib.roast_m_planes_bytes.restype = C.c_size_t
    lib.roast_m_planes_bf16.argtypes = [vp, i64, vp, vp]
    lib.roast_mm_fwd.argtypes = [MP, i32, i64, vp, i64, vp, vp, vp, i64, vp]
    lib.roast_mm_bwd_dx.argtypes = [MP, i32, i64, vp, i64, vp, vp, vp, i64, vp]
    for name in ("roast_mm_fwd_workspace", "roast_mm_bwd_dx_workspace"):
        getattr(lib, name).argtypes = [MP, i32, i64]
        getattr(lib, name).restype = sz
    lib.roast_mm_fwd_ws.argtypes = [MP, i32, i64, vp, i64, vp, vp, vp, i64, vp, sz, vp]
    lib.roast_mm_strip_blocks.argtypes = [MP, i64, i32]
    lib.roast_mm_bwd_dx_ws.argtypes = [MP, i32, i64, vp, i64, vp, vp, vp, i64, vp, sz, vp]
    lib.roast_mm_bwd_dM_workspace.argtypes = [MP, i64, i32]
    lib.roast_mm_bwd_dM_workspace.restype = sz
    lib.roast_mm_bwd_dM_workspace_f32.argtypes = [MP, i64]
    lib.roast_mm_bwd_dM_workspace_f32.restype = sz
    lib.roast_mm_bwd_dM.argtypes = [MP, i32, i64, vp, i64, vp, i64, vp, i32, vp, sz, vp]
    lib.roast_embed_fwd.argtypes = [EP, i64, vp, vp, vp, vp, vp]
    lib.roast_embed_bwd_workspace.argtypes = [EP, i64, i32]
    lib.roast_embed_bwd_workspace.restype = sz
    lib.roast_embed_bwd.argtypes = [EP, i64, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.roast_embed_bwd_noalloc.argtypes = [EP, i64, vp, vp, vp, vp, i32, vp]
    lib.roast_embed_bag_fwd.argtypes = [EP, i64, i64, vp, vp, vp, vp, vp, vp]
    lib.roast_embed_bag_bwd_workspace.argtypes = [EP, i64, i64, i32]
    lib.roast_embed_bag_bwd_workspace.restype = sz
    lib.roast_embed_bag_bwd.argtypes = [EP, i64, i64, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.roast_optim_step.argtypes = [C.POINTER(RoastOptimDesc), i64, vp, vp, vp, vp, vp, vp]
    for name in EXPORTS:
        f = getattr(lib, name)
        if name not in ("roast_status_string", "roast_m_shadow_bytes", "roast_mm_bwd_dM_workspace",
                        "roast_embed_bwd_workspace", "roast_mm_fwd_workspace", "roast_mm_bwd_dx_workspace",
                        "roast_embed_bag_bwd_workspace", "roast_mm_bwd_dM_workspace_f32", "roast_m_planes_bytes"):
            f.restype = i32
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().roast_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != 0:
        raise RoastError(status, what)


def make_hash(h: Dict[str, int]) -> RoastHash:
    return RoastHash(*(int(h[k]) for k in ("P", "a0", "a1", "a2", "a3", "s0", "s1", "s2", "s3", "use_sign", "align")))


def mm_desc(H: int, O: int, Z1: int, Z2: int, m_size: int, layer_id: int, lam: float, h: Dict[str, int]) -> RoastMMDesc:
    return RoastMMDesc(int(H), int(O), int(Z1), int(Z2), int(m_size), int(layer_id), float(lam), make_hash(h))


def embed_desc(D: int, Z: int, m_size: int, lam: float, h: Dict[str, int]) -> RoastEmbedDesc:
    return RoastEmbedDesc(int(D), int(Z), int(m_size), float(lam), make_hash(h))


# ----------------------------------------------------------------------------- tensor plumbing
def _torch():
    import torch
    return torch


def _stream(stream) -> int:
    if stream is None:
        return int(_torch().cuda.current_stream().cuda_stream)
    return int(getattr(stream, "cuda_stream", stream))


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return ROAST_F32
    if t.dtype == torch.bfloat16:
        return ROAST_BF16
    raise TypeError(f"activations must be float32 or bfloat16, got {t.dtype}")


def _mat(t, name: str) -> Tuple[int, int]:
    """Device pointer and leading dimension of a 2-D row-major (possibly row-strided) tensor."""
    if not t.is_cuda or t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be a 2-D device tensor with unit column stride")
    return t.data_ptr(), (t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0)))


def _vec(t, dtype, name: str) -> int:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor of {dtype}")
    return t.data_ptr()


# ----------------------------------------------------------------------------- entry points
def roast_tile_index(desc: RoastMMDesc) -> Tuple[np.ndarray, np.ndarray]:
    """Host evaluation of the tile -> (offset, sign) map; arrays are row-major over (x, y)."""
    ntx, nty = -(-desc.H // desc.Z1), -(-desc.O // desc.Z2)
    off = np.empty(max(ntx * nty, 0), dtype=np.int64)
    sgn = np.empty(max(ntx * nty, 0), dtype=np.int8)
    _check(load().roast_tile_index(C.byref(desc), off.ctypes.data, sgn.ctypes.data), "roast_tile_index")
    return off, sgn


def roast_tile_index_device(desc: RoastMMDesc, stream=None):
    torch = _torch()
    ntx, nty = -(-desc.H // desc.Z1), -(-desc.O // desc.Z2)
    off = torch.empty(ntx * nty, dtype=torch.int64, device="cuda")
    sgn = torch.empty(ntx * nty, dtype=torch.int8, device="cuda")
    _check(load().roast_tile_index_device(C.byref(desc), off.data_ptr(), sgn.data_ptr(), _stream(stream)),
           "roast_tile_index_device")
    return off, sgn


def roast_chunk_index_device(desc: RoastEmbedDesc, rows, table_ids, stream=None):
    torch = _torch()
    N = rows.numel()
    chunks = -(-desc.D // desc.Z)
    off = torch.empty(N * chunks, dtype=torch.int64, device="cuda")
    sgn = torch.empty(N * chunks, dtype=torch.int8, device="cuda")
    _check(load().roast_chunk_index_device(C.byref(desc), N, _vec(rows, torch.int64, "rows"),
                                           _vec(table_ids, torch.int32, "table_ids"), off.data_ptr(),
                                           sgn.data_ptr(), _stream(stream)), "roast_chunk_index_device")
    return off, sgn


def roast_m_shadow_bytes(m_size: int) -> int:
    return int(load().roast_m_shadow_bytes(int(m_size)))


def roast_m_shadow_bf16(M, shadow=None, stream=None):
    """bf16 shadow of M for the bf16 ROAST-MM kernels (make it once per update of M); a bfloat16
    tensor of roast_m_shadow_bytes(|M|) / 2 elements whose layout is private to the library."""
    torch = _torch()
    n = roast_m_shadow_bytes(M.numel()) // 2
    if shadow is None:
        shadow = torch.empty(n, dtype=torch.bfloat16, device=M.device)
    if shadow.numel() != n:
        raise ValueError("shadow must have roast_m_shadow_bytes(|M|) / 2 elements")
    _check(load().roast_m_shadow_bf16(_vec(M, torch.float32, "M"), M.numel(), _vec(shadow, torch.bfloat16, "shadow"),
                                      _stream(stream)), "roast_m_shadow_bf16")
    return shadow


def roast_m_planes_bytes(m_size: int) -> int:
    return int(load().roast_m_planes_bytes(int(m_size)))


def roast_m_planes_bf16(M, planes=None, stream=None):
    """Three bfloat16 planes of M for fp32 roast_mm_fwd / roast_mm_bwd_dx calls with a workspace
    (pass as M_bf16; make once per update of M)."""
    torch = _torch()
    n = roast_m_planes_bytes(M.numel()) // 2
    if planes is None:
        planes = torch.empty(n, dtype=torch.bfloat16, device=M.device)
    if planes.numel() != n:
        raise ValueError("planes must have roast_m_planes_bytes(|M|) / 2 elements")
    _check(load().roast_m_planes_bf16(_vec(M, torch.float32, "M"), M.numel(), _vec(planes, torch.bfloat16, "planes"),
                                      _stream(stream)), "roast_m_planes_bf16")
    return planes


def _shadow_ptr(M, M_bf16, f32: bool = False) -> int:
    """bf16 calls: the shadow made by roast_m_shadow_bf16; fp32 calls: the planes made by roast_m_planes_bf16."""
    if M_bf16 is None:
        return 0
    torch = _torch()
    want = (roast_m_planes_bytes(M.numel()) if f32 else roast_m_shadow_bytes(M.numel())) // 2
    if M_bf16.numel() != want:
        raise ValueError("M_bf16 must be the tensor made by roast_m_shadow_bf16 (bf16 calls) or "
                         "roast_m_planes_bf16 (fp32 calls) for this M")
    return _vec(M_bf16, torch.bfloat16, "M_bf16")


def _ws(ws):
    return (0, 0) if ws is None else (ws.data_ptr(), ws.numel() * ws.element_size())


def roast_mm_fwd_workspace(desc: RoastMMDesc, dtype, I: int) -> int:
    """Bytes of workspace that help roast_mm_fwd(..., ws=) at these sizes (0: none)."""
    torch = _torch()
    code = {torch.float32: ROAST_F32, torch.bfloat16: ROAST_BF16}[dtype]
    return int(load().roast_mm_fwd_workspace(C.byref(desc), code, int(I)))


def roast_mm_bwd_dx_workspace(desc: RoastMMDesc, dtype, I: int) -> int:
    torch = _torch()
    code = {torch.float32: ROAST_F32, torch.bfloat16: ROAST_BF16}[dtype]
    return int(load().roast_mm_bwd_dx_workspace(C.byref(desc), code, int(I)))


def roast_mm_strip_blocks(desc: RoastMMDesc, I: int, which: int) -> int:
    """Consecutive column blocks per workgroup in roast_mm_fwd (which = 0) / roast_mm_bwd_dx (which = 1)."""
    return int(load().roast_mm_strip_blocks(C.byref(desc), int(I), int(which)))


def roast_mm_fwd(desc: RoastMMDesc, X, M, Y=None, stream=None, M_bf16=None, ws=None):
    """`ws` (optional): uint8 device tensor of at least roast_mm_fwd_workspace(...) bytes; the call then
    goes through roast_mm_fwd_ws."""
    torch = _torch()
    I = X.shape[0]
    if X.shape[1] != desc.H:
        raise ValueError("X must be I x H")
    if Y is None:
        Y = torch.empty((I, desc.O), dtype=X.dtype, device=X.device)
    if Y.dtype != X.dtype or tuple(Y.shape) != (I, desc.O):
        raise ValueError("Y must be I x O with X's dtype")
    xp, ldx = _mat(X, "X")
    yp, ldy = _mat(Y, "Y")
    if ws is not None:
        _check(load().roast_mm_fwd_ws(C.byref(desc), _dtype_code(X), I, xp, ldx, _vec(M, torch.float32, "M"),
                                      _shadow_ptr(M, M_bf16, X.dtype == torch.float32), yp, ldy, *_ws(ws), _stream(stream)), "roast_mm_fwd_ws")
        return Y
    _check(load().roast_mm_fwd(C.byref(desc), _dtype_code(X), I, xp, ldx, _vec(M, torch.float32, "M"),
                               _shadow_ptr(M, M_bf16, X.dtype == torch.float32), yp, ldy, _stream(stream)),
           "roast_mm_fwd")
    return Y


def roast_mm_bwd_dx(desc: RoastMMDesc, dY, M, dX=None, stream=None, M_bf16=None, ws=None):
    torch = _torch()
    I = dY.shape[0]
    if dY.shape[1] != desc.O:
        raise ValueError("dY must be I x O")
    if dX is None:
        dX = torch.empty((I, desc.H), dtype=dY.dtype, device=dY.device)
    if dX.dtype != dY.dtype or tuple(dX.shape) != (I, desc.H):
        raise ValueError("dX must be I x H with dY's dtype")
    gp, ldy = _mat(dY, "dY")
    xp, ldx = _mat(dX, "dX")
    if ws is not None:
        _check(load().roast_mm_bwd_dx_ws(C.byref(desc), _dtype_code(dY), I, gp, ldy, _vec(M, torch.float32, "M"),
                                         _shadow_ptr(M, M_bf16, dY.dtype == torch.float32), xp, ldx, *_ws(ws), _stream(stream)),
               "roast_mm_bwd_dx_ws")
        return dX
    _check(load().roast_mm_bwd_dx(C.byref(desc), _dtype_code(dY), I, gp, ldy, _vec(M, torch.float32, "M"),
                                  _shadow_ptr(M, M_bf16, dY.dtype == torch.float32), xp, ldx, _stream(stream)),
           "roast_mm_bwd_dx")
    return dX


def roast_mm_bwd_dM_workspace(desc: RoastMMDesc, I: int, mode: int = ROAST_REDUCE_ATOMIC) -> int:
    return int(load().roast_mm_bwd_dM_workspace(C.byref(desc), int(I), int(mode)))


def roast_mm_bwd_dM_workspace_f32(desc: RoastMMDesc, I: int) -> int:
    return int(load().roast_mm_bwd_dM_workspace_f32(C.byref(desc), int(I)))


def roast_mm_bwd_dM(desc: RoastMMDesc, X, dY, dM, mode: int = ROAST_REDUCE_ATOMIC, ws=None, stream=None):
    """dM += gradient of this layer.  `ws` is a uint8 device tensor of at least
    roast_mm_bwd_dM_workspace(...) bytes (only the deterministic mode needs one)."""
    torch = _torch()
    I = X.shape[0]
    if X.shape[1] != desc.H or tuple(dY.shape) != (I, desc.O) or X.dtype != dY.dtype:
        raise ValueError("X must be I x H and dY I x O, same dtype")
    if dM.numel() != desc.m_size:
        raise ValueError("dM must have m_size entries")
    xp, ldx = _mat(X, "X")
    gp, ldy = _mat(dY, "dY")
    wp, wb = (0, 0) if ws is None else (ws.data_ptr(), ws.numel() * ws.element_size())
    _check(load().roast_mm_bwd_dM(C.byref(desc), _dtype_code(X), I, xp, ldx, gp, ldy,
                                  _vec(dM, torch.float32, "dM"), int(mode), wp, wb, _stream(stream)),
           "roast_mm_bwd_dM")
    return dM


def roast_embed_fwd(desc: RoastEmbedDesc, rows, table_ids, M, out=None, stream=None):
    torch = _torch()
    N = rows.numel()
    if out is None:
        out = torch.empty((N, desc.D), dtype=torch.float32, device=rows.device)
    if tuple(out.shape) != (N, desc.D):
        raise ValueError("out must be N x D")
    _check(load().roast_embed_fwd(C.byref(desc), N, _vec(rows, torch.int64, "rows"),
                                  _vec(table_ids, torch.int32, "table_ids"), _vec(M, torch.float32, "M"),
                                  _vec(out, torch.float32, "out"), _stream(stream)), "roast_embed_fwd")
    return out


def roast_embed_bwd_workspace(desc: RoastEmbedDesc, N: int, mode: int = ROAST_REDUCE_ATOMIC) -> int:
    return int(load().roast_embed_bwd_workspace(C.byref(desc), int(N), int(mode)))


def roast_embed_bwd(desc: RoastEmbedDesc, rows, table_ids, dOut, dM, mode: int = ROAST_REDUCE_ATOMIC, ws=None,
                    stream=None):
    torch = _torch()
    N = rows.numel()
    if tuple(dOut.shape) != (N, desc.D) or dM.numel() != desc.m_size:
        raise ValueError("dOut must be N x D and dM must have m_size entries")
    wp, wb = (0, 0) if ws is None else (ws.data_ptr(), ws.numel() * ws.element_size())
    _check(load().roast_embed_bwd(C.byref(desc), N, _vec(rows, torch.int64, "rows"),
                                  _vec(table_ids, torch.int32, "table_ids"), _vec(dOut, torch.float32, "dOut"),
                                  _vec(dM, torch.float32, "dM"), int(mode), wp, wb, _stream(stream)),
           "roast_embed_bwd")
    return dM


def roast_embed_bwd_noalloc(desc: RoastEmbedDesc, rows, table_ids, dOut, dM, mode: int = ROAST_REDUCE_ATOMIC,
                            stream=None):
    """roast_embed_bwd with the library's own static scratch array: no workspace, no allocation."""
    torch = _torch()
    N = rows.numel()
    if tuple(dOut.shape) != (N, desc.D) or dM.numel() != desc.m_size:
        raise ValueError("dOut must be N x D and dM must have m_size entries")
    _check(load().roast_embed_bwd_noalloc(C.byref(desc), N, _vec(rows, torch.int64, "rows"),
                                          _vec(table_ids, torch.int32, "table_ids"), _vec(dOut, torch.float32, "dOut"),
                                          _vec(dM, torch.float32, "dM"), int(mode), _stream(stream)),
           "roast_embed_bwd_noalloc")
    return dM


def roast_embed_bag_fwd(desc: RoastEmbedDesc, rows, table_ids, bag_offsets, M, out=None, stream=None):
    """Pooled lookup: out[b] = sum of the rows of the lookups [bag_offsets[b], bag_offsets[b+1])."""
    torch = _torch()
    N, B = rows.numel(), bag_offsets.numel() - 1
    if B < 0:
        raise ValueError("bag_offsets must have B + 1 entries")
    if out is None:
        out = torch.empty((B, desc.D), dtype=torch.float32, device=M.device)
    if tuple(out.shape) != (B, desc.D):
        raise ValueError("out must be B x D")
    _check(load().roast_embed_bag_fwd(C.byref(desc), N, B, _vec(rows, torch.int64, "rows"),
                                      _vec(table_ids, torch.int32, "table_ids"),
                                      _vec(bag_offsets, torch.int64, "bag_offsets"), _vec(M, torch.float32, "M"),
                                      _vec(out, torch.float32, "out"), _stream(stream)), "roast_embed_bag_fwd")
    return out


def roast_embed_bag_bwd_workspace(desc: RoastEmbedDesc, N: int, B: int, mode: int = ROAST_REDUCE_ATOMIC) -> int:
    return int(load().roast_embed_bag_bwd_workspace(C.byref(desc), int(N), int(B), int(mode)))


def roast_embed_bag_bwd(desc: RoastEmbedDesc, rows, table_ids, bag_offsets, dOut, dM, mode: int = ROAST_REDUCE_ATOMIC,
                        ws=None, stream=None):
    torch = _torch()
    N, B = rows.numel(), bag_offsets.numel() - 1
    if B < 0 or tuple(dOut.shape) != (B, desc.D) or dM.numel() != desc.m_size:
        raise ValueError("dOut must be B x D and dM must have m_size entries")
    _check(load().roast_embed_bag_bwd(C.byref(desc), N, B, _vec(rows, torch.int64, "rows"),
                                      _vec(table_ids, torch.int32, "table_ids"),
                                      _vec(bag_offsets, torch.int64, "bag_offsets"), _vec(dOut, torch.float32, "dOut"),
                                      _vec(dM, torch.float32, "dM"), int(mode), *_ws(ws), _stream(stream)),
           "roast_embed_bag_bwd")
    return dM


def optim_desc(kind: int, lr: float, weight_decay: float = 0.0, beta1: float = 0.9, beta2: float = 0.999,
               eps: float = 1e-8, step: int = 1, zero_grad: bool = True) -> RoastOptimDesc:
    return RoastOptimDesc(int(kind), float(lr), float(weight_decay), float(beta1), float(beta2), float(eps),
                          int(step), 1 if zero_grad else 0)


def roast_optim_step(desc: RoastOptimDesc, M, dM, state1=None, state2=None, M_bf16=None, stream=None):
    """One optimizer step on M (in place); clears dM when desc.zero_grad; refreshes M_bf16 when given."""
    torch = _torch()
    n = M.numel()
    if dM.numel() != n:
        raise ValueError("dM must have as many entries as M")
    ptr = lambda t, what: 0 if t is None else _vec(t, torch.float32, what)
    for t, what in ((state1, "state1"), (state2, "state2")):
        if t is not None and t.numel() != n:
            raise ValueError(f"{what} must have as many entries as M")
    _check(load().roast_optim_step(C.byref(desc), n, _vec(M, torch.float32, "M"), _vec(dM, torch.float32, "dM"),
                                   ptr(state1, "state1"), ptr(state2, "state2"), _shadow_ptr(M, M_bf16),
                                   _stream(stream)), "roast_optim_step")
    return M
