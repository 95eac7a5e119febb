"""ctypes wrapper over oracle/roast_oracle.c -- TEST INFRASTRUCTURE ONLY.

Every function marshals numpy arrays to the C oracle and returns float64 /
integer numpy arrays.  Hash parameters are a plain mapping with the keys
P, a0..a3, s0..s3, use_sign, align (see roast_oracle.c for their meaning).
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))


class OracleHash(C.Structure):
    _fields_ = [("P", C.c_uint64),
                ("a0", C.c_uint64), ("a1", C.c_uint64), ("a2", C.c_uint64), ("a3", C.c_uint64),
                ("s0", C.c_uint64), ("s1", C.c_uint64), ("s2", C.c_uint64), ("s3", C.c_uint64),
                ("use_sign", C.c_uint32), ("align", C.c_uint32)]


def _as_hash(h) -> OracleHash:
    if isinstance(h, OracleHash):
        return h
    return OracleHash(*(int(h[k]) for k in ("P", "a0", "a1", "a2", "a3", "s0", "s1", "s2", "s3",
                                            "use_sign", "align")))


_lib = None


def _load():
    global _lib
    if _lib is None:
        # ROAST_ORACLE_LIB lets the mutation test point the pins at a deliberately broken build.
        path = os.environ.get("ROAST_ORACLE_LIB") or _build.build(force=False)
        lib = C.CDLL(path)
        HP = C.POINTER(OracleHash)
        i64, i32, u32, u64, dbl = C.c_int64, C.c_int32, C.c_uint32, C.c_uint64, C.c_double
        vp = C.c_void_p
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = C.c_int
        lib.oracle_locate.argtypes = [HP, u64, u64, u64, i64, i64, C.POINTER(i64), C.POINTER(i32)]
        lib.oracle_tile_index.argtypes = [HP, u32, i64, i64, i32, i32, i64, vp, vp]
        lib.oracle_element_index.argtypes = [HP, u32, i32, i32, i64, i64, i64, C.POINTER(i64), C.POINTER(i32)]
        lib.oracle_round_bf16.argtypes = [dbl]
        lib.oracle_round_bf16.restype = dbl
        lib.oracle_materialize_w.argtypes = [HP, u32, i64, i64, i32, i32, i64, dbl, vp, i32, vp]
        for f in (lib.oracle_gemm_nn, lib.oracle_gemm_nt, lib.oracle_gemm_tn):
            f.argtypes = [i64, i64, i64, vp, vp, vp]
            f.restype = None
        lib.oracle_scatter_dm.argtypes = [HP, u32, i64, i64, i32, i32, i64, dbl, vp, vp]
        lib.oracle_dm_window.argtypes = [HP, u32, i64, i64, i64, i32, i32, i64, dbl, vp, vp, i64, i64, vp]
        lib.oracle_embed_fwd.argtypes = [HP, i64, i32, i64, dbl, i64, vp, vp, vp, vp]
        lib.oracle_embed_bwd.argtypes = [HP, i64, i32, i64, dbl, i64, vp, vp, vp, vp]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle: {what} rejected its arguments (block does not fit in M, or bad shape)")


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle really get (asked of the OpenMP runtime itself)."""
    return int(_load().oracle_num_threads())


def locate(h, k0, k1, k2, m_size, length):
    off, sgn = C.c_int64(), C.c_int32()
    hs = _as_hash(h)
    _check(_load().oracle_locate(C.byref(hs), int(k0), int(k1), int(k2), int(m_size), int(length),
                                 C.byref(off), C.byref(sgn)), "locate")
    return off.value, sgn.value


def tile_index(h, layer, H, O, Z1, Z2, m_size):
    ntx, nty = -(-H // Z1), -(-O // Z2)
    off = np.empty(ntx * nty, dtype=np.int64)
    sgn = np.empty(ntx * nty, dtype=np.int8)
    hs = _as_hash(h)
    _check(_load().oracle_tile_index(C.byref(hs), int(layer), H, O, Z1, Z2, int(m_size), _ptr(off), _ptr(sgn)),
           "tile_index")
    return off, sgn


def element_index(h, layer, Z1, Z2, m_size, i, j):
    idx, sgn = C.c_int64(), C.c_int32()
    hs = _as_hash(h)
    _check(_load().oracle_element_index(C.byref(hs), int(layer), Z1, Z2, int(m_size), int(i), int(j),
                                        C.byref(idx), C.byref(sgn)), "element_index")
    return idx.value, sgn.value


def round_bf16(v: float) -> float:
    return _load().oracle_round_bf16(float(v))


def materialize_w(h, layer, H, O, Z1, Z2, lam, M, round_bf16=False) -> np.ndarray:
    M = np.ascontiguousarray(M, dtype=np.float32)
    W = np.empty((H, O), dtype=np.float64)
    hs = _as_hash(h)
    _check(_load().oracle_materialize_w(C.byref(hs), int(layer), H, O, Z1, Z2, M.size, float(lam), _ptr(M),
                                        int(bool(round_bf16)), _ptr(W)), "materialize_w")
    return W


def mm_fwd(X, W) -> np.ndarray:
    X, W = _f64(X), _f64(W)
    I, H = X.shape
    O = W.shape[1]
    assert W.shape[0] == H
    Y = np.empty((I, O), dtype=np.float64)
    _load().oracle_gemm_nn(I, H, O, _ptr(X), _ptr(W), _ptr(Y))
    return Y


def mm_bwd_dx(dY, W) -> np.ndarray:
    dY, W = _f64(dY), _f64(W)
    I, O = dY.shape
    H = W.shape[0]
    assert W.shape[1] == O
    dX = np.empty((I, H), dtype=np.float64)
    _load().oracle_gemm_nt(I, H, O, _ptr(dY), _ptr(W), _ptr(dX))
    return dX


def mm_bwd_dw(X, dY) -> np.ndarray:
    X, dY = _f64(X), _f64(dY)
    I, H = X.shape
    O = dY.shape[1]
    assert dY.shape[0] == I
    dW = np.empty((H, O), dtype=np.float64)
    _load().oracle_gemm_tn(I, H, O, _ptr(X), _ptr(dY), _ptr(dW))
    return dW


def scatter_dm(h, layer, Z1, Z2, m_size, lam, dW, dM=None) -> np.ndarray:
    dW = _f64(dW)
    H, O = dW.shape
    if dM is None:
        dM = np.zeros(m_size, dtype=np.float64)
    assert dM.dtype == np.float64 and dM.size == m_size and dM.flags.c_contiguous
    hs = _as_hash(h)
    _check(_load().oracle_scatter_dm(C.byref(hs), int(layer), H, O, Z1, Z2, int(m_size), float(lam),
                                     _ptr(dW), _ptr(dM)), "scatter_dm")
    return dM


def mm_bwd_dm(h, layer, Z1, Z2, m_size, lam, X, dY, dM=None) -> np.ndarray:
    """dM (+)= scatter of lambda * sign * (X^T dY): the two oracle steps in sequence."""
    return scatter_dm(h, layer, Z1, Z2, m_size, lam, mm_bwd_dw(X, dY), dM)


def dm_window(h, layer, Z1, Z2, m_size, lam, X, dY, j0, j1) -> np.ndarray:
    X, dY = _f64(X), _f64(dY)
    I, H = X.shape
    O = dY.shape[1]
    win = np.zeros(j1 - j0, dtype=np.float64)
    hs = _as_hash(h)
    _check(_load().oracle_dm_window(C.byref(hs), int(layer), I, H, O, Z1, Z2, int(m_size), float(lam),
                                    _ptr(X), _ptr(dY), int(j0), int(j1), _ptr(win)), "dm_window")
    return win


def embed_fwd(h, D, Z, lam, rows, tables, M) -> np.ndarray:
    M = np.ascontiguousarray(M, dtype=np.float32)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    tables = np.ascontiguousarray(tables, dtype=np.uint32)
    N = rows.size
    assert tables.size == N
    out = np.empty((N, D), dtype=np.float64)
    hs = _as_hash(h)
    _check(_load().oracle_embed_fwd(C.byref(hs), D, Z, M.size, float(lam), N, _ptr(rows), _ptr(tables),
                                    _ptr(M), _ptr(out)), "embed_fwd")
    return out


def embed_bwd(h, D, Z, m_size, lam, rows, tables, dOut, dM=None) -> np.ndarray:
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    tables = np.ascontiguousarray(tables, dtype=np.uint32)
    dOut = _f64(dOut)
    N = rows.size
    assert dOut.shape == (N, D)
    if dM is None:
        dM = np.zeros(m_size, dtype=np.float64)
    assert dM.dtype == np.float64 and dM.size == m_size and dM.flags.c_contiguous
    hs = _as_hash(h)
    _check(_load().oracle_embed_bwd(C.byref(hs), D, Z, int(m_size), float(lam), N, _ptr(rows), _ptr(tables),
                                    _ptr(dOut), _ptr(dM)), "embed_bwd")
    return dM
