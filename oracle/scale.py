"""ctypes front end of the plain-C oracle (``xfbq_oracle.c``).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Holds no arithmetic of
its own beyond re-viewing the C oracle's 64-bit plane words as the 32-bit
exchange layout.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "xfbq_oracle.c")
_LIB = os.path.join(_HERE, "libxfbq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-mpopcnt", "-shared", "-fPIC",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, vp, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_float
        lib.xfbq_oracle_threads.restype = i32
        lib.xfbq_oracle_quantize.argtypes = [vp, i64, i32, i32, f32, vp]
        lib.xfbq_oracle_quantize.restype = None
        lib.xfbq_oracle_pack.argtypes = [vp, i64, i32, i32, vp]
        lib.xfbq_oracle_pack.restype = None
        lib.xfbq_oracle_scores.argtypes = [vp, i64, i32, vp, i64, i32, i32, vp]
        lib.xfbq_oracle_scores.restype = None
        lib.xfbq_oracle_scores_at.argtypes = [vp, i32, vp, i32, i32, vp, vp, i64, vp]
        lib.xfbq_oracle_scores_at.restype = None
        lib.xfbq_oracle_search.argtypes = [vp, i64, i32, vp, i64, i32, i32, i32, vp, vp]
        lib.xfbq_oracle_search.restype = i32
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(_load().xfbq_oracle_threads())


def quantize(X: np.ndarray, B: int, scale: float = 1.0) -> np.ndarray:
    """fp32 [n, d] -> per-coordinate codes uint8 [n, d]."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    n, d = X.shape
    codes = np.empty((n, d), dtype=np.uint8)
    _load().xfbq_oracle_quantize(_p(X), n, d, B, float(np.float32(scale)), _p(codes))
    return codes


def pack(codes: np.ndarray, B: int) -> np.ndarray:
    """codes uint8 [n, d] -> planes uint64 [n, B, ceil(d/64)]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    n, d = codes.shape
    planes = np.empty((n, B, (d + 63) // 64), dtype=np.uint64)
    _load().xfbq_oracle_pack(_p(codes), n, d, B, _p(planes))
    return planes


def encode(X: np.ndarray, B: int, scale: float = 1.0) -> np.ndarray:
    return pack(quantize(X, B, scale), B)


def planes_as_u32(planes64: np.ndarray, d: int) -> np.ndarray:
    """View [n, B, W64] uint64 planes as the exchange layout [n, B, ceil(d/32)] uint32."""
    n, B, W64 = planes64.shape
    W = (d + 31) // 32
    return np.ascontiguousarray(planes64.view("<u4").reshape(n, B, 2 * W64)[:, :, :W])


def scores(db: np.ndarray, q: np.ndarray, d: int) -> np.ndarray:
    """All scores S[m, n] (int32) from uint64 planes."""
    n, Bd, _ = db.shape
    m, Bq, _ = q.shape
    S = np.empty((m, n), dtype=np.int32)
    _load().xfbq_oracle_scores(_p(db), n, Bd, _p(q), m, Bq, d, _p(S))
    return S


def scores_at(db: np.ndarray, q: np.ndarray, d: int, qi, ri) -> np.ndarray:
    """Scores of the listed (query, row) pairs."""
    qi = np.ascontiguousarray(qi, dtype=np.int64)
    ri = np.ascontiguousarray(ri, dtype=np.int64)
    S = np.empty(qi.shape[0], dtype=np.int32)
    _load().xfbq_oracle_scores_at(_p(db), db.shape[1], _p(q), q.shape[1], d, _p(qi), _p(ri),
                                  qi.shape[0], _p(S))
    return S


def search(db: np.ndarray, q: np.ndarray, d: int, K: int):
    """Top-K per query: (idx int32 [m, K], score int32 [m, K])."""
    db = np.ascontiguousarray(db)
    q = np.ascontiguousarray(q)
    n, Bd, _ = db.shape
    m, Bq, _ = q.shape
    idx = np.empty((m, K), dtype=np.int32)
    sc = np.empty((m, K), dtype=np.int32)
    rc = _load().xfbq_oracle_search(_p(db), n, Bd, _p(q), m, Bq, d, K, _p(idx), _p(sc))
    if rc != 0:
        raise ValueError("xfbq_oracle_search: bad arguments")
    return idx, sc
