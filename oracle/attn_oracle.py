"""ctypes front end of the CPU checker (oracle/attn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark.  The product package never imports it.
All arrays are host numpy float64; nothing here touches a GPU.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Iterable, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "libattn_oracle.so")

FULL, SYMMETRIC, CAUSAL = 0, 1, 2
PLAIN, NOSKIP, SKIP = 0, 1, 2


class OrcCfg(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n", C.c_int32), ("d_model", C.c_int32),
                ("n_heads", C.c_int32), ("d_k", C.c_int32), ("p", C.c_int32),
                ("scale", C.c_double), ("skip_padded_rows", C.c_int32)]


class OrcCounts(C.Structure):
    _fields_ = [("pairs_full", C.c_uint64), ("pairs_needed", C.c_uint64 * 3),
                ("pairs_scheduled", C.c_uint64 * 3), ("tiles_full", C.c_uint64),
                ("tiles_executed", C.c_uint64), ("pairs_executed", C.c_uint64)]


def build(force: bool = False) -> str:
    """Compile the checker with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        dp = C.POINTER(C.c_double)
        ip = C.POINTER(C.c_int32)
        _lib.attn_oracle_forward.restype = C.c_int
        _lib.attn_oracle_forward.argtypes = [C.POINTER(OrcCfg), dp, dp, dp, dp, C.c_int, ip, C.c_int, dp, dp]
        _lib.attn_oracle_head_rows.restype = C.c_int
        _lib.attn_oracle_head_rows.argtypes = [C.POINTER(OrcCfg), dp, dp, dp, dp, C.c_int, ip,
                                               C.c_int, C.c_int, C.c_int, ip, dp]
        _lib.attn_oracle_counts.restype = C.c_int
        _lib.attn_oracle_counts.argtypes = [C.POINTER(OrcCfg), C.c_int, ip, C.POINTER(OrcCounts)]
        _lib.attn_oracle_ring_cycles.restype = C.c_int64
        _lib.attn_oracle_ring_cycles.argtypes = [C.c_int, C.c_int, C.c_int]
        _lib.attn_oracle_num_threads.restype = C.c_int
    return _lib


def _dptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _iptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _cfg(batch, n, d_model, n_heads, d_k, p, scale, skip_padded_rows=False) -> OrcCfg:
    return OrcCfg(batch, n, d_model, n_heads, d_k, p, float(scale), 1 if skip_padded_rows else 0)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle returned {code}")
        self.code = code


def forward(X, Wq, Wk, Wv, *, n_heads: int, d_k: int, p: int, scheme: int, scale: float,
            lens=None, variant: int = PLAIN, return_weights: bool = False, skip_padded_rows: bool = False):
    """out [B,n,H*d_k] (and weights [B,H,n,n] if asked) in float64."""
    X = _f64(X)
    B, n, D = X.shape
    Wq, Wk, Wv, lens = _f64(Wq), _f64(Wk), _f64(Wv), _i32(lens)
    cfg = _cfg(B, n, D, n_heads, d_k, p, scale, skip_padded_rows)
    out = np.zeros((B, n, n_heads * d_k), dtype=np.float64)
    w = np.zeros((B, n_heads, n, n), dtype=np.float64) if return_weights else None
    rc = lib().attn_oracle_forward(C.byref(cfg), _dptr(X), _dptr(Wq), _dptr(Wk), _dptr(Wv),
                                   scheme, _iptr(lens), variant, _dptr(out), _dptr(w))
    if rc:
        raise OracleError(rc)
    return (out, w) if return_weights else out


def head_rows(X, Wq, Wk, Wv, *, n_heads: int, d_k: int, p: int, scheme: int, scale: float,
              b: int, h: int, rows: Sequence[int], lens=None, skip_padded_rows: bool = False) -> np.ndarray:
    """Rows `rows` of head h of batch item b: float64 [len(rows), d_k]."""
    X = _f64(X)
    B, n, D = X.shape
    Wq, Wk, Wv, lens = _f64(Wq), _f64(Wk), _f64(Wv), _i32(lens)
    cfg = _cfg(B, n, D, n_heads, d_k, p, scale, skip_padded_rows)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    out = np.zeros((len(rows), d_k), dtype=np.float64)
    rc = lib().attn_oracle_head_rows(C.byref(cfg), _dptr(X), _dptr(Wq), _dptr(Wk), _dptr(Wv),
                                     scheme, _iptr(lens), b, h, len(rows), _iptr(rows), _dptr(out))
    if rc:
        raise OracleError(rc)
    return out


def counts(*, batch: int, n: int, n_heads: int, p: int, scheme: int, lens=None,
           d_model: int = 1, d_k: int = 1, skip_padded_rows: bool = False) -> dict:
    cfg = _cfg(batch, n, d_model, n_heads, d_k, p, 1.0, skip_padded_rows)
    st = OrcCounts()
    rc = lib().attn_oracle_counts(C.byref(cfg), scheme, _iptr(_i32(lens)), C.byref(st))
    if rc:
        raise OracleError(rc)
    return {"pairs_full": st.pairs_full, "pairs_needed": list(st.pairs_needed),
            "pairs_scheduled": list(st.pairs_scheduled), "tiles_full": st.tiles_full,
            "tiles_executed": st.tiles_executed, "pairs_executed": st.pairs_executed}


def ring_cycles(n: int, m: int, algo: int) -> int:
    return int(lib().attn_oracle_ring_cycles(n, m, algo))


def num_threads() -> int:
    return int(lib().attn_oracle_num_threads())
