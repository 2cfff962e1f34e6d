"""ctypes front end of the fp64 C oracle (ragc_oracle.c) plus the route that
recomputes the whole sequence.  Test infrastructure only.

Two routes that must agree:
  * `prefill_attn`  -- the row-wise definition, in C (Sec. 3.2 "Full prefill
    computation": only the request tokens are computed, over cached K/V);
  * `prefill_attn_full_recompute` -- numpy causal attention over ALL P+N
    positions, keeping the last N rows: the statement that caching changes
    nothing (Sec. 9) written as code.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ragc_oracle.c")
_LIB = os.path.join(_HERE, "libragc_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.ragc_oracle_prefill_attn.restype = ctypes.c_int
        lib.ragc_oracle_prefill_attn.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                 ctypes.c_int, ctypes.c_double, ctypes.POINTER(ctypes.c_int),
                                                 ctypes.c_long, dp, dp, ctypes.c_int]
        lib.ragc_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().ragc_oracle_max_threads())


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def prefill_attn(q: np.ndarray, k_full: np.ndarray, v_full: np.ndarray, prefix_len: int, scale: float,
                 rows: Optional[Sequence[Tuple[int, int]]] = None, threads: int = 0,
                 return_weight_sums: bool = False):
    """q [N,Hq,D], k_full/v_full [P+N,Hkv,D] (float64).  Returns out [N,Hq,D], or
    [n_rows,D] when `rows` (pairs (i,h)) selects rows."""
    q = np.ascontiguousarray(q, np.float64)
    k_full = np.ascontiguousarray(k_full, np.float64)
    v_full = np.ascontiguousarray(v_full, np.float64)
    N, Hq, D = q.shape
    L, Hkv, D2 = k_full.shape
    assert D2 == D and v_full.shape == k_full.shape and L == prefix_len + N
    if rows is None:
        out = np.zeros((N, Hq, D), np.float64)
        n_rows, rows_p = N * Hq, None
    else:
        ra = np.ascontiguousarray(np.asarray(rows, np.int32).reshape(-1, 2))
        n_rows = ra.shape[0]
        rows_p = ra.ctypes.data_as(ctypes.POINTER(ctypes.c_int))
        out = np.zeros((n_rows, D), np.float64)
    ws = np.zeros(max(n_rows, 1), np.float64)
    if threads <= 0:
        threads = max_threads()
    rc = _load().ragc_oracle_prefill_attn(_dptr(q), _dptr(k_full), _dptr(v_full), int(prefix_len), int(N), int(Hq),
                                          int(Hkv), int(D), float(scale), rows_p, n_rows, _dptr(out), _dptr(ws),
                                          int(threads))
    if rc != 0:
        raise RuntimeError(f"ragc_oracle_prefill_attn failed: {rc}")
    if return_weight_sums:
        return out, ws[:n_rows]
    return out


def causal_attention_all_positions(q_all: np.ndarray, k_full: np.ndarray, v_full: np.ndarray, scale: float) -> np.ndarray:
    """Plain causal attention of a whole sequence, [L,Hq,D] -> [L,Hq,D], numpy fp64:
    scores as one matrix per head, lower-triangular visibility, softmax, times V."""
    L, Hq, D = q_all.shape
    Hkv = k_full.shape[1]
    G = Hq // Hkv
    out = np.zeros((L, Hq, D), np.float64)
    visible = np.tril(np.ones((L, L), bool))
    for h in range(Hq):
        g = h // G
        s = scale * (q_all[:, h, :] @ k_full[:, g, :].T)
        s = np.where(visible, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        e = np.exp(s)
        w = e / e.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ v_full[:, g, :]
    return out


def prefill_attn_full_recompute(q: np.ndarray, k_full: np.ndarray, v_full: np.ndarray, prefix_len: int,
                                scale: float, q_prefix: Optional[np.ndarray] = None) -> np.ndarray:
    """Full recomputation over [prefix || new]; the queries of the prefix positions
    are whatever the caller supplies (they cannot influence the last N rows)."""
    N, Hq, D = q.shape
    if q_prefix is None:
        q_prefix = np.zeros((prefix_len, Hq, D), np.float64)
    q_all = np.concatenate([np.asarray(q_prefix, np.float64), np.asarray(q, np.float64)], axis=0)
    return causal_attention_all_positions(q_all, np.asarray(k_full, np.float64), np.asarray(v_full, np.float64), scale)[prefix_len:]
