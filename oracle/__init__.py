"""fp64 CPU oracle for decayed causal linear attention -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the HIP binding and the
HIP binding never imports it.

``quadratic`` / ``quadratic_rows``  form 1: the definition O = ((Q K^T) .* M) V
    with M[i][j] = gamma^(i-j) for i >= j (Section 2.2, Eq. "BCMV"), in C.
``recurrent`` / ``decode_step``     form 2: the row-based algorithm
    (Appendix B.1, Alg. 1) with the discounted update of Appendix C.1, in C.
``chunked`` / ``fleet`` / ``recursion`` (numpy, :mod:`oracle.forms_np`) are further
    independent forms used to pin the first two and the chunk algebra.

Every function takes arrays that ``numpy.asarray(..., float64)`` accepts, laid out
[B, H, N, d] (gamma: [H]); states are [B, H, d, d] (row = key index, column =
value index).  ``quadratic``, ``recurrent`` and ``decode_step`` also take q, k of
rank r and v of another width dv (Section 2.2: B, C in R^(N x r), V in R^(N x d));
out is then [B, H, N, dv] and a state [B, H, r, dv].  Parity status: every function here is pinned by
``tests/test_oracle_pins.py`` (closed forms, a hand-computed case, brute force and
mutual agreement of independent forms); nothing is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

from .forms_np import chunked, fleet, recursion  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "leet_oracle.c")
_SO = os.path.join(_HERE, "libleet_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP, -O2, strict IEEE: no -ffast-math)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        lp = ctypes.POINTER(ctypes.c_long)
        lib.leet_oracle_quadratic.argtypes = [dp, dp, dp, dp, dp, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_long, ctypes.c_int]
        lib.leet_oracle_quadratic_rows.argtypes = [dp, dp, dp, dp, lp, ctypes.c_long, dp,
                                                   ctypes.c_int, ctypes.c_int, ctypes.c_long,
                                                   ctypes.c_int]
        lib.leet_oracle_recurrent.argtypes = [dp, dp, dp, dp, dp, dp, dp, ctypes.c_int,
                                              ctypes.c_int, ctypes.c_long, ctypes.c_int]
        lib.leet_oracle_decode_step.argtypes = [dp, dp, dp, dp, dp, dp, ctypes.c_int,
                                                ctypes.c_int, ctypes.c_int]
        lib.leet_oracle_quadratic_rd.argtypes = [dp, dp, dp, dp, dp, ctypes.c_int, ctypes.c_int,
                                                 ctypes.c_long, ctypes.c_int, ctypes.c_int]
        lib.leet_oracle_recurrent_rd.argtypes = [dp, dp, dp, dp, dp, dp, dp, ctypes.c_int,
                                                 ctypes.c_int, ctypes.c_long, ctypes.c_int, ctypes.c_int]
        lib.leet_oracle_decode_step_rd.argtypes = [dp, dp, dp, dp, dp, dp, ctypes.c_int,
                                                   ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.leet_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _ptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check_qkv(q, k, v, gamma):
    q, k, v, gamma = _f64(q), _f64(k), _f64(v), _f64(gamma).reshape(-1)
    if q.ndim != 4 or q.shape != k.shape or v.ndim != 4 or q.shape[:3] != v.shape[:3]:
        raise ValueError("q, k must share one [B, H, N, r] shape and v be [B, H, N, dv]")
    if gamma.shape[0] != q.shape[1]:
        raise ValueError("gamma must hold one value per head")
    return q, k, v, gamma


def max_threads() -> int:
    return int(_load().leet_oracle_max_threads())


def quadratic(q, k, v, gamma) -> np.ndarray:
    """Form 1 (Eq. "BCMV"): out[b,h,i] = sum_{j<=i} gamma_h^(i-j) (q_i . k_j) v_j."""
    q, k, v, gamma = _check_qkv(q, k, v, gamma)
    B, H, N, r = q.shape
    out = np.empty_like(v)
    rc = _load().leet_oracle_quadratic_rd(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), B, H, N, r,
                                          v.shape[3])
    if rc:
        raise RuntimeError("leet_oracle_quadratic failed")
    return out


def quadratic_rows(q, k, v, gamma, rows) -> np.ndarray:
    """Form 1 on selected rows: ``rows`` is [R, 2] of (b*H+h, i); returns [R, d]."""
    q, k, v, gamma = _check_qkv(q, k, v, gamma)
    if v.shape != q.shape:
        raise ValueError("quadratic_rows takes r = dv only")
    B, H, N, d = q.shape
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64).reshape(-1, 2))
    out = np.empty((rows.shape[0], d), dtype=np.float64)
    rc = _load().leet_oracle_quadratic_rows(
        _ptr(q), _ptr(k), _ptr(v), _ptr(gamma),
        rows.ctypes.data_as(ctypes.POINTER(ctypes.c_long)), rows.shape[0], _ptr(out), B, H, N, d)
    if rc:
        raise RuntimeError("leet_oracle_quadratic_rows failed (row out of range?)")
    return out


def recurrent(q, k, v, gamma, state_in=None) -> Tuple[np.ndarray, np.ndarray]:
    """Form 2 (Alg. 1 + Appendix C.1): returns (out [B,H,N,d], final state [B,H,d,d])."""
    q, k, v, gamma = _check_qkv(q, k, v, gamma)
    B, H, N, r = q.shape
    dv = v.shape[3]
    s_in = None
    if state_in is not None:
        s_in = _f64(state_in)
        if s_in.shape != (B, H, r, dv):
            raise ValueError("state_in must be [B, H, r, dv]")
    out = np.empty_like(v)
    s_out = np.empty((B, H, r, dv), dtype=np.float64)
    rc = _load().leet_oracle_recurrent_rd(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(s_in),
                                          _ptr(out), _ptr(s_out), B, H, N, r, dv)
    if rc:
        raise RuntimeError("leet_oracle_recurrent failed")
    return out, s_out


def decode_step(q, k, v, gamma, state) -> np.ndarray:
    """One token of form 2: q, k, v are [B, H, d]; ``state`` (float64 [B,H,d,d]) is updated in place."""
    q, k, v, gamma = _f64(q), _f64(k), _f64(v), _f64(gamma).reshape(-1)
    if q.ndim != 3 or q.shape != k.shape or v.ndim != 3 or q.shape[:2] != v.shape[:2]:
        raise ValueError("q, k must share one [B, H, r] shape and v be [B, H, dv]")
    B, H, r = q.shape
    dv = v.shape[2]
    if not (isinstance(state, np.ndarray) and state.dtype == np.float64 and state.flags.c_contiguous
            and state.shape == (B, H, r, dv)):
        raise ValueError("state must be a C-contiguous float64 [B, H, r, dv] array (updated in place)")
    out = np.empty_like(v)
    rc = _load().leet_oracle_decode_step_rd(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(state),
                                            _ptr(out), B, H, r, dv)
    if rc:
        raise RuntimeError("leet_oracle_decode_step failed")
    return out
