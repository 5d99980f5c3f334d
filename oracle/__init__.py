"""fp64 CPU oracle for Local Linear Attention -- TEST INFRASTRUCTURE ONLY.

Loads ``llla_oracle.c`` (the plain normal-equations solver of the local linear regression
objective, Section 2.3 Eq. (lla_obj)) and wraps it for arrays shaped ``[B, H, n, d]``.  Nothing in
the GPU package imports this module, and this module imports nothing from it.  Callers: tests,
the smoke check, and the CPU-baseline leg of the benchmark.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "llla_oracle.c")
_LIB = os.path.join(_HERE, "libllla_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over rows).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.llla_oracle_rows.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_double, ctypes.c_double, ctypes.c_int,
                                         ip, ctypes.c_int, dp]
        lib.llla_oracle_rows.restype = ctypes.c_int
        lib.llla_oracle_rows_ex.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                            ctypes.c_double, dp, ctypes.c_double, ctypes.c_int,
                                            ip, ctypes.c_int, dp, dp, dp]
        lib.llla_oracle_rows_ex.restype = ctypes.c_int
        lib.llla_oracle_rows_cg.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                            ctypes.c_double, ctypes.c_double, ctypes.c_int, ctypes.c_int,
                                            ctypes.c_double, ip, ctypes.c_int, dp, dp, dp, ip]
        lib.llla_oracle_rows_cg.restype = ctypes.c_int
        lib.llla_oracle_decode.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_double, ctypes.c_double, dp]
        lib.llla_oracle_decode.restype = ctypes.c_int
        lib.llla_oracle_decode_batch.argtypes = [dp, dp, dp, ip, ctypes.c_int, ctypes.c_int,
                                                 ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                                 ctypes.c_double, dp]
        lib.llla_oracle_decode_batch.restype = ctypes.c_int
        lib.llla_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the row loop uses."""
    return int(_load().llla_oracle_threads())


def _f64(x) -> np.ndarray:
    """Widen the given (already rounded) inputs exactly to fp64; accepts numpy or torch."""
    if hasattr(x, "detach"):                       # torch tensor (bf16 has no numpy dtype)
        x = x.detach().cpu().double().numpy()
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def forward_head(Q, K, V, lam: float, scale: float, causal: bool = True, rows=None) -> np.ndarray:
    """One head.  Q, K: [n, d]; V: [n, dv].  Returns O[rows] as [len(rows), dv] fp64."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    n, d = Q.shape
    assert K.shape == (n, d) and V.shape[0] == n
    dv = V.shape[1]
    rows = np.arange(n, dtype=np.int32) if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    out = np.empty((len(rows), dv), dtype=np.float64)
    bad = _load().llla_oracle_rows(_dp(Q), _dp(K), _dp(V), n, d, dv, float(lam), float(scale),
                                   1 if causal else 0,
                                   rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), len(rows), _dp(out))
    if bad:
        raise FloatingPointError("oracle: %d rows had a non positive-definite normal matrix" % bad)
    return out


def forward_head_ex(Q, K, V, lam, scale: float, causal: bool = True, rows=None):
    """One head with the extras: ``lam`` a float or an [n] array of per-row ridges.  Returns
    (O [len(rows), dv], rho [len(rows), d], delta [len(rows)]) in fp64."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    n, d = Q.shape
    dv = V.shape[1]
    rows = np.arange(n, dtype=np.int32) if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    lam_rows = None if np.ndim(lam) == 0 else _f64(lam)
    assert lam_rows is None or lam_rows.shape == (n,)
    out = np.empty((len(rows), dv), dtype=np.float64)
    rho = np.empty((len(rows), d), dtype=np.float64)
    delta = np.empty((len(rows),), dtype=np.float64)
    bad = _load().llla_oracle_rows_ex(_dp(Q), _dp(K), _dp(V), n, d, dv, float(lam) if lam_rows is None else 0.0,
                                      _dp(lam_rows) if lam_rows is not None else None, float(scale),
                                      1 if causal else 0, rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                      len(rows), _dp(out), _dp(rho), _dp(delta))
    if bad:
        raise FloatingPointError("oracle: %d rows had a non positive-definite normal matrix" % bad)
    return out, rho, delta


def forward_ex(Q, K, V, lam, scale: float, causal: bool = True, rows=None):
    """Q, K, V: [B, H, n, d]; ``lam`` a float or a [B, H, n] array.  Returns (O, rho, delta) stacked over B, H."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, H = Q.shape[:2]
    lam_a = None if np.ndim(lam) == 0 else _f64(lam)
    res = [[forward_head_ex(Q[b, h], K[b, h], V[b, h], lam if lam_a is None else lam_a[b, h], scale, causal, rows)
            for h in range(H)] for b in range(B)]
    O = np.asarray([[r[0] for r in row] for row in res])
    R = np.asarray([[r[1] for r in row] for row in res])
    Dl = np.asarray([[r[2] for r in row] for row in res])
    return O, R, Dl


def forward_head_cg(Q, K, V, lam: float, scale: float, T: int, eps: float = 0.0, causal: bool = True, rows=None):
    """One head in the paper's approximate mode (T conjugate-gradient steps for rho, Appendix C).  Returns
    (O [len(rows), dv], rho [len(rows), d], delta [len(rows)], iterations used [len(rows)])."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    n, d = Q.shape
    dv = V.shape[1]
    rows = np.arange(n, dtype=np.int32) if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    out = np.empty((len(rows), dv), dtype=np.float64)
    rho = np.empty((len(rows), d), dtype=np.float64)
    delta = np.empty((len(rows),), dtype=np.float64)
    used = np.zeros((len(rows),), dtype=np.int32)
    ipp = ctypes.POINTER(ctypes.c_int)
    bad = _load().llla_oracle_rows_cg(_dp(Q), _dp(K), _dp(V), n, d, dv, float(lam), float(scale), 1 if causal else 0,
                                      int(T), float(eps), rows.ctypes.data_as(ipp), len(rows), _dp(out), _dp(rho),
                                      _dp(delta), used.ctypes.data_as(ipp))
    if bad:
        raise ValueError("oracle cg: %d bad row indices" % bad)
    return out, rho, delta, used


def forward(Q, K, V, lam: float, scale: float, causal: bool = True, rows=None) -> np.ndarray:
    """Q, K, V: [B, H, n, d].  Returns [B, H, len(rows) or n, dv] fp64."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, H = Q.shape[:2]
    outs = [[forward_head(Q[b, h], K[b, h], V[b, h], lam, scale, causal, rows) for h in range(H)]
            for b in range(B)]
    return np.asarray(outs)


def decode(q, Kc, Vc, lam: float, scale: float, seqlens=None) -> np.ndarray:
    """q: [B, H, d]; Kc, Vc: [B, H, L_max, d] caches holding the new token as entry seqlens[b]-1.
    Returns [B, H, dv] fp64."""
    q, Kc, Vc = _f64(q), _f64(Kc), _f64(Vc)
    B, H, Lmax, d = Kc.shape
    dv = Vc.shape[-1]
    lens = np.full(B * H, Lmax, dtype=np.int32)
    if seqlens is not None:
        lens = np.repeat(np.asarray(seqlens, dtype=np.int32), H)
    out = np.empty((B, H, dv), dtype=np.float64)
    bad = _load().llla_oracle_decode_batch(
        _dp(q), _dp(Kc), _dp(Vc), lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
        B * H, Lmax, d, dv, float(lam), float(scale), _dp(out))
    if bad:
        raise FloatingPointError("oracle decode: %d heads not positive definite / bad length" % bad)
    return out
