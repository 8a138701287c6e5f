"""ctypes front end of the CPU oracle (oracle/ws_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  Nothing in the product package imports it, and it
imports nothing from the product package.  All arithmetic is in the C file; this
module only builds the shared object (gcc), widens inputs to float64 (exact for
fp32 and bf16 values) and loops over heads.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ws_oracle.c")
_LIB = os.path.join(_HERE, "libws_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle.  No fast-math, no FMA contraction: plain IEEE f64."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        L.wso_density.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp]
        L.wso_density.restype = None
        L.wso_density_rows.argtypes = [dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, ip, ctypes.c_int, dp]
        L.wso_density_rows.restype = None
        L.wso_inverse_density.argtypes = [dp, ctypes.c_int, dp]
        L.wso_inverse_density.restype = None
        L.wso_select.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, ip, dp, dp]
        L.wso_select.restype = ctypes.c_int
        L.wso_select_verify.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                        ip, ip, dp]
        L.wso_select_verify.restype = ctypes.c_int
        L.wso_gather.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ip, ctypes.c_int,
                                 ctypes.c_void_p, ctypes.c_void_p]
        L.wso_gather.restype = None
        L.wso_attend.argtypes = [dp, dp, dp] + [ctypes.c_int] * 5 + [ctypes.c_double, dp]
        L.wso_attend.restype = ctypes.c_int
        L.wso_attention_mass.argtypes = [dp, dp] + [ctypes.c_int] * 4 + [ctypes.c_double, dp]
        L.wso_attention_mass.restype = ctypes.c_int
        L.wso_mass_to_density.argtypes = [dp, ctypes.c_int, dp]
        L.wso_mass_to_density.restype = None
        L.wso_gate.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp, ip]
        L.wso_gate.restype = None
        L.wso_rope.argtypes = [dp, ip, ctypes.c_int, ctypes.c_int, ctypes.c_double, dp]
        L.wso_rope.restype = ctypes.c_int
        L.wso_num_threads.argtypes = []
        L.wso_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def num_threads() -> int:
    return int(_load().wso_num_threads())


def density(K, sigma: float) -> np.ndarray:
    """rho [L] of one head.  K [L,d]; sigma > 0."""
    K = _f64(K)
    L, d = K.shape
    rho = np.empty(L, dtype=np.float64)
    _load().wso_density(_dp(K), L, d, float(sigma), _dp(rho))
    return rho


def density_rows(K, sigma: float, rows) -> np.ndarray:
    """rho at the given rows only (same arithmetic as density)."""
    K = _f64(K)
    L, d = K.shape
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    out = np.empty(rows.shape[0], dtype=np.float64)
    _load().wso_density_rows(_dp(K), L, d, float(sigma), _ip(rows), rows.shape[0], _dp(out))
    return out


def inverse_density(rho) -> np.ndarray:
    rho = _f64(rho)
    u = np.empty_like(rho)
    _load().wso_inverse_density(_dp(rho), rho.shape[0], _dp(u))
    return u


def select(K, rho, k: int, alpha: float):
    """Greedy landmark choice of one head -> (idx [k] int32, score [k], gap [k])."""
    K = _f64(K)
    rho = _f64(rho)
    L, d = K.shape
    idx = np.empty(k, dtype=np.int32)
    score = np.empty(k, dtype=np.float64)
    gap = np.empty(k, dtype=np.float64)
    rc = _load().wso_select(_dp(K), _dp(rho), L, d, int(k), float(alpha), _ip(idx), _dp(score), _dp(gap))
    if rc != 0:
        raise ValueError("wso_select rejected its arguments")
    return idx, score, gap


def select_verify(K, rho, k: int, alpha: float, cand):
    """Replay the greedy rule along cand's own prefix.

    Returns (n_forks, oracle_pick [k], deficit [k]); see ws_oracle.c."""
    K = _f64(K)
    rho = _f64(rho)
    L, d = K.shape
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    pick = np.empty(k, dtype=np.int32)
    deficit = np.zeros(k, dtype=np.float64)
    rc = _load().wso_select_verify(_dp(K), _dp(rho), L, d, int(k), float(alpha), _ip(cand), _ip(pick), _dp(deficit))
    if rc == -1:
        raise ValueError("wso_select_verify rejected its arguments")
    return rc, pick, deficit


def gather(K, V, idx):
    """Bit copy of rows idx of K and V (any dtype, [L,d]) -> (Ks, Vs) [k,d]."""
    K = np.ascontiguousarray(K)
    V = np.ascontiguousarray(V)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    k = idx.shape[0]
    Ks = np.empty((k, K.shape[1]), dtype=K.dtype)
    Vs = np.empty((k, V.shape[1]), dtype=V.dtype)
    _load().wso_gather(K.ctypes.data, V.ctypes.data, K.shape[1] * K.itemsize, _ip(idx), k,
                       Ks.ctypes.data, Vs.ctypes.data)
    return Ks, Vs


def attend(Q, Ks, Vs, scale: float | None = None) -> np.ndarray:
    """Q [N,Hq,d], Ks,Vs [Hkv,k,d] -> O [N,Hq,d] float64."""
    Q = _f64(Q)
    Ks = _f64(Ks)
    Vs = _f64(Vs)
    N, Hq, d = Q.shape
    Hkv, k, _ = Ks.shape
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    O = np.empty((N, Hq, d), dtype=np.float64)
    rc = _load().wso_attend(_dp(Q), _dp(Ks), _dp(Vs), N, Hq, Hkv, k, d, float(scale), _dp(O))
    if rc != 0:
        raise ValueError("wso_attend rejected its arguments")
    return O


def attention_mass(K, Q, scale: float | None = None) -> np.ndarray:
    """One layer: K [Hkv,L,d], Q [Hq,d] -> A [L] (sum over query heads of the softmax over tokens)."""
    K = _f64(K)
    Q = _f64(Q)
    Hkv, L, d = K.shape
    Hq = Q.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    A = np.empty(L, dtype=np.float64)
    rc = _load().wso_attention_mass(_dp(K), _dp(Q), Hkv, Hq, L, d, float(scale), _dp(A))
    if rc != 0:
        raise ValueError("wso_attention_mass rejected its arguments")
    return A


def mass_to_density(A) -> np.ndarray:
    A = _f64(A)
    rho = np.empty_like(A)
    _load().wso_mass_to_density(_dp(A), A.shape[0], _dp(rho))
    return rho


def gate(hmain, T, theta: float):
    """hmain [dm], T [N,dm] -> (score [N] float64, accept [N] int32)."""
    hmain = _f64(hmain)
    T = _f64(T)
    N, dm = T.shape
    score = np.empty(N, dtype=np.float64)
    accept = np.empty(N, dtype=np.int32)
    _load().wso_gate(_dp(hmain), _dp(T), N, dm, float(theta), _dp(score), _ip(accept))
    return score, accept


def rope(X, pos, base: float = 10000.0) -> np.ndarray:
    """X [m,d], pos [m] -> rows rotated at their virtual positions, float64."""
    X = _f64(X)
    m, d = X.shape
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    Y = np.empty_like(X)
    rc = _load().wso_rope(_dp(X), _ip(pos), m, d, float(base), _dp(Y))
    if rc != 0:
        raise ValueError("wso_rope rejected its arguments")
    return Y


if __name__ == "__main__":
    print(build(force=True))
