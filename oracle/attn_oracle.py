"""ctypes front end of the float64 CPU oracle (attn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the cpu_baseline leg of
the benchmark, never by the GPU library or its Python binding.  All arrays are numpy
float64, contiguous, [batch, heads, n, d] (LSE: [batch, heads, n]); `keep` is None or an
[nblk, nblk] uint8 matrix (row = query block, column = key block) with `block` rows per
block edge.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_attn.so")

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int)
_bp = ctypes.POINTER(ctypes.c_ubyte)


def build(force=False):
    """Compile attn_oracle.c with gcc (OpenMP over independent rows / heads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("oracle_attn_fwd", "oracle_attn_bwd", "oracle_attn_bwd_head",
                     "oracle_attn_bwd_sampled", "oracle_wgrad", "oracle_small_cache_wgrad"):
            getattr(_lib, name).restype = None
    return _lib


def _d(a):
    return a.ctypes.data_as(_dp) if a is not None else None


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _mask(keep, block, n):
    if keep is None:
        return None, 1, 1, None
    keep = np.ascontiguousarray(keep, dtype=np.uint8)
    nblk = keep.shape[0]
    assert keep.shape == (nblk, nblk) and nblk * block >= n
    return keep, int(block), int(nblk), keep.ctypes.data_as(_bp)


def attn_fwd(Q, K, V, scale, causal=False, keep=None, block=1):
    """O, LSE of softmax(scale Q K^T over visible keys) V."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    b, h, n, d = Q.shape
    _keep, block, nblk, kp = _mask(keep, block, n)
    O = np.empty_like(Q)
    LSE = np.empty((b, h, n), dtype=np.float64)
    _load().oracle_attn_fwd(b, h, n, d, ctypes.c_double(scale), int(bool(causal)), block, nblk,
                            kp, _d(Q), _d(K), _d(V), _d(O), _d(LSE))
    return O, LSE


def attn_bwd(Q, K, V, O, dO, LSE, scale, causal=False, keep=None, block=1):
    """dQ, dK, dV from the given O and LSE."""
    Q, K, V, O, dO, LSE = map(_f64, (Q, K, V, O, dO, LSE))
    b, h, n, d = Q.shape
    _keep, block, nblk, kp = _mask(keep, block, n)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    _load().oracle_attn_bwd(b, h, n, d, ctypes.c_double(scale), int(bool(causal)), block, nblk,
                            kp, _d(Q), _d(K), _d(V), _d(O), _d(dO), _d(LSE), _d(dQ), _d(dK), _d(dV))
    return dQ, dK, dV


def attn_bwd_head(Q, K, V, O, dO, LSE, scale, causal=False, keep=None, block=1):
    """One head ([n, d] inputs): dQ, dK, dV and the n x n intermediates f (P), q (dP), p (dS)."""
    Q, K, V, O, dO, LSE = map(_f64, (Q, K, V, O, dO, LSE))
    n, d = Q.shape
    _keep, block, nblk, kp = _mask(keep, block, n)
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    f, q, p = (np.empty((n, n)) for _ in range(3))
    _load().oracle_attn_bwd_head(n, d, ctypes.c_double(scale), int(bool(causal)), block, nblk, kp,
                                 _d(Q), _d(K), _d(V), _d(O), _d(dO), _d(LSE), _d(dQ), _d(dK),
                                 _d(dV), _d(f), _d(q), _d(p))
    return dQ, dK, dV, f, q, p


def attn_bwd_sampled(Q, K, V, O, dO, LSE, scale, q_rows, k_rows, causal=False, keep=None, block=1):
    """One head: dQ[q_rows], dK[k_rows], dV[k_rows] only (for full-size sampled parity)."""
    Q, K, V, O, dO, LSE = map(_f64, (Q, K, V, O, dO, LSE))
    n, d = Q.shape
    _keep, block, nblk, kp = _mask(keep, block, n)
    q_rows = np.ascontiguousarray(q_rows, dtype=np.int32)
    k_rows = np.ascontiguousarray(k_rows, dtype=np.int32)
    dQ = np.empty((len(q_rows), d))
    dK = np.empty((len(k_rows), d))
    dV = np.empty((len(k_rows), d))
    _load().oracle_attn_bwd_sampled(n, d, ctypes.c_double(scale), int(bool(causal)), block, nblk,
                                    kp, _d(Q), _d(K), _d(V), _d(O), _d(dO), _d(LSE),
                                    len(q_rows), q_rows.ctypes.data_as(_ip), _d(dQ),
                                    len(k_rows), k_rows.ctypes.data_as(_ip), _d(dK), _d(dV))
    return dQ, dK, dV


def wgrad(A1, A2, A3, dO, X, Y):
    """The paper's weight gradient g = A_1^T p A_2 (d x d) and its f, q, p (n x n)."""
    A1, A2, A3, dO, X, Y = map(_f64, (A1, A2, A3, dO, X, Y))
    n, d = A1.shape
    g = np.empty((d, d))
    f, q, p = (np.empty((n, n)) for _ in range(3))
    _load().oracle_wgrad(n, d, _d(A1), _d(A2), _d(A3), _d(dO), _d(X), _d(Y), _d(g),
                         _d(f), _d(q), _d(p))
    return g, f, q, p


def small_cache_wgrad(A1, A2, A3, dO, X, Y, B):
    """The same g by the four-phase small-cache scheme over B x B blocks, and the number of
    elements it reads from / writes to memory: (g, reads, writes)."""
    A1, A2, A3, dO, X, Y = map(_f64, (A1, A2, A3, dO, X, Y))
    n, d = A1.shape
    g = np.empty((d, d))
    io = (ctypes.c_longlong * 2)(0, 0)
    _load().oracle_small_cache_wgrad(n, d, int(B), _d(A1), _d(A2), _d(A3), _d(dO), _d(X), _d(Y),
                                     _d(g), io)
    return g, int(io[0]), int(io[1])
