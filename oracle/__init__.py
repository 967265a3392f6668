"""CPU oracle for the md_hom hot path -- TEST INFRASTRUCTURE, not product code.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg
may import this package.  It holds

* ``mdh_oracle.c``  plain nested-loop C (fp64 / int32) for the four instances,
* ``mdhom.py``      a generic from-the-definition md_hom evaluator (tiny spaces),
* ``instances.py``  the four instances written as  out_view . md_hom . inp_view
                    with the generic evaluator (brute-force cross-check).

The functions below are thin numpy wrappers over the C library; they compile it
with gcc on first use (``build()``), and never touch the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mdh_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_i64 = ctypes.c_int64
_i32 = ctypes.c_int32
_fp = ctypes.c_float


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O3 -march=native -fopenmp)."""
    global _lib
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O3", "-march=native", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
        _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32a(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64a(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def dot(x, y):
    x, y = _f32(x).ravel(), _f32(y).ravel()
    assert x.shape == y.shape
    out = ctypes.c_double()
    outabs = ctypes.c_double()
    _load().oracle_dot(_i64(len(x)), _p(x), _p(y), ctypes.byref(out), ctypes.byref(outabs))
    return out.value, outabs.value


def scan_rows(X, with_abs: bool = False):
    """Row-wise inclusive prefix sums in fp64 of an fp32 matrix (rows x n)."""
    X = _f32(X)
    if X.ndim == 1:
        X = X[None, :]
    R, n = X.shape
    out = np.empty((R, n), dtype=np.float64)
    outabs = np.empty((R, n), dtype=np.float64) if with_abs else None
    _load().oracle_scan_rows(_i64(R), _i64(n), _p(X), _p(out), _p(outabs) if with_abs else None)
    return (out, outabs) if with_abs else out


def matvec(A, x, with_abs: bool = False):
    A, x = _f32(A), _f32(x).ravel()
    M, K = A.shape
    assert len(x) == K
    y = np.empty(M, dtype=np.float64)
    yabs = np.empty(M, dtype=np.float64) if with_abs else None
    _load().oracle_matvec(_i64(M), _i64(K), _p(A), _p(x), _p(y), _p(yabs) if with_abs else None)
    return (y, yabs) if with_abs else y


def matmul(A, B, with_abs: bool = False):
    A, B = _f32(A), _f32(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    C = np.empty((M, N), dtype=np.float64)
    Cabs = np.empty((M, N), dtype=np.float64) if with_abs else None
    _load().oracle_matmul(_i64(M), _i64(N), _i64(K), _p(A), _p(B), _p(C), _p(Cabs) if with_abs else None)
    return (C, Cabs) if with_abs else C


def matmul_at(A, B, is_, js):
    A, B = _f32(A), _f32(B)
    M, K = A.shape
    _, N = B.shape
    is_, js = _i64a(is_), _i64a(js)
    out = np.empty(len(is_), dtype=np.float64)
    outabs = np.empty(len(is_), dtype=np.float64)
    _load().oracle_matmul_at(_i64(M), _i64(N), _i64(K), _p(A), _p(B), _i64(len(is_)), _p(is_), _p(js), _p(out), _p(outabs))
    return out, outabs


def jacobi3d(x, c0, c1):
    x = _f32(x)
    nx, ny, nz = (s - 2 for s in x.shape)
    out = np.empty((nx, ny, nz), dtype=np.float64)
    _load().oracle_jacobi3d(_i64(nx), _i64(ny), _i64(nz), _p(x), _p(out), _fp(c0), _fp(c1))
    return out


def mcc(x, filt, stride=(1, 1), with_abs: bool = False):
    x, filt = _f32(x), _f32(filt)
    N, H, W, C = x.shape
    K, R, S, C2 = filt.shape
    assert C == C2
    sh, sw = stride
    P, Q = (H - R) // sh + 1, (W - S) // sw + 1
    out = np.empty((N, P, Q, K), dtype=np.float64)
    outabs = np.empty((N, P, Q, K), dtype=np.float64) if with_abs else None
    _load().oracle_mcc(_i64(N), _i64(H), _i64(W), _i64(C), _i64(K), _i64(R), _i64(S), _i64(sh), _i64(sw),
                       _p(x), _p(filt), _p(out), _p(outabs) if with_abs else None)
    return (out, outabs) if with_abs else out


def mcc_at(x, filt, idx, stride=(1, 1)):
    x, filt = _f32(x), _f32(filt)
    N, H, W, C = x.shape
    K, R, S, _ = filt.shape
    sh, sw = stride
    idx = _i64a(idx).reshape(-1, 4)
    out = np.empty(len(idx), dtype=np.float64)
    outabs = np.empty(len(idx), dtype=np.float64)
    _load().oracle_mcc_at(_i64(N), _i64(H), _i64(W), _i64(C), _i64(K), _i64(R), _i64(S), _i64(sh), _i64(sw),
                          _p(x), _p(filt), _i64(len(idx)), _p(idx), _p(out), _p(outabs))
    return out, outabs


def mcc_capsule(x, filt, stride=(1, 1), with_abs: bool = False):
    """x: (N,H,W,C,MI,MK), filt: (K,R,S,C,MK,MJ) -> (N,P,Q,K,MI,MJ)."""
    x, filt = _f32(x), _f32(filt)
    N, H, W, C, MI, MK = x.shape
    K, R, S, C2, MK2, MJ = filt.shape
    assert C == C2 and MK == MK2
    sh, sw = stride
    P, Q = (H - R) // sh + 1, (W - S) // sw + 1
    out = np.empty((N, P, Q, K, MI, MJ), dtype=np.float64)
    outabs = np.empty(out.shape, dtype=np.float64) if with_abs else None
    _load().oracle_mcc_capsule(_i64(N), _i64(H), _i64(W), _i64(C), _i64(K), _i64(R), _i64(S), _i64(sh), _i64(sw),
                               _i64(MI), _i64(MJ), _i64(MK), _p(x), _p(filt), _p(out), _p(outabs) if with_abs else None)
    return (out, outabs) if with_abs else out


def mcc_capsule_at(x, filt, idx, stride=(1, 1)):
    """The same definition at chosen output positions idx = (n,p,q,k,mi,mj) rows."""
    x, filt = _f32(x), _f32(filt)
    N, H, W, C, MI, MK = x.shape
    K, R, S, _, _, MJ = filt.shape
    sh, sw = stride
    idx = _i64a(idx).reshape(-1, 6)
    out = np.empty(len(idx), dtype=np.float64)
    outabs = np.empty(len(idx), dtype=np.float64)
    _load().oracle_mcc_capsule_at(_i64(H), _i64(W), _i64(C), _i64(R), _i64(S), _i64(sh), _i64(sw), _i64(MI), _i64(MJ),
                                  _i64(MK), _p(x), _p(filt), _i64(len(idx)), _p(idx), _p(out), _p(outabs))
    return out, outabs


def custom_reduce(A, B, w_agree, w_disagree):
    A, B, wp, wm = _i32a(A), _i32a(B), _i32a(w_agree), _i32a(w_disagree)
    nA, nF = A.shape
    nB, nF2 = B.shape
    assert nF == nF2 == len(wp) == len(wm) and nB >= 1
    score = np.empty(nA, dtype=np.int32)
    index = np.empty(nA, dtype=np.int32)
    _load().oracle_custom_reduce(_i64(nA), _i64(nB), _i32(nF), _p(A), _p(B), _p(wp), _p(wm), _p(score), _p(index))
    return score, index


def custom_reduce_rows(A, B, w_agree, w_disagree, rows):
    A, B, wp, wm = _i32a(A), _i32a(B), _i32a(w_agree), _i32a(w_disagree)
    nA, nF = A.shape
    nB, _ = B.shape
    rows = _i64a(rows)
    score = np.empty(len(rows), dtype=np.int32)
    index = np.empty(len(rows), dtype=np.int32)
    _load().oracle_custom_reduce_rows(_i64(nA), _i64(nB), _i32(nF), _p(A), _p(B), _p(wp), _p(wm),
                                      _i64(len(rows)), _p(rows), _p(score), _p(index))
    return score, index


def histo(elems, bins):
    """Histo (md_hom(f_Histo, (++, +)) over (bins, elements)): out[b] = number of elements equal to
    bins[b], as int64."""
    elems, bins = _i32a(elems), _i32a(bins)
    out = np.empty(len(bins), dtype=np.int64)
    _load().oracle_histo(_i64(len(bins)), _i64(len(elems)), _p(elems), _p(bins), _p(out))
    return out


def maxidx_combine(s1, b1, s2, b2):
    s1, b1 = _i32a(s1).copy(), _i32a(b1).copy()
    s2, b2 = _i32a(s2), _i32a(b2)
    _load().oracle_maxidx_combine(_i64(len(s1)), _p(s1), _p(b1), _p(s2), _p(b2))
    return s1, b1
