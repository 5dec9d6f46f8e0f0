"""ctypes front end of the CPU oracle (``rii_oracle.cpp``).

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``; the product package never imports it.  All arguments and
results are numpy arrays on the host.  See the header of ``rii_oracle.cpp`` for which passage of
the paper each routine follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rii_oracle.cpp")
_SO = os.path.join(_HERE, "librii_oracle.so")

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with the host compiler.  No fused multiply-add, no fast-math."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c++17", "-shared", "-fPIC",
               _SRC, "-o", _SO]
        subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_SO)
        _lib.orc_num_lists.restype = ctypes.c_int64
        _lib.orc_index_bytes.restype = ctypes.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int64)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def encode(cb, x):
    """Eq. (1).  cb [M][Z][Ds], x [n][D] -> codes uint8 [n][M]."""
    cb, x = _f32(cb), _f32(x)
    M, Z, Ds = cb.shape
    n, D = x.shape
    out = np.empty((n, M), dtype=np.uint8)
    _check(lib().orc_encode(_p(cb), D, M, Z, _p(x), ctypes.c_int64(n), _p(out)), "encode")
    return out


def decode(cb, codes):
    cb, codes = _f32(cb), _u8(codes)
    M, Z, Ds = cb.shape
    n = codes.shape[0]
    out = np.empty((n, M * Ds), dtype=np.float32)
    _check(lib().orc_decode(_p(cb), M * Ds, M, Z, _p(codes), ctypes.c_int64(n), _p(out)), "decode")
    return out


def lut(cb, q, f64=False):
    """Distance tables (Sec. 3).  q [Q][D] -> A [Q][M][Z] (fp32, or fp64 with ``f64``)."""
    cb, q = _f32(cb), _f32(np.atleast_2d(q))
    M, Z, Ds = cb.shape
    Q, D = q.shape
    if f64:
        out = np.empty((Q, M, Z), dtype=np.float64)
        _check(lib().orc_lut_f64(_p(cb), D, M, Z, _p(q), Q, _p(out)), "lut")
    else:
        out = np.empty((Q, M, Z), dtype=np.float32)
        _check(lib().orc_lut(_p(cb), D, M, Z, _p(q), Q, _p(out)), "lut")
    return out


def adc(A, codes, ids=None):
    """Eq. (2) for rows ``ids`` (all rows when None) with one table A [M][Z]."""
    codes = _u8(codes)
    ids = _i32(ids)
    n = codes.shape[0] if ids is None else ids.shape[0]
    M, Z = A.shape
    if A.dtype == np.float64:
        A = np.ascontiguousarray(A)
        out = np.empty(n, dtype=np.float64)
        _check(lib().orc_adc_f64(_p(A), M, Z, _p(codes), _p(ids), ctypes.c_int64(n), _p(out)), "adc")
    else:
        A = _f32(A)
        out = np.empty(n, dtype=np.float32)
        _check(lib().orc_adc(_p(A), M, Z, _p(codes), _p(ids), ctypes.c_int64(n), _p(out)), "adc")
    return out


def linear_scan(A, codes, R, S=None):
    """Alg. 1 for one table.  Returns (ids int32 [R], dist float32 [R])."""
    A, codes, S = _f32(A), _u8(codes), _i32(S)
    M, Z = A.shape
    N = codes.shape[0]
    ids = np.empty(R, dtype=np.int32)
    dist = np.empty(R, dtype=np.float32)
    nS = 0 if S is None else S.shape[0]
    _check(lib().orc_linear_scan(_p(A), M, Z, _p(codes), ctypes.c_int64(N), _p(S), ctypes.c_int64(nS), R,
                                 _p(ids), _p(dist)), "linear_scan")
    return ids, dist


def num_lists(K, L, nS):
    return int(lib().orc_num_lists(ctypes.c_int64(K), ctypes.c_int64(L), ctypes.c_int64(nS)))


def coarse_rank(A, coarse, P):
    A, coarse = _f32(A), _u8(coarse)
    M, Z = A.shape
    K = coarse.shape[0]
    ks = np.empty(P, dtype=np.int32)
    d0 = np.empty(P, dtype=np.float32)
    _check(lib().orc_coarse_rank(_p(A), M, Z, _p(coarse), K, P, _p(ks), _p(d0)), "coarse_rank")
    return ks, d0


def inverted_index(A, codes, coarse, list_off, list_ids, R, P, S=None, Lcap=0):
    """Alg. 2 for one table.  Returns (ids, dist, number of candidates scored)."""
    A, codes, coarse, S = _f32(A), _u8(codes), _u8(coarse), _i32(S)
    list_off, list_ids = _i64(list_off), _i32(list_ids)
    M, Z = A.shape
    N, K = codes.shape[0], coarse.shape[0]
    ids = np.empty(R, dtype=np.int32)
    dist = np.empty(R, dtype=np.float32)
    scored = ctypes.c_int64(0)
    nS = 0 if S is None else S.shape[0]
    _check(lib().orc_inverted_index(_p(A), M, Z, _p(codes), ctypes.c_int64(N), _p(coarse), K, _p(list_off),
                                    _p(list_ids), _p(S), ctypes.c_int64(nS), P, ctypes.c_int64(Lcap), R,
                                    _p(ids), _p(dist), ctypes.byref(scored)), "inverted_index")
    return ids, dist, scored.value


def query(cb, q, codes, coarse, list_off, list_ids, R, L, theta, S=None):
    """Alg. 3 for one query vector.  Returns (ids, dist, mode) with mode 0 = Alg. 1, 1 = Alg. 2."""
    cb, q, codes, coarse, S = _f32(cb), _f32(q), _u8(codes), _u8(coarse), _i32(S)
    list_off, list_ids = _i64(list_off), _i32(list_ids)
    M, Z, Ds = cb.shape
    N, K = codes.shape[0], coarse.shape[0]
    ids = np.empty(R, dtype=np.int32)
    dist = np.empty(R, dtype=np.float32)
    mode = ctypes.c_int(0)
    nS = 0 if S is None else S.shape[0]
    _check(lib().orc_query(_p(cb), M * Ds, M, Z, _p(q), _p(codes), ctypes.c_int64(N), _p(coarse), K,
                           _p(list_off), _p(list_ids), _p(S), ctypes.c_int64(nS), ctypes.c_int64(L),
                           ctypes.c_int64(theta), R, _p(ids), _p(dist), ctypes.byref(mode)), "query")
    return ids, dist, mode.value


def sym_table(cb):
    cb = _f32(cb)
    M, Z, Ds = cb.shape
    out = np.empty((M, Z, Z), dtype=np.float32)
    _check(lib().orc_sym_table(_p(cb), M * Ds, M, Z, _p(out)), "sym_table")
    return out


def assign(T, codes, coarse):
    """a(n) of Sec. 4.1 for every row of ``codes``."""
    T, codes, coarse = _f32(T), _u8(codes), _u8(coarse)
    M, Z, _ = T.shape
    n, K = codes.shape[0], coarse.shape[0]
    out = np.empty(n, dtype=np.int32)
    _check(lib().orc_assign(_p(T), M, Z, _p(codes), ctypes.c_int64(n), _p(coarse), K, _p(out)), "assign")
    return out


def build_lists(a, K):
    """Eq. (4) as CSR: (list_off int64 [K+1], list_ids int32 [N])."""
    a = _i32(a)
    N = a.shape[0]
    off = np.empty(K + 1, dtype=np.int64)
    ids = np.empty(N, dtype=np.int32)
    _check(lib().orc_build_lists(_p(a), ctypes.c_int64(N), K, _p(off), _p(ids)), "build_lists")
    return off, ids


def index_bytes(N, K, M):
    return int(lib().orc_index_bytes(ctypes.c_int64(N), ctypes.c_int64(K), ctypes.c_int64(M)))


def rotate(R, x):
    """Sec. 4.5: y = R x for every row of x (fp32, fixed summation order)."""
    R, x = _f32(R), _f32(np.atleast_2d(x))
    n, D = x.shape
    if R.shape != (D, D):
        raise ValueError("rotation must be D x D")
    out = np.empty((n, D), dtype=np.float32)
    _check(lib().orc_rotate(_p(R), D, _p(x), ctypes.c_int64(n), _p(out)), "rotate")
    return out
