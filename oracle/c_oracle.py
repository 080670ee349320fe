"""ctypes access to the plain-C oracle (byz_oracle.c).  TEST INFRASTRUCTURE ONLY."""
import ctypes
import os

import numpy as np

from . import build_oracle

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.build()
        L = ctypes.CDLL(path)
        i32p = ctypes.POINTER(ctypes.c_int32)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        L.oracle_vote.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int,
                                  ctypes.c_int, i32p, i32p, u32p]
        L.oracle_vote.restype = ctypes.c_int
        L.oracle_vote_threads.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int,
                                          ctypes.c_int, i32p, i32p, u32p, ctypes.c_int]
        L.oracle_vote_threads.restype = ctypes.c_int
        L.oracle_vote_tolerant.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_float, ctypes.c_float, i32p,
                                           i32p, u32p]
        L.oracle_vote_tolerant.restype = ctypes.c_int
        L.oracle_median.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int,
                                    u32p, ctypes.c_int]
        L.oracle_median.restype = ctypes.c_int
        L.oracle_trimmed_mean.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int,
                                          ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                          ctypes.c_int]
        L.oracle_trimmed_mean.restype = ctypes.c_int
        L.oracle_bulyan.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int,
                                    ctypes.c_int, ctypes.POINTER(ctypes.c_double), i32p,
                                    ctypes.POINTER(ctypes.c_double), ctypes.c_int]
        L.oracle_bulyan.restype = ctypes.c_int
        L.oracle_mean_around_median.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, i32p, i32p,
                                                ctypes.c_int, ctypes.c_int,
                                                ctypes.POINTER(ctypes.c_double), ctypes.c_int]
        L.oracle_mean_around_median.restype = ctypes.c_int
        L.oracle_aggregate.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, i32p, ctypes.c_int,
                                       ctypes.c_int, u32p, i32p, ctypes.c_int]
        L.oracle_aggregate.restype = ctypes.c_int
        L.oracle_worst_case.argtypes = [u8p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_int, i32p, i32p]
        L.oracle_worst_case.restype = ctypes.c_int
        _lib = L
    return _lib


def _u32(X):
    X = np.asarray(X)
    assert X.ndim == 2 and X.dtype.itemsize == 4 and X.flags["C_CONTIGUOUS"]
    return X.view(np.uint32)


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def default_threads():
    return len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)


def vote(X, rows, d, threads=None):
    """Returns (winner_replica[f], winner_row[f], pair_neq[f]); with `threads` the files are spread
    over that many host threads (same decisions) and the number used is returned as a 4th item."""
    U = _u32(X)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    f, r = rows.shape
    wrep = np.zeros(f, dtype=np.int32)
    wrow = np.zeros(f, dtype=np.int32)
    neq = np.zeros(f, dtype=np.uint32)
    if threads is None:
        rc = lib().oracle_vote(_ptr(U, ctypes.c_uint32), d, U.shape[1], _ptr(rows, ctypes.c_int32),
                               f, r, _ptr(wrep, ctypes.c_int32), _ptr(wrow, ctypes.c_int32),
                               _ptr(neq, ctypes.c_uint32))
        if rc != 0:
            raise ValueError("oracle_vote rc=%d" % rc)
        return wrep, wrow, neq
    rc = lib().oracle_vote_threads(_ptr(U, ctypes.c_uint32), d, U.shape[1], _ptr(rows, ctypes.c_int32),
                                   f, r, _ptr(wrep, ctypes.c_int32), _ptr(wrow, ctypes.c_int32),
                                   _ptr(neq, ctypes.c_uint32), int(threads))
    if rc < 0:
        raise ValueError("oracle_vote_threads rc=%d" % rc)
    return wrep, wrow, neq, rc


def vote_tolerant(X, rows, d, atol, rtol):
    U = _u32(X)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    f, r = rows.shape
    wrep = np.zeros(f, dtype=np.int32)
    wrow = np.zeros(f, dtype=np.int32)
    far = np.zeros(f, dtype=np.uint32)
    rc = lib().oracle_vote_tolerant(_ptr(U, ctypes.c_uint32), d, U.shape[1],
                                    _ptr(rows, ctypes.c_int32), f, r, float(atol), float(rtol),
                                    _ptr(wrep, ctypes.c_int32), _ptr(wrow, ctypes.c_int32),
                                    _ptr(far, ctypes.c_uint32))
    if rc != 0:
        raise ValueError("oracle_vote_tolerant rc=%d" % rc)
    return wrep, wrow, far


def median(X, row_index, d, threads=None):
    U = _u32(X)
    row_index = np.ascontiguousarray(row_index, dtype=np.int32)
    out = np.zeros(d, dtype=np.uint32)
    t = default_threads() if threads is None else threads
    rc = lib().oracle_median(_ptr(U, ctypes.c_uint32), d, U.shape[1],
                             _ptr(row_index, ctypes.c_int32), len(row_index),
                             _ptr(out, ctypes.c_uint32), t)
    if rc < 0:
        raise ValueError("oracle_median rc=%d" % rc)
    return out.view(np.float32)


def trimmed_mean(X, row_index, d, b, threads=None):
    U = _u32(X)
    row_index = np.ascontiguousarray(row_index, dtype=np.int32)
    out = np.zeros(d, dtype=np.float64)
    t = default_threads() if threads is None else threads
    rc = lib().oracle_trimmed_mean(_ptr(U, ctypes.c_uint32), d, U.shape[1],
                                   _ptr(row_index, ctypes.c_int32), len(row_index), int(b),
                                   _ptr(out, ctypes.c_double), t)
    if rc < 0:
        raise ValueError("oracle_trimmed_mean rc=%d" % rc)
    return out


def bulyan(X, row_index, d, c, threads=None):
    """Returns (out[d] float64, chosen indices in order, dist[f, f] float64)."""
    U = _u32(X)
    row_index = np.ascontiguousarray(row_index, dtype=np.int32)
    f = len(row_index)
    out = np.zeros(d, dtype=np.float64)
    chosen = np.zeros(max(f - 2 * int(c), 1), dtype=np.int32)
    dist = np.zeros((f, f), dtype=np.float64)
    t = default_threads() if threads is None else threads
    rc = lib().oracle_bulyan(_ptr(U, ctypes.c_uint32), d, U.shape[1],
                             _ptr(row_index, ctypes.c_int32), f, int(c),
                             _ptr(out, ctypes.c_double), _ptr(chosen, ctypes.c_int32),
                             _ptr(dist, ctypes.c_double), t)
    if rc < 0:
        raise ValueError("oracle_bulyan rc=%d" % rc)
    return out, [int(x) for x in chosen[:f - 2 * int(c)]], dist


def mean_around_median(X, row_index, chosen, d, beta, threads=None):
    """Second phase of Bulyan on the rows row_index[chosen]: out[d] float64."""
    U = _u32(X)
    row_index = np.ascontiguousarray(row_index, dtype=np.int32)
    chosen = np.ascontiguousarray(chosen, dtype=np.int32)
    out = np.zeros(d, dtype=np.float64)
    t = default_threads() if threads is None else threads
    rc = lib().oracle_mean_around_median(_ptr(U, ctypes.c_uint32), d, U.shape[1],
                                         _ptr(row_index, ctypes.c_int32),
                                         _ptr(chosen, ctypes.c_int32), len(chosen), int(beta),
                                         _ptr(out, ctypes.c_double), t)
    if rc < 0:
        raise ValueError("oracle_mean_around_median rc=%d" % rc)
    return out


def aggregate(X, rows, d, threads=None):
    """Returns (median[d] float32, winner_replica[f], threads used)."""
    U = _u32(X)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    f, r = rows.shape
    out = np.zeros(d, dtype=np.uint32)
    wrep = np.zeros(f, dtype=np.int32)
    t = default_threads() if threads is None else threads
    rc = lib().oracle_aggregate(_ptr(U, ctypes.c_uint32), d, U.shape[1],
                                _ptr(rows, ctypes.c_int32), f, r, _ptr(out, ctypes.c_uint32),
                                _ptr(wrep, ctypes.c_int32), t)
    if rc < 0:
        raise ValueError("oracle_aggregate rc=%d" % rc)
    return out.view(np.float32), wrep, rc


def worst_case(H, q):
    H8 = np.ascontiguousarray(H, dtype=np.uint8)
    K, f = H8.shape
    r = int(H8[:, 0].sum())
    S = np.zeros(max(q, 1), dtype=np.int32)
    cmax = np.zeros(1, dtype=np.int32)
    rc = lib().oracle_worst_case(_ptr(H8, ctypes.c_uint8), K, f, r, q,
                                 _ptr(S, ctypes.c_int32), _ptr(cmax, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_worst_case rc=%d" % rc)
    return int(cmax[0]), tuple(int(x) for x in S[:q])
