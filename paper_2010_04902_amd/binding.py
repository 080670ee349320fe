"""ctypes binding of libbyzshield.so: same names as the C-ABI, argument marshalling only.

Device arguments are torch CUDA tensors (their data_ptr() is passed through); outputs that
the caller does not supply are allocated with torch.  There is no CPU fallback: if the
library cannot be loaded the import of this module's functions raises.
"""
import ctypes
import os
import weakref

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libbyzshield.so")

BYZ_SCHEME_MOLS = 0
BYZ_SCHEME_RAMANUJAN = 1
BYZ_SCHEME_FRC = 2
BYZ_MAX_F = 64
BYZ_MAX_F_KRUM = 128
BYZ_MAX_F_WIDE = 256
BYZ_MAX_R = 7

_lib = None


class ByzError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = "%s failed: %d (%s)" % (where, code, byz_strerror(code))
        if code == -4:
            msg += ", hipError_t=%d" % _load().byz_last_hip_error()
        super().__init__(msg)


def library_path():
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        # nothing built yet: build once, loudly
        from . import build as _build
        _build.build()
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32p, u32p, u64p = (ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32),
                            ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint64))
    ip = ctypes.POINTER(ctypes.c_int)
    c_int, i64, sz = ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
    sig = {
        "byz_build_assignment": (c_int, [c_int, c_int, c_int, ctypes.POINTER(vp)]),
        "byz_free_assignment": (None, [vp]),
        "byz_assignment_dims": (c_int, [vp, ip, ip, ip, ip]),
        "byz_assignment_worker_files": (c_int, [vp, i32p]),
        "byz_assignment_file_workers": (c_int, [vp, i32p]),
        "byz_assignment_file_rows": (c_int, [vp, i32p]),
        "byz_worst_case": (c_int, [vp, c_int, i32p, i32p, u64p]),
        "byz_worst_case_opts": (c_int, [vp, c_int, ctypes.c_uint, i32p, i32p, u64p]),
        "byz_worst_case_last_visited": (ctypes.c_uint64, []),
        "byz_gamma_bound": (ctypes.c_double, [vp, c_int]),
        "byz_vote": (c_int, [vp, i64, i64, vp, c_int, c_int, vp, vp, vp, vp]),
        "byz_vote_tolerant": (c_int, [vp, i64, i64, vp, c_int, c_int, ctypes.c_float,
                                      ctypes.c_float, vp, vp, vp, vp]),
        "byz_median": (c_int, [vp, i64, i64, vp, c_int, vp, vp]),
        "byz_trimmed_mean": (c_int, [vp, i64, i64, vp, c_int, c_int, vp, vp]),
        "byz_multi_krum_workspace_bytes": (sz, [c_int]),
        "byz_multi_krum": (c_int, [vp, i64, i64, vp, c_int, c_int, c_int, vp, vp, vp, vp, vp, sz, vp]),
        "byz_aggregate_workspace_bytes": (sz, [c_int, c_int]),
        "byz_aggregate_has_single_pass": (c_int, [c_int, c_int]),
        "byz_bulyan_workspace_bytes": (sz, [c_int]),
        "byz_bulyan": (c_int, [vp, i64, i64, vp, c_int, c_int, vp, vp, vp, vp, vp, sz, vp]),
        "byz_mean_around_median": (c_int, [vp, i64, i64, vp, c_int, c_int, vp, vp]),
        "byz_aggregate": (c_int, [vp, i64, i64, vp, c_int, c_int, vp, vp, vp, sz, vp]),
        "byz_aggregate_opts": (c_int, [vp, i64, i64, vp, c_int, c_int, vp, vp, vp, sz,
                                       ctypes.c_uint, vp]),
        "byz_aggregate_static": (c_int, [vp, i64, i64, vp, c_int, c_int, vp, vp, ctypes.c_uint, vp]),
        "byz_aggregate_path": (c_int, [vp, ip, vp]),
        "byz_calibration_copy": (c_int, [vp, vp, sz, vp]),
        "byz_calibration_read_rows": (c_int, [vp, i64, i64, c_int, vp, c_int, vp]),
        "byz_profile_enable": (c_int, [c_int]),
        "byz_profile_collect": (c_int, [ctypes.POINTER(ctypes.c_float), c_int, ip]),
        "byz_strerror": (ctypes.c_char_p, [c_int]),
        "byz_last_hip_error": (c_int, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def _check(code, where):
    if code != 0:
        raise ByzError(code, where)


def byz_strerror(code):
    return _load().byz_strerror(int(code)).decode()


class Assignment:
    """Owns a byz_assignment handle (worker-file graph of Sec. 4)."""

    def __init__(self, handle):
        self._h = handle
        K, f, l, r = (ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int())
        _check(_load().byz_assignment_dims(self._h, K, f, l, r), "byz_assignment_dims")
        self.K, self.f, self.l, self.r = K.value, f.value, l.value, r.value

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.byz_free_assignment(self._h)
            self._h = None

    def _table(self, fn, rows, cols):
        out = np.zeros((rows, cols), dtype=np.int32)
        _check(getattr(_load(), fn)(self._h, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))), fn)
        return out

    def worker_files(self):
        return self._table("byz_assignment_worker_files", self.K, self.l)

    def file_workers(self):
        return self._table("byz_assignment_file_workers", self.f, self.r)

    def file_rows(self):
        return self._table("byz_assignment_file_rows", self.f, self.r)


def byz_build_assignment(scheme, a, b):
    h = ctypes.c_void_p()
    _check(_load().byz_build_assignment(int(scheme), int(a), int(b), ctypes.byref(h)),
           "byz_build_assignment")
    return Assignment(h)


BYZ_SEARCH_EXHAUSTIVE = 1
BYZ_SEARCH_SYMMETRY = 2


def byz_worst_case(asg, q, flags=0):
    """Returns (byzantine workers as a tuple, c_max, distorted-file bit mask)."""
    S = np.zeros(max(int(q), 1), dtype=np.int32)
    cmax = ctypes.c_int32()
    words = np.zeros(max((asg.f + 63) // 64, 1), dtype=np.uint64)
    _check(_load().byz_worst_case_opts(asg._h, int(q), int(flags),
                                       S.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                       ctypes.byref(cmax),
                                       words.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))),
           "byz_worst_case")
    mask = sum(int(w) << (64 * i) for i, w in enumerate(words))
    return tuple(int(x) for x in S[:max(int(q), 0)]), int(cmax.value), mask


def byz_worst_case_last_visited():
    return int(_load().byz_worst_case_last_visited())


def byz_gamma_bound(asg, q):
    return float(_load().byz_gamma_bound(asg._h, int(q)))


# ------------------------------------------------------------------ device entry points


def _torch():
    import torch
    return torch


def _stream_ptr(stream):
    if stream is None:
        stream = _torch().cuda.current_stream()
    return ctypes.c_void_p(getattr(stream, "cuda_stream", stream))


def _dev_ptr(t, dtype_names, what):
    if not t.is_cuda:
        raise ValueError("%s must be a CUDA tensor" % what)
    if str(t.dtype).replace("torch.", "") not in dtype_names:
        raise ValueError("%s has dtype %s" % (what, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % what)
    return ctypes.c_void_p(t.data_ptr())


def _need(t, n, what):
    """The C side trusts pointer/size pairs: refuse a tensor shorter than the call will read."""
    if n > 0 and int(t.numel()) < n:
        raise ValueError("%s has %d elements, the call needs %d" % (what, int(t.numel()), n))


_checked_tables = {}


def _need_rows_in_range(table, count, n_rows, what):
    """The kernels trust the row numbers they are given (they are not range-checked on the
    device): refuse, before any launch, a table whose first `count` entries do not all lie in
    [0, n_rows).  The minimum and maximum are read back once per tensor object -- remembered
    through a weak reference, with torch's modification counter -- so repeated calls with one
    table cost nothing, and a new tensor that happens to reuse the memory is looked at afresh."""
    if count <= 0:
        return
    _need(table, count, what)
    if table.is_cuda and _torch().cuda.is_current_stream_capturing():
        # nothing can be read back while a graph is being captured, and a table a captured
        # kernel will write (winner rows of a vote in the same graph) has no contents yet:
        # there the caller vouches for the table
        return
    entry = _checked_tables.get(id(table))
    if entry is not None and entry[0]() is table and entry[1] == (int(table._version), int(count)):
        bounds = entry[2]
    else:
        head = table.reshape(-1)[:count]
        bounds = (int(head.min()), int(head.max()))
        if len(_checked_tables) >= 256:
            _checked_tables.clear()
        _checked_tables[id(table)] = (weakref.ref(table), (int(table._version), int(count)), bounds)
    if bounds[0] < 0 or bounds[1] >= n_rows:
        raise ValueError("%s names rows %d..%d, the matrix has rows 0..%d"
                         % (what, bounds[0], bounds[1], n_rows - 1))


def _rows_2d(copies):
    if copies.dim() != 2:
        raise ValueError("copies must be [rows, ld]")
    return int(copies.shape[1])


def byz_vote(copies, d, file_rows_dev, f, r, stream=None):
    """-> (winner_replica[f] int32, winner_row[f] int32, pair_neq[f] int32 bit masks), on device."""
    torch = _torch()
    ld = _rows_2d(copies)
    _need_rows_in_range(file_rows_dev, int(f) * int(r), int(copies.shape[0]), "file_rows_dev")
    wrep = torch.empty(max(int(f), 0), dtype=torch.int32, device=copies.device)
    wrow = torch.empty(max(int(f), 0), dtype=torch.int32, device=copies.device)
    neq = torch.empty(max(int(f), 0), dtype=torch.int32, device=copies.device)
    _check(_load().byz_vote(_dev_ptr(copies, ("float32",), "copies"), int(d), ld,
                            _dev_ptr(file_rows_dev, ("int32",), "file_rows_dev"), int(f), int(r),
                            _dev_ptr(wrep, ("int32",), "winner_replica"),
                            _dev_ptr(wrow, ("int32",), "winner_row"),
                            _dev_ptr(neq, ("int32",), "pair_neq"), _stream_ptr(stream)),
           "byz_vote")
    return wrep, wrow, neq


def byz_vote_tolerant(copies, d, file_rows_dev, f, r, atol, rtol, stream=None):
    """-> (winner_replica[f] int32, winner_row[f] int32, pair_far[f] int32 bit masks), on device."""
    torch = _torch()
    ld = _rows_2d(copies)
    _need_rows_in_range(file_rows_dev, int(f) * int(r), int(copies.shape[0]), "file_rows_dev")
    wrep = torch.empty(max(int(f), 0), dtype=torch.int32, device=copies.device)
    wrow = torch.empty(max(int(f), 0), dtype=torch.int32, device=copies.device)
    far = torch.empty(max(int(f), 0), dtype=torch.int32, device=copies.device)
    _check(_load().byz_vote_tolerant(_dev_ptr(copies, ("float32",), "copies"), int(d), ld,
                                     _dev_ptr(file_rows_dev, ("int32",), "file_rows_dev"),
                                     int(f), int(r), float(atol), float(rtol),
                                     _dev_ptr(wrep, ("int32",), "winner_replica"),
                                     _dev_ptr(wrow, ("int32",), "winner_row"),
                                     _dev_ptr(far, ("int32",), "pair_far"), _stream_ptr(stream)),
           "byz_vote_tolerant")
    return wrep, wrow, far


def byz_median(rows_base, d, row_index_dev, out=None, stream=None):
    torch = _torch()
    ld = _rows_2d(rows_base)
    f = int(row_index_dev.numel())
    _need_rows_in_range(row_index_dev, f, int(rows_base.shape[0]), "row_index_dev")
    if out is None:
        out = torch.empty(int(d), dtype=torch.float32, device=rows_base.device)
    _need(out, int(d), "out")
    _check(_load().byz_median(_dev_ptr(rows_base, ("float32",), "rows_base"), int(d), ld,
                              _dev_ptr(row_index_dev, ("int32",), "row_index_dev"), f,
                              _dev_ptr(out, ("float32",), "out"), _stream_ptr(stream)),
           "byz_median")
    return out


def byz_trimmed_mean(rows_base, d, row_index_dev, b, out=None, stream=None):
    torch = _torch()
    ld = _rows_2d(rows_base)
    f = int(row_index_dev.numel())
    _need_rows_in_range(row_index_dev, f, int(rows_base.shape[0]), "row_index_dev")
    if out is None:
        out = torch.empty(int(d), dtype=torch.float32, device=rows_base.device)
    _need(out, int(d), "out")
    _check(_load().byz_trimmed_mean(_dev_ptr(rows_base, ("float32",), "rows_base"), int(d), ld,
                                    _dev_ptr(row_index_dev, ("int32",), "row_index_dev"), f,
                                    int(b), _dev_ptr(out, ("float32",), "out"),
                                    _stream_ptr(stream)), "byz_trimmed_mean")
    return out


def byz_multi_krum_workspace_bytes(f):
    return int(_load().byz_multi_krum_workspace_bytes(int(f)))


def byz_multi_krum(rows_base, d, row_index_dev, c, m, out=None, workspace=None, stream=None):
    """-> (out[d] float32, selected[f] int32, scores[f] float64, dist[f, f] float64), on device."""
    torch = _torch()
    ld = _rows_2d(rows_base)
    f = int(row_index_dev.numel())
    dev = rows_base.device
    _need_rows_in_range(row_index_dev, f, int(rows_base.shape[0]), "row_index_dev")
    if out is None:
        out = torch.empty(int(d), dtype=torch.float32, device=dev)
    _need(out, int(d), "out")
    if workspace is None:
        workspace = torch.empty(max(byz_multi_krum_workspace_bytes(f), 256), dtype=torch.uint8, device=dev)
    selected = torch.empty(f, dtype=torch.int32, device=dev)
    scores = torch.empty(f, dtype=torch.float64, device=dev)
    dist = torch.empty((f, f), dtype=torch.float64, device=dev)
    _check(_load().byz_multi_krum(_dev_ptr(rows_base, ("float32",), "rows_base"), int(d), ld,
                                  _dev_ptr(row_index_dev, ("int32",), "row_index_dev"), f, int(c),
                                  int(m), _dev_ptr(out, ("float32",), "out"),
                                  _dev_ptr(selected, ("int32",), "selected"),
                                  _dev_ptr(scores, ("float64",), "scores"),
                                  _dev_ptr(dist, ("float64",), "dist"),
                                  _dev_ptr(workspace, ("uint8",), "workspace"),
                                  int(workspace.numel()), _stream_ptr(stream)), "byz_multi_krum")
    return out, selected, scores, dist


def byz_bulyan_workspace_bytes(f):
    return int(_load().byz_bulyan_workspace_bytes(int(f)))


def byz_bulyan(rows_base, d, row_index_dev, c, out=None, workspace=None, stream=None):
    """-> (out[d] float32, selected[f] int32, order[f-2c] int32, dist[f, f] float64), on device."""
    torch = _torch()
    ld = _rows_2d(rows_base)
    f = int(row_index_dev.numel())
    dev = rows_base.device
    _need_rows_in_range(row_index_dev, f, int(rows_base.shape[0]), "row_index_dev")
    if out is None:
        out = torch.empty(int(d), dtype=torch.float32, device=dev)
    _need(out, int(d), "out")
    if workspace is None:
        workspace = torch.empty(max(byz_bulyan_workspace_bytes(f), 256), dtype=torch.uint8, device=dev)
    selected = torch.empty(f, dtype=torch.int32, device=dev)
    order = torch.empty(max(f - 2 * int(c), 1), dtype=torch.int32, device=dev)
    dist = torch.empty((f, f), dtype=torch.float64, device=dev)
    _check(_load().byz_bulyan(_dev_ptr(rows_base, ("float32",), "rows_base"), int(d), ld,
                              _dev_ptr(row_index_dev, ("int32",), "row_index_dev"), f, int(c),
                              _dev_ptr(out, ("float32",), "out"),
                              _dev_ptr(selected, ("int32",), "selected"),
                              _dev_ptr(order, ("int32",), "order"),
                              _dev_ptr(dist, ("float64",), "dist"),
                              _dev_ptr(workspace, ("uint8",), "workspace"),
                              int(workspace.numel()), _stream_ptr(stream)), "byz_bulyan")
    return out, selected, order[:max(f - 2 * int(c), 0)], dist


def byz_mean_around_median(rows_base, d, row_index_dev, beta, out=None, stream=None):
    """-> out[d] float32 on device: mean of the beta values closest to the median, per coordinate."""
    torch = _torch()
    ld = _rows_2d(rows_base)
    f = int(row_index_dev.numel())
    _need_rows_in_range(row_index_dev, f, int(rows_base.shape[0]), "row_index_dev")
    if out is None:
        out = torch.empty(int(d), dtype=torch.float32, device=rows_base.device)
    _need(out, int(d), "out")
    _check(_load().byz_mean_around_median(_dev_ptr(rows_base, ("float32",), "rows_base"), int(d), ld,
                                          _dev_ptr(row_index_dev, ("int32",), "row_index_dev"), f,
                                          int(beta), _dev_ptr(out, ("float32",), "out"),
                                          _stream_ptr(stream)), "byz_mean_around_median")
    return out


def byz_aggregate_workspace_bytes(f, r):
    return int(_load().byz_aggregate_workspace_bytes(int(f), int(r)))


BYZ_AGG_EARLY_MAJORITY = 1
BYZ_AGG_TRIMMED_MEAN = 2


def BYZ_AGG_TRIM(b):
    return BYZ_AGG_TRIMMED_MEAN | (int(b) << 8)


def BYZ_AGG_PROBE_SHIFT(s):
    """Flag value that moves the single pass's probe sample (s in 0..65535); see byzshield.h."""
    return (int(s) & 0xFFFF) << 16


def byz_aggregate_opts(copies, d, file_rows_dev, f, r, flags, out=None, winner_replica=None,
                       workspace=None, stream=None):
    """byz_aggregate with option flags (BYZ_AGG_EARLY_MAJORITY); same returns."""
    return byz_aggregate(copies, d, file_rows_dev, f, r, out=out, winner_replica=winner_replica,
                         workspace=workspace, stream=stream, _flags=int(flags))


def byz_aggregate(copies, d, file_rows_dev, f, r, out=None, winner_replica=None, workspace=None,
                  stream=None, _flags=None):
    """-> (out[d] float32, winner_replica[f] int32, workspace uint8 tensor), on device."""
    torch = _torch()
    ld = _rows_2d(copies)
    if out is None:
        out = torch.empty(int(d), dtype=torch.float32, device=copies.device)
    if winner_replica is None:
        winner_replica = torch.empty(int(f), dtype=torch.int32, device=copies.device)
    if workspace is None:
        nbytes = byz_aggregate_workspace_bytes(f, r)
        if nbytes == 0:
            raise ByzError(-1, "byz_aggregate_workspace_bytes")
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=copies.device)
    _need_rows_in_range(file_rows_dev, int(f) * int(r), int(copies.shape[0]), "file_rows_dev")
    _need(out, int(d), "out")
    _need(winner_replica, int(f), "winner_replica")
    args = [_dev_ptr(copies, ("float32",), "copies"), int(d), ld,
            _dev_ptr(file_rows_dev, ("int32",), "file_rows_dev"), int(f), int(r),
            _dev_ptr(out, ("float32",), "out"),
            _dev_ptr(winner_replica, ("int32",), "winner_replica"),
            _dev_ptr(workspace, ("uint8",), "workspace"), int(workspace.numel())]
    if _flags is None:
        _check(_load().byz_aggregate(*args, _stream_ptr(stream)), "byz_aggregate")
    else:
        _check(_load().byz_aggregate_opts(*args, _flags, _stream_ptr(stream)), "byz_aggregate_opts")
    return out, winner_replica, workspace


def byz_aggregate_static(copies, d, file_rows_dev, f, r, out, winner_replica, flags=0, stream=None):
    """byz_aggregate_opts on the library's own fixed scratch; the caller supplies every buffer."""
    ld = _rows_2d(copies)
    _need_rows_in_range(file_rows_dev, int(f) * int(r), int(copies.shape[0]), "file_rows_dev")
    _need(out, int(d), "out")
    _need(winner_replica, int(f), "winner_replica")
    _check(_load().byz_aggregate_static(_dev_ptr(copies, ("float32",), "copies"), int(d), ld,
                                        _dev_ptr(file_rows_dev, ("int32",), "file_rows_dev"),
                                        int(f), int(r), _dev_ptr(out, ("float32",), "out"),
                                        _dev_ptr(winner_replica, ("int32",), "winner_replica"),
                                        int(flags), _stream_ptr(stream)), "byz_aggregate_static")
    return out, winner_replica


def byz_aggregate_has_single_pass(f, r):
    return bool(_load().byz_aggregate_has_single_pass(int(f), int(r)))


BYZ_PATH_SINGLE_PASS = 0
BYZ_PATH_MEDIAN_REDONE = 1
BYZ_PATH_REVOTED = 2
BYZ_PATH_TWO_STEP = 4


def byz_aggregate_path(workspace, stream=None):
    """-> byz_path bits of the last byz_aggregate call on this workspace (synchronises the stream)."""
    path = ctypes.c_int()
    _check(_load().byz_aggregate_path(_dev_ptr(workspace, ("uint8",), "workspace"),
                                      ctypes.byref(path), _stream_ptr(stream)), "byz_aggregate_path")
    return int(path.value)


def byz_profile_enable(max_calls):
    _check(_load().byz_profile_enable(int(max_calls)), "byz_profile_enable")


def byz_profile_collect(capacity):
    """-> list of single-pass kernel durations (ms) recorded since the last collect."""
    buf = (ctypes.c_float * max(int(capacity), 1))()
    n = ctypes.c_int()
    _check(_load().byz_profile_collect(buf, int(capacity), ctypes.byref(n)), "byz_profile_collect")
    return [float(buf[i]) for i in range(n.value)]


def byz_calibration_read_rows(rows_base, d, n_rows, out, store, stream=None):
    """Reads rows 0..n_rows-1 of rows_base the way the single pass does; store != 0 also writes."""
    ld = _rows_2d(rows_base)
    if int(n_rows) > rows_base.shape[0]:
        raise ValueError("rows_base has fewer than n_rows rows")
    _need(out, int(d), "out")
    _check(_load().byz_calibration_read_rows(_dev_ptr(rows_base, ("float32",), "rows_base"), int(d), ld,
                                             int(n_rows), _dev_ptr(out, ("float32",), "out"),
                                             int(bool(store)), _stream_ptr(stream)),
           "byz_calibration_read_rows")


def byz_calibration_copy(src, dst, stream=None):
    """dst <- src (same-sized contiguous CUDA tensors) with the library's plain copy kernel."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("src and dst must be contiguous and of equal size")
    _check(_load().byz_calibration_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()),
                                        nbytes, _stream_ptr(stream)), "byz_calibration_copy")
