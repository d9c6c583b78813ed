"""ctypes binding of include/rnn_schedule.h (host-side scheduling of the cell graph); marshalling only."""
from __future__ import annotations

import ctypes

import numpy as np

from . import rnn

EXPORTS = ("rnn_schedule_grid_size", "rnn_schedule_grid", "rnn_schedule_order", "rnn_schedule_simulate",
           "rnn_schedule_place_resident")

_declared = False


def _lib():
    global _declared
    lib = rnn.load_library()
    if not _declared:
        ci, vp = ctypes.c_int, ctypes.c_void_p
        lib.rnn_schedule_grid_size.restype = ci
        lib.rnn_schedule_grid_size.argtypes = [ci, ci, ci, ctypes.POINTER(ci), ctypes.POINTER(ci)]
        lib.rnn_schedule_grid.restype = ci
        lib.rnn_schedule_grid.argtypes = [ci, ci, ci, vp, vp]
        lib.rnn_schedule_order.restype = ci
        lib.rnn_schedule_order.argtypes = [ci, vp, vp, vp, vp, vp]
        lib.rnn_schedule_simulate.restype = ci
        lib.rnn_schedule_simulate.argtypes = [ci, vp, vp, vp, ci, vp, vp, vp, vp, ctypes.POINTER(ctypes.c_double)]
        lib.rnn_schedule_place_resident.restype = ci
        lib.rnn_schedule_place_resident.argtypes = [ci, vp, vp, vp, ci, vp, vp, vp, vp, vp, vp,
                                                    ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ci)]
        _declared = True
    return lib


def _p(a):
    return None if a is None else a.ctypes.data


def rnn_schedule_grid(L: int, T: int, D: int):
    """Returns (status, pred_offset int32 [n+1], pred_index int32 [edges])."""
    n, ne = ctypes.c_int(0), ctypes.c_int(0)
    rc = _lib().rnn_schedule_grid_size(L, T, D, ctypes.byref(n), ctypes.byref(ne))
    if rc != rnn.RNN_OK:
        return rc, None, None
    off = np.zeros(n.value + 1, dtype=np.int32)
    idx = np.zeros(max(ne.value, 1), dtype=np.int32)
    rc = _lib().rnn_schedule_grid(L, T, D, _p(off), _p(idx))
    return rc, off, idx[:ne.value]


def rnn_schedule_order(pred_offset, pred_index, comm, avg_exec):
    """Returns (status, order int32 [n])."""
    off = np.ascontiguousarray(pred_offset, dtype=np.int32)
    idx = np.ascontiguousarray(pred_index, dtype=np.int32)
    cm = np.ascontiguousarray(comm, dtype=np.float64)
    av = np.ascontiguousarray(avg_exec, dtype=np.float64)
    n = off.size - 1
    order = np.full(n, -1, dtype=np.int32)
    rc = _lib().rnn_schedule_order(n, _p(off), _p(idx) if idx.size else None, _p(cm) if cm.size else None, _p(av),
                                   _p(order))
    return rc, order


def rnn_schedule_simulate(pred_offset, pred_index, order, P: int, exec_time, comm):
    """Returns (status, proc int32 [n], aft float64 [n], latency)."""
    off = np.ascontiguousarray(pred_offset, dtype=np.int32)
    idx = np.ascontiguousarray(pred_index, dtype=np.int32)
    od = np.ascontiguousarray(order, dtype=np.int32)
    ex = np.ascontiguousarray(exec_time, dtype=np.float64)
    cm = np.ascontiguousarray(comm, dtype=np.float64)
    n = off.size - 1
    proc = np.full(n, -1, dtype=np.int32)
    aft = np.zeros(n, dtype=np.float64)
    lat = ctypes.c_double(0.0)
    rc = _lib().rnn_schedule_simulate(n, _p(off), _p(idx) if idx.size else None, _p(od), P, _p(ex),
                                      _p(cm) if cm.size else None, _p(proc), _p(aft), ctypes.byref(lat))
    return rc, proc, aft, lat.value


def rnn_schedule_place_resident(pred_offset, pred_index, order, P: int, exec_time, comm, kind):
    """Returns (status, proc int32 [n], pass int32 [n], aft float64 [n], latency, number of passes)."""
    off = np.ascontiguousarray(pred_offset, dtype=np.int32)
    idx = np.ascontiguousarray(pred_index, dtype=np.int32)
    od = np.ascontiguousarray(order, dtype=np.int32)
    ex = np.ascontiguousarray(exec_time, dtype=np.float64)
    cm = np.ascontiguousarray(comm, dtype=np.float64)
    kd = np.ascontiguousarray(kind, dtype=np.int32)
    n = off.size - 1
    proc = np.full(n, -1, dtype=np.int32)
    rnd = np.full(n, -1, dtype=np.int32)
    aft = np.zeros(n, dtype=np.float64)
    lat = ctypes.c_double(0.0)
    npass = ctypes.c_int(0)
    rc = _lib().rnn_schedule_place_resident(n, _p(off), _p(idx) if idx.size else None, _p(od), P, _p(ex),
                                            _p(cm) if cm.size else None, _p(kd), _p(proc), _p(rnd), _p(aft),
                                            ctypes.byref(lat), ctypes.byref(npass))
    return rc, proc, rnd, aft, lat.value, npass.value
