"""ctypes binding of the C oracle (oracle/rnn_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may use this module.
It knows nothing about the GPU library and imports nothing from it.

The oracle follows the cell grid of the paper's unfolded-RNN figure (Section 2.2) with the
standard LSTM / GRU cell equations (the paper prints none); see the header of rnn_oracle.c.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rnn_oracle.c")
_LIB = os.path.join(_HERE, "librnn_oracle.so")

LSTM = 0
GRU = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (plus OpenMP for the optional outer-loop threading)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.rnn_oracle_forward.restype = ctypes.c_int
        lib.rnn_oracle_forward.argtypes = [ctypes.c_int] * 8 + [
            ctypes.POINTER(dp), dp, ctypes.POINTER(ctypes.c_int), dp, dp, dp, dp, dp, dp,
            ctypes.c_int]
        lib.rnn_oracle_forward_ext.restype = ctypes.c_int
        lib.rnn_oracle_forward_ext.argtypes = [ctypes.c_int] * 8 + [
            ctypes.POINTER(dp), ctypes.POINTER(dp), ctypes.c_double, dp, ctypes.POINTER(ctypes.c_int),
            dp, dp, dp, dp, dp, dp, ctypes.c_int]
        lib.rnn_oracle_projection.restype = ctypes.c_int
        lib.rnn_oracle_projection.argtypes = [ctypes.c_int] * 3 + [dp, dp, dp]
        _lib = lib
    return _lib


def _as_f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a: Optional[np.ndarray]):
    dp = ctypes.POINTER(ctypes.c_double)
    return ctypes.cast(None, dp) if a is None else a.ctypes.data_as(dp)


def forward(cell: int, L: int, D: int, I: int, H: int, weights: Sequence[Optional[np.ndarray]],
            x, lengths=None, h0=None, c0=None, gru_variant: int = 0, nthreads: int = 1,
            return_layers: bool = False, peepholes=None, clip: float = 0.0):
    """Run the oracle.  weights: L*D*4 arrays (W_ih, W_hh, b_ih, b_hh per layer and direction;
    a bias may be None).  x: [T, B, I].  peepholes: None or L*D arrays [3, H] (p_i, p_f, p_o; LSTM
    only, an entry may be None); clip: clipping threshold of the gate arguments, 0 = none.
    Returns (y [T,B,D*H], hT [L*D,B,H], cT or None) in float64, plus layer outputs [L,T,B,D*H]
    when return_layers is set."""
    lib = _load()
    x = _as_f64(x)
    T, B, I_x = x.shape
    assert I_x == I, "x last dimension must equal the input size"
    assert len(weights) == L * D * 4
    G = 4 if cell == LSTM else 3
    ws: List[Optional[np.ndarray]] = []
    for l in range(L):
        il = I if l == 0 else D * H
        for d in range(D):
            base = (l * D + d) * 4
            shapes = ((G * H, il), (G * H, H), (G * H,), (G * H,))
            for j, shp in enumerate(shapes):
                w = weights[base + j]
                if w is None:
                    assert j >= 2, "only biases may be omitted"
                    ws.append(None)
                else:
                    w = _as_f64(w)
                    assert w.shape == shp, (l, d, j, w.shape, shp)
                    ws.append(w)
    dp = ctypes.POINTER(ctypes.c_double)
    wptrs = (dp * len(ws))(*[_ptr(w) for w in ws])
    len_arr = None
    len_ptr = ctypes.cast(None, ctypes.POINTER(ctypes.c_int))
    if lengths is not None:
        len_arr = np.ascontiguousarray(np.asarray(lengths, dtype=np.int32))
        assert len_arr.shape == (B,)
        len_ptr = len_arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int))
    h0a = None if h0 is None else _as_f64(h0)
    c0a = None if c0 is None else _as_f64(c0)
    for s in (h0a, c0a):
        assert s is None or s.shape == (L * D, B, H)
    y = np.empty((T, B, D * H), dtype=np.float64)
    hT = np.empty((L * D, B, H), dtype=np.float64)
    cT = np.zeros((L * D, B, H), dtype=np.float64) if cell == LSTM else None
    layers = np.empty((L, T, B, D * H), dtype=np.float64) if return_layers else None
    if peepholes is None and not clip:
        rc = lib.rnn_oracle_forward(cell, gru_variant, L, D, I, H, T, B, wptrs, _ptr(x), len_ptr,
                                    _ptr(h0a), _ptr(c0a), _ptr(y), _ptr(hT), _ptr(cT), _ptr(layers),
                                    int(nthreads))
    else:
        pp = ctypes.cast(None, ctypes.POINTER(dp))
        keep = []
        if peepholes is not None:
            assert len(peepholes) == L * D
            for q in peepholes:
                if q is not None:
                    q = _as_f64(q)
                    assert q.shape == (3, H)
                keep.append(q)
            pp = (dp * (L * D))(*[_ptr(q) for q in keep])
        rc = lib.rnn_oracle_forward_ext(cell, gru_variant, L, D, I, H, T, B, wptrs, pp, float(clip),
                                        _ptr(x), len_ptr, _ptr(h0a), _ptr(c0a), _ptr(y), _ptr(hT),
                                        _ptr(cT), _ptr(layers), int(nthreads))
    if rc != 0:
        raise ValueError("rnn_oracle_forward failed with status %d" % rc)
    if return_layers:
        return y, hT, cT, layers
    return y, hT, cT


def forward_workload(wl, nthreads: int = 1, **kw):
    """Convenience: run the oracle on an object with fields cfg, weights, x, lengths, h0, c0."""
    c = wl.cfg
    return forward(c.cell, c.L, c.D, c.I, c.H, wl.weights, wl.x, wl.lengths, wl.h0, wl.c0,
                   nthreads=nthreads, **kw)


def projection(inp, W_ih):
    """P = inp @ W_ih.T, one scalar dot product per element (inp [rows, K], W_ih [n_out, K])."""
    lib = _load()
    inp = _as_f64(inp)
    W_ih = _as_f64(W_ih)
    rows, K = inp.shape
    n_out, K2 = W_ih.shape
    assert K == K2
    P = np.empty((rows, n_out), dtype=np.float64)
    rc = lib.rnn_oracle_projection(rows, n_out, K, _ptr(inp), _ptr(W_ih), _ptr(P))
    if rc != 0:
        raise ValueError("rnn_oracle_projection failed with status %d" % rc)
    return P
