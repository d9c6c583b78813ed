"""Helpers for the tests, the smoke check and the benchmark: move a seeded workload into device
memory (PyTorch tensors) and call the C ABI.  No arithmetic of the method lives here."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import rnn
from . import workloads as W


def to_device_storage(a: np.ndarray, dtype: int, device="cuda") -> torch.Tensor:
    """float32 values (already exactly representable in `dtype`) -> device tensor of the storage type."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if dtype == W.BF16:
        t = t.to(torch.bfloat16)  # exact: the values are bf16-representable
    return t.to(device).contiguous()


class DeviceModel:
    """Owns an rnn_model handle created from a Workload's weights."""

    def __init__(self, wl: W.Workload, plan: int = rnn.RNN_PLAN_AUTO, weights_on_device: bool = False):
        c = wl.cfg
        self.cfg = c
        if weights_on_device:
            self._w = [to_device_storage(w, c.dtype) for w in wl.weights]
            torch.cuda.synchronize()
            ws = self._w
        else:
            ws = []
            for w in wl.weights:
                if c.dtype == W.BF16:
                    ws.append(W.f32_to_bf16_bits(w).reshape(w.shape))
                else:
                    ws.append(np.ascontiguousarray(w, dtype=np.float32))
            self._w = ws
        self.handle = rnn.rnn_model_create(c.cell, c.L, c.I, c.H, c.D, c.dtype, ws, int(weights_on_device))
        rc = rnn.rnn_model_set_plan(self.handle, plan)
        if rc != rnn.RNN_OK:
            rnn.rnn_model_destroy(self.handle)
            self.handle = None
            raise rnn.RnnError(rc, "rnn_model_set_plan")

    def close(self):
        if getattr(self, "handle", None):
            torch.cuda.synchronize()
            rnn.rnn_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class DeviceIO:
    """Device tensors for one workload: inputs uploaded once, outputs preallocated."""

    def __init__(self, wl: W.Workload, want_state: bool = True):
        c = wl.cfg
        tdt = torch.bfloat16 if c.dtype == W.BF16 else torch.float32
        self.cfg = c
        self.x = to_device_storage(wl.x, c.dtype)
        self.lengths = None if wl.lengths is None else torch.from_numpy(wl.lengths).to("cuda")
        self.h0 = None if wl.h0 is None else torch.from_numpy(wl.h0).to("cuda")
        self.c0 = None if wl.c0 is None else torch.from_numpy(wl.c0).to("cuda")
        # outputs start from a non-zero pattern so that padded positions must really be written
        self.y = torch.full((c.T, c.B, c.D * c.H), 7.0, dtype=tdt, device="cuda")
        self.hT = torch.full((c.L * c.D, c.B, c.H), 7.0, device="cuda") if want_state else None
        self.cT = torch.full((c.L * c.D, c.B, c.H), 7.0, device="cuda") if want_state else None


def forward(model: DeviceModel, io: DeviceIO, stream: Optional[torch.cuda.Stream] = None, check: bool = True):
    c = io.cfg
    s = stream if stream is not None else torch.cuda.current_stream()
    rc = rnn.rnn_forward(model.handle, io.x, io.lengths, io.h0, io.c0, io.y, io.hT, io.cT, c.T, c.B, s)
    if check and rc != rnn.RNN_OK:
        raise rnn.RnnError(rc, "rnn_forward")
    return rc


def results(io: DeviceIO):
    """(y, hT, cT) as float64 numpy arrays plus the raw bit patterns of y."""
    torch.cuda.synchronize()
    y = io.y.float().cpu().numpy().astype(np.float64)
    if io.y.dtype == torch.bfloat16:
        ybits = io.y.view(torch.int16).cpu().numpy().view(np.uint16)
    else:
        ybits = io.y.view(torch.int32).cpu().numpy().view(np.uint32)
    hT = None if io.hT is None else io.hT.cpu().numpy().astype(np.float64)
    cT = None if io.cT is None else io.cT.cpu().numpy().astype(np.float64)
    return y, hT, cT, ybits
