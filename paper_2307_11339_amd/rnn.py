"""Thin ctypes binding of the C ABI declared in include/rnn.h.

The functions below have the names and argument order of the C entry points and do argument
marshalling only (tensor -> device pointer); every step of the forward pass runs in the HIP
library.  There is no fallback: if the compiled library is missing, loading fails loudly.
PyTorch is used for device memory and streams, nothing else.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librnn_mi355x.so")

RNN_LSTM, RNN_GRU = 0, 1
RNN_F32, RNN_BF16 = 0, 1
RNN_OK, RNN_EINVAL, RNN_EUNSUPPORTED, RNN_ENOMEM, RNN_EDEVICE, RNN_ESCRATCH = 0, 1, 2, 3, 4, 5
RNN_STATIC_SCRATCH_MIB = 64
RNN_PLAN_AUTO, RNN_PLAN_CELLWISE, RNN_PLAN_WAVEFRONT = 0, 1, 2
RNN_ORDER_IFGO_RZN, RNN_ORDER_ONNX = 0, 1
RNN_KERNEL_PROJECTION, RNN_KERNEL_RECURRENT = 0, 1
RNN_PROFILE_KERNELS, RNN_PROFILE_STEP_TICKS = 1, 2

EXPORTS = ("rnn_model_create", "rnn_model_destroy", "rnn_model_set_plan", "rnn_model_reserve",
           "rnn_forward", "rnn_input_projection", "rnn_model_check", "rnn_model_device_bytes",
           "rnn_status_string", "rnn_model_set_profiling", "rnn_model_profile_read",
           "rnn_model_read_step_ticks", "rnn_model_input_product_placement", "rnn_model_create_ordered",
           "rnn_model_set_gru_reset_before", "rnn_plan_query", "rnn_model_set_spin_limit",
           "rnn_model_set_clip", "rnn_model_set_peepholes", "rnn_model_set_batch_first", "rnn_forward_static",
           "rnn_model_set_validation", "rnn_model_set_launch_tag", "rnn_probe_matrix_rate", "rnn_plan_launches", "rnn_probe_exchange_step",
           "rnn_stack_create", "rnn_stack_destroy", "rnn_stack_runs", "rnn_stack_run", "rnn_stack_device_bytes",
           "rnn_stack_forward")

_lib = None


class RnnError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__("%s: %s (status %d)" % (what, rnn_status_string(status), status))
        self.status = status


def load_library() -> ctypes.CDLL:
    """Load librnn_mi355x.so (built by paper_2307_11339_amd._build or __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("HIP library not built: %s is missing; run `python __graft_entry__.py build` "
                          "(there is no CPU fallback)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.rnn_model_create.restype = ci
    lib.rnn_model_create.argtypes = [ctypes.POINTER(vp), ci, ci, ci, ci, ci, ci, ctypes.POINTER(vp), ci]
    lib.rnn_model_create_ordered.restype = ci
    lib.rnn_model_create_ordered.argtypes = [ctypes.POINTER(vp), ci, ci, ci, ci, ci, ci, ctypes.POINTER(vp), ci, ci]
    lib.rnn_model_set_gru_reset_before.restype = ci
    lib.rnn_model_set_gru_reset_before.argtypes = [vp, ci]
    lib.rnn_model_destroy.restype = None
    lib.rnn_model_destroy.argtypes = [vp]
    lib.rnn_model_set_plan.restype = ci
    lib.rnn_model_set_plan.argtypes = [vp, ci]
    lib.rnn_model_reserve.restype = ci
    lib.rnn_model_reserve.argtypes = [vp, ci, ci]
    lib.rnn_forward.restype = ci
    lib.rnn_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, vp]
    lib.rnn_forward_static.restype = ci
    lib.rnn_forward_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, vp]
    lib.rnn_input_projection.restype = ci
    lib.rnn_input_projection.argtypes = [vp, ci, vp, vp, ci, vp]
    lib.rnn_model_check.restype = ci
    lib.rnn_model_check.argtypes = [vp]
    lib.rnn_model_set_clip.restype = ci
    lib.rnn_model_set_clip.argtypes = [vp, ctypes.c_float]
    lib.rnn_model_set_peepholes.restype = ci
    lib.rnn_model_set_peepholes.argtypes = [vp, ctypes.POINTER(vp), ci]
    lib.rnn_model_set_validation.restype = ci
    lib.rnn_model_set_validation.argtypes = [vp, ci]
    lib.rnn_stack_create.restype = ci
    lib.rnn_stack_create.argtypes = [ctypes.POINTER(vp), ci, ci, ci, ctypes.POINTER(ci), ci, ci, ctypes.POINTER(vp), ci]
    lib.rnn_stack_destroy.restype = None
    lib.rnn_stack_destroy.argtypes = [vp]
    lib.rnn_stack_runs.restype = ci
    lib.rnn_stack_runs.argtypes = [vp]
    lib.rnn_stack_run.restype = ci
    lib.rnn_stack_run.argtypes = [vp, ci, ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(vp)]
    lib.rnn_stack_device_bytes.restype = ctypes.c_size_t
    lib.rnn_stack_device_bytes.argtypes = [vp]
    lib.rnn_stack_forward.restype = ci
    lib.rnn_stack_forward.argtypes = [vp, vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, ctypes.POINTER(vp),
                                      ctypes.POINTER(vp), ci, ci, vp]
    lib.rnn_probe_exchange_step.restype = ci
    lib.rnn_probe_exchange_step.argtypes = [ci, ci, ci, ci] + [ctypes.POINTER(ctypes.c_double)] * 2 + [vp]
    lib.rnn_probe_matrix_rate.restype = ci
    lib.rnn_probe_matrix_rate.argtypes = [ci, ci] + [ctypes.POINTER(ctypes.c_double)] * 3 + [vp]
    lib.rnn_model_set_launch_tag.restype = ci
    lib.rnn_model_set_launch_tag.argtypes = [vp, ctypes.c_uint32]
    lib.rnn_model_set_batch_first.restype = ci
    lib.rnn_model_set_batch_first.argtypes = [vp, ci]
    lib.rnn_model_set_spin_limit.restype = ci
    lib.rnn_model_set_spin_limit.argtypes = [vp, ctypes.c_uint]
    lib.rnn_model_device_bytes.restype = ctypes.c_size_t
    lib.rnn_model_device_bytes.argtypes = [vp]
    lib.rnn_model_input_product_placement.restype = ci
    lib.rnn_model_input_product_placement.argtypes = [vp, ci, ci, ci, ctypes.POINTER(ci)]
    lib.rnn_plan_launches.restype = ci
    lib.rnn_plan_launches.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci, ci, ci, ctypes.c_size_t, ctypes.POINTER(ci),
                                      ctypes.POINTER(ci)]
    lib.rnn_plan_query.restype = ci
    lib.rnn_plan_query.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci, ci, ci, ctypes.c_size_t, ctypes.POINTER(ci),
                                   ctypes.POINTER(ci)]
    lib.rnn_status_string.restype = ctypes.c_char_p
    lib.rnn_status_string.argtypes = [ci]
    lib.rnn_model_set_profiling.restype = ci
    lib.rnn_model_set_profiling.argtypes = [vp, ci]
    lib.rnn_model_profile_read.restype = ci
    lib.rnn_model_profile_read.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_longlong)]
    lib.rnn_model_read_step_ticks.restype = ci
    lib.rnn_model_read_step_ticks.argtypes = [vp, vp, ctypes.c_size_t]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device or host address of a tensor / array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        assert t.flags["C_CONTIGUOUS"]
        return t.ctypes.data
    assert t.is_contiguous(), "tensors crossing the C ABI must be contiguous"
    return t.data_ptr()


def rnn_status_string(status: int) -> str:
    return load_library().rnn_status_string(int(status)).decode()


def rnn_model_create(cell: int, num_layers: int, input_size: int, hidden_size: int,
                     num_directions: int, dtype: int, weights: Sequence, weights_on_device: int) -> int:
    """weights: L*D*4 tensors/arrays/None in order (l, d, {W_ih, W_hh, b_ih, b_hh}).  Returns the handle."""
    lib = load_library()
    n = num_layers * num_directions * 4
    assert len(weights) == n
    arr = (ctypes.c_void_p * n)(*[_ptr(w) for w in weights])
    out = ctypes.c_void_p()
    rc = lib.rnn_model_create(ctypes.byref(out), cell, num_layers, input_size, hidden_size,
                              num_directions, dtype, arr, weights_on_device)
    if rc != RNN_OK:
        raise RnnError(rc, "rnn_model_create")
    return out.value


def rnn_model_create_ordered(cell: int, num_layers: int, input_size: int, hidden_size: int,
                             num_directions: int, dtype: int, weights: Sequence, weights_on_device: int,
                             gate_order: int) -> int:
    """rnn_model_create for weights whose gate row blocks are in `gate_order`.  Returns the handle."""
    lib = load_library()
    n = num_layers * num_directions * 4
    assert len(weights) == n
    arr = (ctypes.c_void_p * n)(*[_ptr(w) for w in weights])
    out = ctypes.c_void_p()
    rc = lib.rnn_model_create_ordered(ctypes.byref(out), cell, num_layers, input_size, hidden_size,
                                      num_directions, dtype, arr, weights_on_device, gate_order)
    if rc != RNN_OK:
        raise RnnError(rc, "rnn_model_create_ordered")
    return out.value


def rnn_model_destroy(model: Optional[int]) -> None:
    load_library().rnn_model_destroy(model)


def rnn_model_set_plan(model: int, plan: int) -> int:
    return load_library().rnn_model_set_plan(model, plan)


def rnn_model_set_gru_reset_before(model: int, on: int) -> int:
    return load_library().rnn_model_set_gru_reset_before(model, on)


def rnn_model_set_clip(model: int, clip: float) -> int:
    return load_library().rnn_model_set_clip(model, clip)


def rnn_model_set_peepholes(model: int, peepholes: Optional[Sequence], on_device: int) -> int:
    """peepholes: None, or L*D float32 tensors/arrays/None of 3*H values each."""
    lib = load_library()
    if peepholes is None:
        return lib.rnn_model_set_peepholes(model, None, on_device)
    arr = (ctypes.c_void_p * len(peepholes))(*[_ptr(q) for q in peepholes])
    return lib.rnn_model_set_peepholes(model, arr, on_device)


def rnn_model_set_batch_first(model: int, on: int) -> int:
    return load_library().rnn_model_set_batch_first(model, on)


def rnn_model_set_validation(model: int, on: int) -> int:
    return load_library().rnn_model_set_validation(model, on)


def rnn_model_set_launch_tag(model: int, tag: int) -> int:
    return load_library().rnn_model_set_launch_tag(model, tag)


def rnn_stack_create(cell: int, input_size: int, hidden_sizes: Sequence[int], num_directions: int, dtype: int,
                     weights: Sequence, weights_on_device: int) -> int:
    """weights: L*D*4 tensors/arrays/None in order (l, d, {W_ih, W_hh, b_ih, b_hh}).  Returns the handle."""
    L = len(hidden_sizes)
    n = L * num_directions * 4
    assert len(weights) == n
    arr = (ctypes.c_void_p * n)(*[_ptr(w) for w in weights])
    hs = (ctypes.c_int * L)(*[int(h) for h in hidden_sizes])
    out = ctypes.c_void_p()
    rc = load_library().rnn_stack_create(ctypes.byref(out), cell, L, input_size, hs, num_directions, dtype, arr,
                                         weights_on_device)
    if rc != RNN_OK:
        raise RnnError(rc, "rnn_stack_create")
    return out.value


def rnn_stack_destroy(stack: Optional[int]) -> None:
    load_library().rnn_stack_destroy(stack)


def rnn_stack_runs(stack: int) -> int:
    return load_library().rnn_stack_runs(stack)


def rnn_stack_run(stack: int, run: int):
    """Returns (status, first layer, layers, hidden size, model handle)."""
    a, b, c = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    m = ctypes.c_void_p()
    rc = load_library().rnn_stack_run(stack, run, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(m))
    return rc, a.value, b.value, c.value, m.value


def rnn_stack_device_bytes(stack: int) -> int:
    return load_library().rnn_stack_device_bytes(stack)


def _ptr_array(items):
    if items is None:
        return None
    return (ctypes.c_void_p * len(items))(*[_ptr(t) for t in items])


def rnn_stack_forward(stack: int, x, lengths, h0, c0, y, hT, cT, T: int, B: int, stream=None) -> int:
    """h0, c0, hT, cT: None or one tensor (or None) per run; see include/rnn.h."""
    s = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    return load_library().rnn_stack_forward(stack, _ptr(x), _ptr(lengths), _ptr_array(h0), _ptr_array(c0), _ptr(y),
                                            _ptr_array(hT), _ptr_array(cT), T, B, s)


def rnn_probe_exchange_step(groups: int, workgroups: int, words: int, steps: int, stream=None):
    """(status, microseconds per step, shader clocks per step); see include/rnn.h."""
    s = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    out = [ctypes.c_double(0.0) for _ in range(2)]
    rc = load_library().rnn_probe_exchange_step(groups, workgroups, words, steps, *[ctypes.byref(o) for o in out], s)
    return (rc,) + tuple(o.value for o in out)


def rnn_probe_matrix_rate(compute_units: int, iterations: int, stream=None):
    """(status, clocks per matrix instruction, shader GHz, TFLOP/s); see include/rnn.h."""
    s = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    out = [ctypes.c_double(0.0) for _ in range(3)]
    rc = load_library().rnn_probe_matrix_rate(compute_units, iterations, *[ctypes.byref(o) for o in out], s)
    return (rc,) + tuple(o.value for o in out)


def rnn_model_reserve(model: int, T: int, B: int) -> int:
    return load_library().rnn_model_reserve(model, T, B)


def rnn_forward(model: int, x, lengths, h0, c0, y, hT, cT, T: int, B: int, stream=None) -> int:
    """Arguments as in include/rnn.h; tensors are passed by device pointer.  `stream` is a
    torch.cuda.Stream, a raw hipStream_t value, or None for the default stream."""
    s = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    return load_library().rnn_forward(model, _ptr(x), _ptr(lengths), _ptr(h0), _ptr(c0), _ptr(y),
                                      _ptr(hT), _ptr(cT), T, B, s)


def rnn_forward_static(model: int, x, lengths, h0, c0, y, hT, cT, T: int, B: int, stream=None) -> int:
    """rnn_forward on the static scratch array of the device: allocates nothing (include/rnn.h)."""
    s = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    return load_library().rnn_forward_static(model, _ptr(x), _ptr(lengths), _ptr(h0), _ptr(c0), _ptr(y),
                                             _ptr(hT), _ptr(cT), T, B, s)


def rnn_input_projection(model: int, layer: int, inp, gx, rows: int, stream=None) -> int:
    s = stream.cuda_stream if hasattr(stream, "cuda_stream") else stream
    return load_library().rnn_input_projection(model, layer, _ptr(inp), _ptr(gx), rows, s)


def rnn_model_check(model: int) -> int:
    return load_library().rnn_model_check(model)


def rnn_model_set_spin_limit(model: int, polls: int) -> int:
    return load_library().rnn_model_set_spin_limit(model, polls)


def rnn_model_device_bytes(model: int) -> int:
    return int(load_library().rnn_model_device_bytes(model))


def rnn_model_input_product_placement(model: int, T: int, B: int, layer: int):
    """Returns (status, separate_launch)."""
    out = ctypes.c_int(-1)
    rc = load_library().rnn_model_input_product_placement(model, T, B, layer, ctypes.byref(out))
    return rc, out.value


PLAN_FIELDS = ("kind", "layers_per_launch", "row_tiles", "col_tiles", "chains", "row_blocks", "col_blocks", "launches")


def rnn_plan_query(cell: int, num_layers: int, input_size: int, hidden_size: int, num_directions: int, dtype: int,
                   requested_plan: int, T: int, B: int, compute_units: int, lds_bytes: int):
    """Host only (no GPU needed).  Returns (status, plan dict keyed by PLAN_FIELDS, separate_projection list)."""
    plan = (ctypes.c_int * 8)()
    sep = (ctypes.c_int * max(num_layers, 1))()
    rc = load_library().rnn_plan_query(cell, num_layers, input_size, hidden_size, num_directions, dtype,
                                       requested_plan, T, B, compute_units, lds_bytes, plan, sep)
    return rc, dict(zip(PLAN_FIELDS, list(plan))), list(sep)[:max(num_layers, 0)]


def rnn_plan_launches(cell: int, num_layers: int, input_size: int, hidden_size: int, num_directions: int, dtype: int,
                      requested_plan: int, T: int, B: int, compute_units: int, lds_bytes: int):
    """Host only (no GPU needed).  Returns (status, launch of every layer, group of every (layer, direction))."""
    lay = (ctypes.c_int * max(num_layers, 1))()
    grp = (ctypes.c_int * max(num_layers * num_directions, 1))()
    rc = load_library().rnn_plan_launches(cell, num_layers, input_size, hidden_size, num_directions, dtype,
                                          requested_plan, T, B, compute_units, lds_bytes, lay, grp)
    return rc, list(lay)[:max(num_layers, 0)], list(grp)[:max(num_layers * num_directions, 0)]


def rnn_model_set_profiling(model: int, flags: int) -> int:
    return load_library().rnn_model_set_profiling(model, flags)


def rnn_model_profile_read(model: int, kind: int):
    """Returns (status, total_ms, launches)."""
    ms = ctypes.c_double(0.0)
    n = ctypes.c_longlong(0)
    rc = load_library().rnn_model_profile_read(model, kind, ctypes.byref(ms), ctypes.byref(n))
    return rc, ms.value, n.value


def rnn_model_read_step_ticks(model: int, count: int):
    """Returns (status, uint64 array of `count` device clock values)."""
    out = np.zeros(count, dtype=np.uint64)
    rc = load_library().rnn_model_read_step_ticks(model, out.ctypes.data, count)
    return rc, out
