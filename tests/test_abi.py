"""The C-ABI library loads without a GPU and exports every function include/rnn.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="rnn.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rnn_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2307_11339_amd import _build, rnn
    if not os.path.exists(rnn.LIB_PATH):
        _build.build(force=True)
    return rnn.load_library()


def test_header_declares_the_entry_points():
    names = declared_functions()
    for required in ("rnn_model_create", "rnn_model_destroy", "rnn_forward", "rnn_input_projection",
                     "rnn_status_string", "rnn_model_device_bytes"):
        assert required in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2307_11339_amd import rnn
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert sorted(rnn.EXPORTS) == declared_functions()


def test_every_header_is_covered(lib):
    """include/ holds two headers; every function either declares is exported and bound."""
    from paper_2307_11339_amd import schedule
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["rnn.h", "rnn_schedule.h"]
    names = declared_functions("rnn_schedule.h")
    assert names == sorted(schedule.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name


def test_host_only_calls(lib):
    from paper_2307_11339_amd import rnn
    assert rnn.rnn_status_string(rnn.RNN_OK) == "ok"
    assert "unsupported" in rnn.rnn_status_string(rnn.RNN_EUNSUPPORTED)
    assert rnn.rnn_status_string(12345) == "unknown status"
    # argument validation happens before any device call
    out = ctypes.c_void_p()
    assert lib.rnn_model_create(ctypes.byref(out), 0, 1, 8, 8, 1, 0, None, 0) == rnn.RNN_EINVAL
    assert lib.rnn_model_create(None, 0, 1, 8, 8, 1, 0, None, 0) == rnn.RNN_EINVAL
    assert rnn.rnn_model_device_bytes(None) == 0
    assert rnn.rnn_model_check(None) == rnn.RNN_EINVAL
    assert rnn.rnn_model_set_spin_limit(None, 5) == rnn.RNN_EINVAL
    rnn.rnn_model_destroy(None)
    # the stack of layers of different widths and the probes refuse bad arguments before touching a device
    assert lib.rnn_stack_create(None, 0, 1, 8, None, 1, 0, None, 0) == rnn.RNN_EINVAL
    assert lib.rnn_stack_create(ctypes.byref(out), 0, 1, 8, None, 1, 0, None, 0) == rnn.RNN_EINVAL
    assert rnn.rnn_stack_runs(None) == 0 and rnn.rnn_stack_device_bytes(None) == 0
    assert rnn.rnn_stack_run(None, 0)[0] == rnn.RNN_EINVAL
    assert rnn.rnn_stack_forward(None, None, None, None, None, None, None, None, 1, 1, None) == rnn.RNN_EINVAL
    rnn.rnn_stack_destroy(None)
    assert rnn.rnn_probe_matrix_rate(0, 10, None)[0] == rnn.RNN_EINVAL
    assert rnn.rnn_probe_exchange_step(1, 8, 60, 10, None)[0] == rnn.RNN_EINVAL


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2307_11339_amd import rnn
    monkeypatch.setattr(rnn, "_lib", None)
    monkeypatch.setattr(rnn, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "librnn_mi355x.so"))
    with pytest.raises(ImportError):
        rnn.load_library()
