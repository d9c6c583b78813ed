"""rnn_forward_static (the entry point that allocates nothing) against rnn_forward, through the C ABI.

Both run the same kernels, so the results are compared bit for bit; two calls in a row share the device's
static array, the second with a smaller input, and rnn_forward is called between them on the same model.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2307_11339_amd import harness, rnn, workloads
    rnn.load_library()
    return harness, rnn, workloads


def _bits(io):
    import torch
    torch.cuda.synchronize()
    y = io.y.view(torch.int16 if io.y.dtype == torch.bfloat16 else torch.int32).cpu().numpy()
    return y, io.hT.cpu().numpy().view(np.uint32), io.cT.cpu().numpy().view(np.uint32)


def _forward_both(harness, rnn, model, wl):
    """(bits from rnn_forward, bits from rnn_forward_static) on the same inputs."""
    import torch
    c = wl.cfg
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    ref = _bits(io)
    st = torch.cuda.current_stream()
    io2 = harness.DeviceIO(wl)      # outputs start from the 7.0 pattern again
    rc = rnn.rnn_forward_static(model.handle, io2.x, io2.lengths, io2.h0, io2.c0, io2.y, io2.hT, io2.cT, c.T, c.B, st)
    assert rc == rnn.RNN_OK, rnn.rnn_status_string(rc)
    got = _bits(io2)
    # once more (every code object is loaded by now): the call takes no device memory
    io3 = harness.DeviceIO(wl)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    rc = rnn.rnn_forward_static(model.handle, io3.x, io3.lengths, io3.h0, io3.c0, io3.y, io3.hT, io3.cT, c.T, c.B, st)
    assert rc == rnn.RNN_OK, rnn.rnn_status_string(rc)
    again = _bits(io3)
    assert torch.cuda.mem_get_info()[0] == free_before
    for a, b in zip(got, again):
        assert np.array_equal(a, b)
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    return ref, got


SHAPES = [
    # name, cell, L, D, I, H, T, B, dtype, ragged: first the larger call, then a smaller one on the same array
    [("lstm_bf16_tagged", 0, 4, 1, 256, 256, 40, 6, 1, True), ("lstm_bf16_tagged_small", 0, 4, 1, 256, 256, 9, 2, 1, True)],
    [("gru_bf16_bidir", 1, 2, 2, 128, 128, 25, 20, 1, True), ("gru_bf16_bidir_small", 1, 2, 2, 128, 128, 7, 3, 1, False)],
    [("lstm_f32_grid", 0, 12, 1, 64, 64, 48, 8, 0, False), ("lstm_f32_grid_small", 0, 12, 1, 64, 64, 16, 1, 0, False)],
    [("lstm_bf16_large_batch", 0, 2, 1, 256, 256, 12, 300, 1, True), ("lstm_bf16_large_batch_small", 0, 2, 1, 256, 256, 5, 130, 1, True)],
    [("lstm_bf16_cellwise_width", 0, 2, 1, 40, 72, 9, 5, 1, True), ("lstm_bf16_padded_small", 0, 2, 1, 40, 72, 4, 2, 1, False)],
]


@pytest.mark.parametrize("pair", SHAPES, ids=[p[0][0] for p in SHAPES])
def test_static_equals_allocating_forward(gpu, pair):
    harness, rnn, W = gpu
    model = None
    for k, (name, cell, L, D, I, H, T, B, dtype, ragged) in enumerate(pair):
        cfg = W.Config(name, cell, L=L, D=D, I=I, H=H, T=T, B=B, dtype=dtype, seed=W.BASE_SEED + 700 + k,
                       h0_std=0.1, len_min=1 if ragged else None)
        wl = W.make_workload(cfg)
        if model is None:
            model = harness.DeviceModel(wl)     # the pair shares one model: same weights, two call shapes
        else:
            wl.weights = first_weights
        first_weights = wl.weights
        ref, got = _forward_both(harness, rnn, model, wl)
        for a, b in zip(ref, got):
            assert np.array_equal(a, b), name
    model.close()


def test_two_models_share_the_array_in_turn(gpu):
    """Calls of two models alternate on one stream: each starts from whatever the other left in the array."""
    harness, rnn, W = gpu
    cfgs = [W.Config("a", W.LSTM, L=3, D=1, I=128, H=128, T=20, B=4, dtype=W.BF16, seed=W.BASE_SEED + 720),
            W.Config("b", W.GRU, L=2, D=1, I=256, H=256, T=11, B=9, dtype=W.BF16, seed=W.BASE_SEED + 721, h0_std=0.1)]
    wls = [W.make_workload(c) for c in cfgs]
    models = [harness.DeviceModel(w) for w in wls]
    for _ in range(3):
        for m, w in zip(models, wls):
            ref, got = _forward_both(harness, rnn, m, w)
            for a, b in zip(ref, got):
                assert np.array_equal(a, b)
    for m in models:
        m.close()


def test_shape_beyond_the_array_is_refused(gpu):
    import torch
    harness, rnn, W = gpu
    cfg = W.Config("big", W.LSTM, L=2, D=2, I=512, H=512, T=256, B=64, dtype=W.BF16, seed=W.BASE_SEED + 730)
    wl = W.make_workload(cfg)
    model = harness.DeviceModel(wl)
    io = harness.DeviceIO(wl)
    rc = rnn.rnn_forward_static(model.handle, io.x, None, None, None, io.y, io.hT, io.cT, cfg.T, cfg.B,
                                torch.cuda.current_stream())
    assert rc == rnn.RNN_ESCRATCH
    assert "static" in rnn.rnn_status_string(rc)
    torch.cuda.synchronize()
    assert float(io.y.float().min()) == 7.0      # nothing ran
    # the model still works through the allocating entry point, and a shape that fits still runs
    harness.forward(model, io)
    small = wl.take_batch([0, 1])
    small_cfg = small.cfg.scaled(T=16)
    small.x = np.ascontiguousarray(small.x[:16]); small.cfg = small_cfg
    io2 = harness.DeviceIO(small)
    rc = rnn.rnn_forward_static(model.handle, io2.x, None, None, None, io2.y, io2.hT, io2.cT, 16, 2,
                                torch.cuda.current_stream())
    assert rc == rnn.RNN_OK
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    model.close()
