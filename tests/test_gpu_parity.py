"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Tolerances (max-abs over y, hT, cT): 1e-4 for fp32 models, 2e-2 for bf16 models with fp32
accumulation; padded positions of y must be +0.0 bit patterns.
"""
import os
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = {0: 1e-4, 1: 2e-2}


def _say(msg):
    sys.stdout.write(msg + "\n")
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2307_11339_amd import harness, rnn, workloads
    rnn.load_library()  # fails loudly when the HIP library has not been built
    return harness, rnn, workloads


def _check(harness, wl, io, ref, rows=None, tol=None):
    """Compare device results with oracle results ref = (y, hT, cT); rows = batch rows that ref covers."""
    c = wl.cfg
    tol = TOL[c.dtype] if tol is None else tol
    y, hT, cT, ybits = harness.results(io)
    ry, rh, rc = ref
    if rows is not None:
        y, hT, ybits = y[:, rows], hT[:, rows], ybits[:, rows]
        cT = cT[:, rows] if cT is not None else None
        lengths = None if wl.lengths is None else wl.lengths[rows]
    else:
        lengths = wl.lengths
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(hT))
    err_y = float(np.max(np.abs(y - ry)))
    err_h = float(np.max(np.abs(hT - rh)))
    err_c = float(np.max(np.abs(cT - rc))) if (rc is not None and cT is not None) else 0.0
    _say("    max-abs error y %.3e hT %.3e cT %.3e (tolerance %.0e)" % (err_y, err_h, err_c, tol))
    assert err_y <= tol and err_h <= tol and err_c <= tol
    if lengths is not None:
        for j, n in enumerate(lengths):
            assert np.all(ybits[int(n):, j] == 0), "padded positions must be +0.0 bit patterns"
    return max(err_y, err_h, err_c)


SMALL = [
    # name, cell, L, D, I, H, T, B, dtype, ragged lengths, h0
    ("lstm_bf16_3layer", 0, 3, 1, 64, 128, 9, 5, 1, True, True),
    ("gru_bf16_2layer", 1, 2, 1, 72, 256, 7, 19, 1, True, True),
    ("lstm_bf16_bidir", 0, 2, 2, 40, 128, 11, 37, 1, True, True),
    ("gru_bf16_bidir", 1, 2, 2, 64, 128, 6, 3, 1, True, False),
    ("lstm_f32_4layer", 0, 4, 1, 20, 64, 10, 3, 0, True, True),
    ("gru_f32_bidir", 1, 2, 2, 12, 32, 8, 18, 0, True, True),
    ("lstm_f32_wide", 0, 1, 1, 64, 128, 5, 70, 0, False, False),
    ("lstm_bf16_oddshape", 0, 2, 1, 24, 72, 5, 4, 1, True, True),   # H not a multiple of 128: runs padded to 128 units
    # widths between the compiled ones run padded to the next one (zero weights and zero state in the added units)
    ("gru_bf16_padded_h200_bidir", 1, 2, 2, 40, 200, 6, 9, 1, True, True),     # 200 -> 256, both directions: [fwd | bwd] re-spaced
    ("lstm_f32_padded_h100", 0, 3, 1, 100, 100, 7, 5, 0, True, True),          # fp32 100 -> 128
    ("lstm_f32_padded_h20", 0, 2, 1, 12, 20, 8, 3, 0, True, True),             # fp32 20 -> 32
    ("lstm_bf16_padded_h896_inside", 0, 2, 1, 896, 896, 5, 130, 1, True, True),  # 896 -> 1024 at a large batch
    ("lstm_bf16_t1", 0, 2, 1, 64, 128, 1, 2, 1, False, True),
    # small batches, several layers in one launch of the tag-in-data kernel (fused layers have their own waves
    # for the input product): taller tiles, a quarter too large to be requested a step early, fp32
    ("lstm_bf16_8layer_h256", 0, 8, 1, 48, 256, 12, 3, 1, True, True),     # 8 layers x 16 workgroups, 16-row tiles x 4
    ("gru_bf16_2layer_h1024_b12", 1, 2, 1, 40, 1024, 6, 12, 1, True, True),  # x fetched after the barriers (12 x 128 words per wave)
    ("lstm_bf16_4layer_sq_h1024_b1", 0, 4, 1, 1024, 1024, 7, 1, 1, False, True),   # one load instruction per wave: the lean fetch loop
    ("gru_bf16_3layer_h1024_b6", 1, 3, 1, 1024, 1024, 5, 6, 1, True, True),   # 6 x 128 words per wave: probe word, then the generic fetch of six instructions
    ("lstm_bf16_2layer_h1024_b3", 0, 2, 1, 1024, 1024, 5, 3, 1, True, True),  # 3 x 128 words per wave: three instructions, fetched outright
    ("lstm_f32_6layer_h128", 0, 6, 1, 24, 128, 9, 5, 0, True, True),
    ("gru_bf16_4layer_h512_t1", 1, 4, 1, 32, 512, 1, 2, 1, False, True),   # a single step
    # input as wide as the layer: the first layer of the launch multiplies the plain input itself (no projection)
    ("lstm_bf16_3layer_sq_h256", 0, 3, 1, 256, 256, 11, 7, 1, True, True),
    ("gru_f32_2layer_sq_h64", 1, 2, 1, 64, 64, 9, 19, 0, True, True),
    ("lstm_bf16_1layer_sq_h512", 0, 1, 1, 512, 512, 8, 1, 1, False, False),
    # input half as wide as the layer, and both directions (first layer H/2 or H wide, upper layer 2H wide)
    ("gru_bf16_3layer_half_h256", 1, 3, 1, 128, 256, 10, 6, 1, True, True),
    ("lstm_f32_half_h64", 0, 1, 1, 32, 64, 7, 33, 0, True, True),
    ("lstm_bf16_bidir_sq_h256", 0, 2, 2, 256, 256, 9, 20, 1, True, True),
    ("gru_bf16_bidir_half_h128", 1, 2, 2, 64, 128, 8, 5, 1, True, False),
    # fp32 layers of 256 and 512 units (tag-in-data kernel: 16 and 32 K blocks of 4 per wave)
    ("lstm_f32_2layer_sq_h256", 0, 2, 1, 256, 256, 7, 5, 0, True, True),
    ("gru_f32_3layer_h512", 1, 3, 1, 100, 512, 5, 3, 0, True, True),
    ("lstm_f32_half_h256", 0, 2, 1, 128, 256, 6, 1, 0, False, True),
    ("gru_f32_bidir_h256_b20", 1, 2, 2, 256, 256, 5, 20, 0, True, True),
    # bf16 layers whose width is not 128 times a power of two (3, 5, 6, 10, 12 K blocks per wave), and 2048 units
    ("lstm_bf16_2layer_sq_h384", 0, 2, 1, 384, 384, 6, 5, 1, True, True),
    ("gru_bf16_2layer_half_h640", 1, 2, 1, 320, 640, 5, 3, 1, True, True),
    ("lstm_bf16_3layer_sq_h768_b20", 0, 3, 1, 768, 768, 5, 20, 1, True, True),
    ("lstm_bf16_bidir_sq_h768", 0, 2, 2, 768, 768, 5, 4, 1, True, True),
    ("gru_bf16_2layer_sq_h1280", 1, 2, 1, 1280, 1280, 4, 2, 1, True, True),
    ("lstm_bf16_2layer_sq_h1536", 0, 2, 1, 1536, 1536, 4, 3, 1, True, True),
    ("lstm_bf16_2layer_sq_h2048", 0, 2, 1, 2048, 2048, 4, 2, 1, True, True),
    ("lstm_bf16_20layer_h256", 0, 20, 1, 256, 256, 6, 2, 1, True, True),     # two launches: the second reads the first's output
    ("gru_bf16_sq_h128_t1", 1, 2, 1, 128, 128, 1, 3, 1, False, True),          # a single step, input read by the x waves
    # a state of more than four load instructions per wave (16 sequences x 64 or 128 words): fetched outright in
    # segments; a last block of 5 sequences, a second half of 4
    ("lstm_bf16_bidir_h512_b37", 0, 2, 2, 64, 512, 6, 37, 1, True, True),
    ("lstm_bf16_b300", 0, 1, 1, 64, 512, 6, 300, 1, True, True),    # large batch: flag-vector kernel, two chains per workgroup
    ("gru_bf16_b256_bidir", 1, 1, 2, 64, 128, 5, 256, 1, True, True),  # large batch, both directions
    ("lstm_bf16_b299", 0, 2, 1, 64, 512, 6, 299, 1, True, True),    # batch not a multiple of 4: padded rows in the blocked state
    # Large batch, wide enough that a layer needs every compute unit: one persistent launch per layer.
    # Layers whose input has the layer's own width compute W_ih x_t inside the recurrent kernel; layers
    # above the first read the state sequence of the layer below.  Checked on 24 sampled sequences.
    ("lstm_bf16_inside", 0, 2, 1, 64, 512, 40, 512, 1, True, True),      # first layer projects (I != H)
    ("gru_bf16_inside", 1, 3, 1, 64, 512, 33, 512, 1, True, True),
    ("lstm_bf16_inside_sq", 0, 2, 1, 512, 512, 21, 500, 1, True, True),  # I == H: no projection launch; ragged batch tail
    ("gru_bf16_inside_sq", 1, 2, 1, 512, 512, 17, 512, 1, True, False),
    ("lstm_f32_inside_sq", 0, 2, 1, 128, 128, 9, 512, 0, True, True),
    ("lstm_bf16_inside_t1", 0, 2, 1, 512, 512, 1, 512, 1, False, True),    # a single step: nothing to pipeline
    ("gru_bf16_inside_t2", 1, 2, 1, 512, 512, 2, 497, 1, True, True),      # two steps, ragged lengths 1..2, ragged batch
    ("lstm_bf16_inside_1layer", 0, 1, 1, 512, 512, 19, 512, 1, True, False),  # one layer: input re-laid out, output written
    ("lstm_f32_inside_b501", 0, 2, 1, 128, 128, 6, 501, 0, True, True),
    # widths that are not 128 times a power of two (3, 5, 6 K blocks per wave) at a large batch
    ("lstm_bf16_inside_sq_h768", 0, 2, 1, 768, 768, 7, 300, 1, True, True),
    ("lstm_bf16_inside_h768_i64", 0, 2, 1, 64, 768, 6, 290, 1, True, True),       # first layer: projection + flag-vector kernel
    ("gru_bf16_inside_sq_h384", 1, 2, 1, 384, 384, 9, 512, 1, True, True),
    ("lstm_bf16_inside_sq_h640", 0, 2, 1, 640, 640, 5, 256, 1, True, False),
    ("lstm_bf16_sidebyside_h768_l4", 0, 4, 1, 768, 768, 6, 64, 1, True, True),
    # more sequences than one persistent launch holds: passes over blocks of sequences (256 + 44; 16 + 2)
    ("lstm_bf16_inside_passes_b300", 0, 2, 1, 1024, 1024, 5, 300, 1, True, True),
    ("gru_bf16_passes_h2048_b18", 1, 1, 1, 2048, 2048, 3, 18, 1, True, True),
    # more than 1024 units at a large batch: workgroups of 8 units (x inside; a narrower first layer projects)
    ("lstm_bf16_inside_sq_h2048_b64", 0, 2, 1, 2048, 2048, 3, 64, 1, True, True),
    ("gru_bf16_inside_h1280_i64_b100", 1, 2, 1, 64, 1280, 4, 100, 1, True, True),     # 64 + 36 sequences
    ("lstm_bf16_inside_sq_h1536_b50", 0, 1, 1, 1536, 1536, 4, 50, 1, True, False),
    ("lstm_bf16_padded_h896_inside_passes", 0, 1, 1, 896, 896, 3, 300, 1, True, True),   # padded to 1024 and 256 + 44 sequences    # odd batch in fp32: padded rows in the blocked state
    # Wide layers at a medium batch: several layers share one launch of the flag-vector kernel, the upper
    # ones fused (x_t taken from the layer below as it is produced).  Checked on sampled sequences.
    ("lstm_bf16_fusedflag_l4", 0, 4, 1, 64, 1024, 5, 40, 1, True, True),    # 4 layers x 64 workgroups, tiles of 64 sequences
    ("gru_bf16_fusedflag_l2", 1, 2, 1, 64, 1024, 6, 100, 1, True, True),    # 2 layers x 128 workgroups, two chains of 32
    # the same regime with inputs as wide as the layers: several layers side by side in the inside-product kernel, the
    # upper ones reading the state sequence below them behind its flags
    ("lstm_bf16_sidebyside_l4", 0, 4, 1, 1024, 1024, 7, 40, 1, True, True),   # 4 layers x 64 workgroups, two chains of 32
    ("gru_bf16_sidebyside_l2", 1, 2, 1, 512, 512, 9, 100, 1, True, True),     # 2 layers x 128 workgroups
    ("lstm_bf16_sidebyside_l3_t1", 0, 3, 1, 512, 512, 1, 64, 1, False, True),  # a single step
    # narrow fp32 layers at a large batch: a K quarter of a wave is narrower than a cache line of the state (H = 32)
    # or of the output of the layer below (H = 32, 64), so a wave waits for the row blocks of the whole line
    ("lstm_f32_fusedflag_h32", 0, 2, 1, 20, 32, 7, 300, 0, True, True),
    ("gru_f32_fusedflag_h64", 1, 3, 1, 24, 64, 6, 290, 0, True, True),
    ("lstm_f32_fusedflag_l6_h32", 0, 6, 1, 20, 32, 7, 300, 0, True, True),   # six layers in one launch of the flag-vector kernel
]
SAMPLED = ("_inside", "_fusedflag", "_sidebyside")


def _small_workload(W, spec):
    name, cell, L, D, I, H, T, B, dtype, ragged, use_h0 = spec
    cfg = W.Config(name, cell, L=L, D=D, I=I, H=H, T=T, B=B, dtype=dtype,
                   seed=W.BASE_SEED + 1000 + sum(map(ord, name)), h0_std=0.5 if use_h0 else 0.0,
                   len_min=1 if ragged else None)
    wl = W.make_workload(cfg, zero_pad_x=False)   # padding content must not matter
    if use_h0 and cell == 0:
        rng = np.random.default_rng(cfg.seed + 7)
        wl.c0 = rng.uniform(-1, 1, size=(L * D, B, H)).astype(np.float32)
    return wl


@pytest.mark.parametrize("plan", ["cellwise", "wavefront"])
@pytest.mark.parametrize("spec", SMALL, ids=[s[0] for s in SMALL])
def test_small_shapes(gpu, oracle, spec, plan):
    harness, rnn, W = gpu
    wl = _small_workload(W, spec)
    _say("\n  case %s plan %s cfg %s" % (spec[0], plan, wl.cfg))
    pid = rnn.RNN_PLAN_CELLWISE if plan == "cellwise" else rnn.RNN_PLAN_WAVEFRONT
    try:
        model = harness.DeviceModel(wl, plan=pid)
    except rnn.RnnError as e:
        assert plan == "wavefront" and e.status == rnn.RNN_EUNSUPPORTED and spec[0] == "lstm_bf16_oddshape"
        return
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    if any(k in spec[0] for k in SAMPLED):
        rows = np.unique(np.linspace(0, wl.cfg.B - 1, 24).astype(int))
        ref = oracle.forward_workload(wl.take_batch(rows), nthreads=8)
        _check(harness, wl, io, ref, rows=rows)
    else:
        ref = oracle.forward_workload(wl, nthreads=8)
        _check(harness, wl, io, ref)
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    # a second call on the same model gives identical bits (fixed reduction order, flags reset)
    y1 = io.y.clone()
    harness.forward(model, io)
    import torch
    torch.cuda.synchronize()
    assert torch.equal(y1, io.y)
    model.close()


# models whose upper layers wait a long time at the start of a launch (the layers below have to get there first)
@pytest.mark.parametrize("name", ["lstm_bf16_8layer_h256", "lstm_bf16_20layer_h256",  # tag-in-data kernel (8 and 16 layers in a launch)
                                  "lstm_bf16_sidebyside_l4",                           # inside-product kernel
                                  "lstm_f32_fusedflag_l6_h32"])                        # flag-vector kernel
def test_abandoned_wait_is_reported_and_the_model_recovers(gpu, oracle, name):
    """A poll budget of one makes healthy launches give up: a wait that is still unsuccessful when the
    kernel first looks at its budget (after 8 polls) is abandoned, the launch still drains (all later
    waits return at once), rnn_model_check reports it once, and the next forward with the default
    budget is correct again."""
    harness, rnn, W = gpu
    import torch
    spec = [s for s in SMALL if s[0] == name][0]
    wl = _small_workload(W, spec)
    _say("\n  case %s, poll budget 1" % name)
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
    io = harness.DeviceIO(wl)
    harness.forward(model, io)            # sizes the workspace, healthy
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    assert rnn.rnn_model_set_spin_limit(model.handle, 1) == rnn.RNN_OK
    for _ in range(5):                    # the launches end by themselves
        harness.forward(model, io)
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_EDEVICE
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK          # reported once, then lowered
    assert rnn.rnn_model_set_spin_limit(model.handle, 0) == rnn.RNN_OK
    harness.forward(model, io)
    rows = np.unique(np.linspace(0, wl.cfg.B - 1, 12).astype(int))
    ref = oracle.forward_workload(wl.take_batch(rows), nthreads=8)
    _check(harness, wl, io, ref, rows=rows)
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    model.close()


def test_null_optionals_and_device_weights(gpu, oracle):
    harness, rnn, W = gpu
    wl = _small_workload(W, SMALL[0])
    wl.h0 = None; wl.c0 = None; wl.lengths = None
    for plan in (rnn.RNN_PLAN_CELLWISE, rnn.RNN_PLAN_WAVEFRONT):
        model = harness.DeviceModel(wl, plan=plan, weights_on_device=True)
        io = harness.DeviceIO(wl, want_state=False)
        harness.forward(model, io)
        ref = oracle.forward_workload(wl, nthreads=8)
        y, _, _, _ = harness.results(io)
        assert np.max(np.abs(y - ref[0])) <= TOL[wl.cfg.dtype]
        model.close()


def test_chained_calls_equal_one_call(gpu):
    """hT/cT of one call fed as h0/c0 of the next reproduce the single long call bit for bit."""
    import torch
    harness, rnn, W = gpu
    cfg = W.Config("chain", 0, L=2, D=1, I=64, H=128, T=12, B=4, dtype=1, seed=W.BASE_SEED + 77)
    wl = W.make_workload(cfg)
    for plan in (rnn.RNN_PLAN_CELLWISE, rnn.RNN_PLAN_WAVEFRONT):
        model = harness.DeviceModel(wl, plan=plan)
        io = harness.DeviceIO(wl)
        harness.forward(model, io)
        torch.cuda.synchronize()
        k = 5
        ya = torch.empty((k, cfg.B, cfg.H), dtype=torch.bfloat16, device="cuda")
        yb = torch.empty((cfg.T - k, cfg.B, cfg.H), dtype=torch.bfloat16, device="cuda")
        h1, c1 = torch.empty_like(io.hT), torch.empty_like(io.cT)
        h2, c2 = torch.empty_like(io.hT), torch.empty_like(io.cT)
        xa, xb = io.x[:k].contiguous(), io.x[k:].contiguous()
        assert rnn.rnn_forward(model.handle, xa, None, None, None, ya, h1, c1, k, cfg.B, torch.cuda.current_stream()) == 0
        assert rnn.rnn_forward(model.handle, xb, None, h1, c1, yb, h2, c2, cfg.T - k, cfg.B, torch.cuda.current_stream()) == 0
        torch.cuda.synchronize()
        assert torch.equal(torch.cat([ya, yb]), io.y)
        assert torch.equal(h2, io.hT) and torch.equal(c2, io.cT)
        model.close()


def test_input_projection(gpu, oracle):
    import torch
    harness, rnn, W = gpu
    # the last two cases take the large-tile kernel: ragged last row tile, K not a multiple of 64
    for dtype, cell, rows, I, H, D in ((1, 0, 300, 72, 128, 2), (0, 1, 70, 20, 32, 1), (1, 1, 2100, 256, 128, 1),
                                       (1, 0, 4500, 72, 128, 1), (1, 0, 4096, 320, 128, 2)):
        cfg = W.Config("proj", cell, L=1, D=D, I=I, H=H, T=rows, B=1, dtype=dtype, seed=W.BASE_SEED + 55)
        wl = W.make_workload(cfg)
        model = harness.DeviceModel(wl)
        x = harness.to_device_storage(wl.x.reshape(rows, I), dtype)
        gx = torch.full((rows, D, H, 4), 9.0, device="cuda")
        assert rnn.rnn_input_projection(model.handle, 0, x, gx, rows, torch.cuda.current_stream()) == 0
        torch.cuda.synchronize()
        got = gx.cpu().numpy().astype(np.float64)
        G = cfg.G
        for d in range(D):
            P = oracle.projection(wl.x.reshape(rows, I), wl.weight(0, d, 0)).reshape(rows, G, H)
            exp = np.zeros((rows, H, 4))
            for s in range(G):
                exp[:, :, s] = P[:, s, :]          # LSTM i,f,g,o / GRU r,z,n -> slots 0..G-1
            err = np.max(np.abs(got[:, d] - exp))
            _say("    projection dtype %d rows %d error %.3e" % (dtype, rows, err))
            assert err <= 1e-4     # exact products, fp32 accumulation over at most 320 terms
        model.close()


def test_input_projection_at_full_size(gpu, oracle):
    """The projection of one layer of the headline workload over all its time steps (131072 x 1024 times
    1024 x 4096): the shape the large-tile kernel with the XCD-blocked tile order is made for.  The oracle computes
    sampled rows, among them the first and last row of a tile, of an XCD band and of the matrix."""
    import torch
    harness, rnn, W = gpu
    base = W.CONFIGS["C5"]
    rows, I, H = base.T * base.B, base.I, base.H
    cfg = W.Config("proj_full", base.cell, L=1, D=1, I=I, H=H, T=1, B=1, dtype=base.dtype, seed=W.BASE_SEED + 56)
    wl = W.make_workload(cfg)
    model = harness.DeviceModel(wl)
    g = torch.Generator(device="cpu").manual_seed(W.BASE_SEED + 57)
    a = torch.randn(rows, I, generator=g, dtype=torch.float32).to(torch.bfloat16)
    x = a.cuda()
    gx = torch.full((rows, 1, H, 4), 9.0, device="cuda")
    assert rnn.rnn_input_projection(model.handle, 0, x, gx, rows, torch.cuda.current_stream()) == 0
    torch.cuda.synchronize()
    pick = [0, 1, 31, 32, 255, 256, 2047, 2048, 16383, 16384, 16385, 65535, 65536, 70001, 114687, 114688,
            rows - 257, rows - 256, rows - 2, rows - 1]
    got = gx[pick, 0].cpu().numpy().astype(np.float64)                     # [n, H, 4]
    P = oracle.projection(a[pick].to(torch.float64).numpy(), wl.weight(0, 0, 0)).reshape(len(pick), 4, H)
    exp = np.transpose(P, (0, 2, 1))
    err = np.max(np.abs(got - exp))
    _say("    projection %d x %d x %d: %d sampled rows, error %.3e" % (rows, I, 4 * H, len(pick), err))
    assert err <= 3e-4     # exact products, fp32 accumulation over 1024 terms of size <= ~0.2
    # every row was written: no element still holds the fill value
    assert int((gx == 9.0).sum().item()) == 0
    model.close()


STACKS = [
    # name, cell, D, I, hidden sizes per layer, T, B, dtype
    ("lstm_bf16_128_128_256_64", 0, 1, 64, [128, 128, 256, 64], 9, 5, 1),       # 64 runs padded to 128 units
    ("gru_f32_bidir_32_64_64", 1, 2, 12, [32, 64, 64], 8, 3, 0),
    ("lstm_bf16_narrowing_512_256_128_b40", 0, 1, 256, [512, 256, 256, 128], 12, 40, 1),
    ("lstm_f32_one_run", 0, 1, 20, [64, 64], 6, 4, 0),                         # one run: the same as a plain model
]


@pytest.mark.parametrize("spec", STACKS, ids=[s[0] for s in STACKS])
def test_layers_of_different_hidden_sizes(gpu, oracle, spec):
    """A stack whose layers differ in width runs as a chain of models, one per run of equal width, each planned on its
    own.  The oracle runs the same chain: every run on the (fp64) output of the one below."""
    import torch
    harness, rnn, W = gpu
    name, cell, D, I, hs, T, B, dtype = spec
    # runs of equal width, each a workload of its own (its input as wide as the output below it)
    runs, l = [], 0
    while l < len(hs):
        n = 1
        while l + n < len(hs) and hs[l + n] == hs[l]:
            n += 1
        runs.append((l, n, hs[l]))
        l += n
    wls = []
    for r, (l0, n, H) in enumerate(runs):
        i_r = I if r == 0 else D * runs[r - 1][2]
        cfg = W.Config("%s_run%d" % (name, r), cell, L=n, D=D, I=i_r, H=H, T=T, B=B, dtype=dtype,
                       seed=W.BASE_SEED + 700 + 10 * STACKS.index(spec) + r, len_min=max(1, T // 2), h0_std=0.5)
        wls.append(W.make_workload(cfg))
    lengths = wls[0].lengths
    weights = []
    for wl in wls:
        for w in wl.weights:
            weights.append(W.f32_to_bf16_bits(w).reshape(w.shape) if dtype == W.BF16 else np.ascontiguousarray(w, dtype=np.float32))
    stack = rnn.rnn_stack_create(cell, I, hs, D, dtype, weights, 0)
    try:
        assert rnn.rnn_stack_runs(stack) == len(runs)
        for r, (l0, n, H) in enumerate(runs):
            rc, a, b, c, handle = rnn.rnn_stack_run(stack, r)
            assert (rc, a, b, c) == (rnn.RNN_OK, l0, n, H) and handle
            assert rnn.rnn_model_set_plan(handle, rnn.RNN_PLAN_WAVEFRONT) == rnn.RNN_OK
        assert rnn.rnn_stack_run(stack, len(runs))[0] == rnn.RNN_EINVAL
        tdt = torch.bfloat16 if dtype == W.BF16 else torch.float32
        x = harness.to_device_storage(wls[0].x, dtype)
        dl = torch.from_numpy(lengths).to("cuda")
        h0 = [torch.from_numpy(wl.h0).to("cuda") for wl in wls]
        y = torch.full((T, B, D * hs[-1]), 7.0, dtype=tdt, device="cuda")
        hT = [torch.full((n * D, B, H), 7.0, device="cuda") for (_, n, H) in runs]
        cT = [torch.full((n * D, B, H), 7.0, device="cuda") for (_, n, H) in runs]
        for call in range(2):          # the second call finds the buffers between the runs in place
            assert rnn.rnn_stack_forward(stack, x, dl, h0, None, y, hT, cT, T, B, torch.cuda.current_stream()) == rnn.RNN_OK
        torch.cuda.synchronize()
        assert rnn.rnn_stack_device_bytes(stack) > 0
        # the oracle, run by run
        inp = wls[0].x
        tol = TOL[dtype]
        for r, wl in enumerate(wls):
            c = wl.cfg
            ry, rh, rc_ = oracle.forward(c.cell, c.L, c.D, c.I, c.H, wl.weights, inp, lengths, wl.h0, None, nthreads=4)
            got_h = hT[r].cpu().numpy().astype(np.float64)
            err_h = float(np.max(np.abs(got_h - rh)))
            err_c = float(np.max(np.abs(cT[r].cpu().numpy().astype(np.float64) - rc_))) if cell == 0 else 0.0
            _say("    run %d (%d layers of %d units): hT error %.3e cT error %.3e" % (r, c.L, c.H, err_h, err_c))
            assert err_h <= tol and err_c <= tol
            inp = ry
        got_y = y.float().cpu().numpy().astype(np.float64)
        err_y = float(np.max(np.abs(got_y - inp)))
        _say("    y error %.3e (tolerance %.0e)" % (err_y, tol))
        assert err_y <= tol
        for j, n in enumerate(lengths):
            assert not np.any(got_y[int(n):, j]), "padded positions must be zero"
        for handle in [rnn.rnn_stack_run(stack, r)[4] for r in range(len(runs))]:
            assert rnn.rnn_model_check(handle) == rnn.RNN_OK
    finally:
        torch.cuda.synchronize()
        rnn.rnn_stack_destroy(stack)


def test_forward_launches_what_the_scheduler_placed(gpu):
    """The number of persistent launches a forward pass really makes (counted by the kernel events) is the number of
    passes in the scheduler's placement that rnn_plan_launches reports for the same shape on this device."""
    import torch
    harness, rnn, W = gpu
    prop = torch.cuda.get_device_properties(0)
    by_name = {s[0]: s for s in SMALL}
    cases = [W.CONFIGS["C2"], W.CONFIGS["C4"], W.paper_grid()[0], W.paper_grid()[3],
             W.CONFIGS["C5"].scaled(T=6, B=40), W.CONFIGS["C5"].scaled(T=5, B=1),
             _small_workload(W, by_name["lstm_bf16_inside_sq"]).cfg]
    for cfg in cases:
        wl = W.make_workload(cfg)
        model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
        io = harness.DeviceIO(wl)
        rc, launch, group = rnn.rnn_plan_launches(cfg.cell, cfg.L, cfg.I, cfg.H, cfg.D, cfg.dtype, rnn.RNN_PLAN_WAVEFRONT,
                                                  cfg.T, cfg.B, prop.multi_processor_count, prop.shared_memory_per_block)
        assert rc == rnn.RNN_OK
        rcq, plan, _ = rnn.rnn_plan_query(cfg.cell, cfg.L, cfg.I, cfg.H, cfg.D, cfg.dtype, rnn.RNN_PLAN_WAVEFRONT,
                                          cfg.T, cfg.B, prop.multi_processor_count, prop.shared_memory_per_block)
        assert rcq == rnn.RNN_OK
        harness.forward(model, io)                      # sizes the workspace
        assert rnn.rnn_model_set_profiling(model.handle, rnn.RNN_PROFILE_KERNELS) == rnn.RNN_OK
        harness.forward(model, io)
        torch.cuda.synchronize()
        rc, ms, n = rnn.rnn_model_profile_read(model.handle, rnn.RNN_KERNEL_RECURRENT)
        assert rc == rnn.RNN_OK
        passes = max(launch) + 1
        _say("    %s: layers -> launches %r, %d recurrent launches counted" % (cfg.name, launch, n))
        assert n == plan["launches"]                    # includes the passes over blocks of sequences, if any
        assert plan["launches"] % passes == 0 and sorted(set(launch)) == list(range(passes))
        assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
        model.close()


def test_matrix_rate_probe(gpu):
    """The measurement aid reports a plausible rate: a 32 x 32 x 16 bf16 matrix instruction takes 8 passes of 4
    clocks on its SIMD, and a wave that issues nothing else keeps the pipe full."""
    import torch
    harness, rnn, W = gpu
    rc, clk, ghz, tf = rnn.rnn_probe_matrix_rate(8, 2000, torch.cuda.current_stream())
    assert rc == rnn.RNN_OK
    _say("    8 compute units: %.2f clocks per instruction, %.3f GHz, %.1f TFLOP/s" % (clk, ghz, tf))
    assert 31.5 <= clk <= 36.0
    assert 0.5 <= ghz <= 3.0
    assert abs(tf - 8 * 4 * 32768 / clk * ghz * 1e9 / 1e12) <= 0.15 * tf     # events and stamps agree
    assert rnn.rnn_probe_matrix_rate(0, 10, None)[0] == rnn.RNN_EINVAL
    assert rnn.rnn_probe_matrix_rate(8, 0, None)[0] == rnn.RNN_EINVAL


def test_exchange_step_probe(gpu):
    """The measurement aid runs to the end (no wait gives up) and reports a step between the cost of one device-scope
    round trip and the step of the kernels built on the same exchange."""
    import torch
    harness, rnn, W = gpu
    for groups, wgs, words in ((1, 8, 64), (1, 64, 512), (4, 64, 512), (3, 5, 40)):
        rc, us, clk = rnn.rnn_probe_exchange_step(groups, wgs, words, 500, torch.cuda.current_stream())
        _say("    %d x %d workgroups, %d words: %.3f us per step, %.0f clocks" % (groups, wgs, words, us, clk))
        assert rc == rnn.RNN_OK
        assert 0.2 <= us <= 5.0
    bad = ((0, 8, 64, 10), (1, 8, 60, 10), (1, 7, 64, 10), (1, 1, 128, 10), (1, 8, 64, 0), (65, 1, 8, 10), (1, 8, 4096, 10))
    for g, w, n, st in bad:
        assert rnn.rnn_probe_exchange_step(g, w, n, st, None)[0] == rnn.RNN_EINVAL


def test_error_codes(gpu):
    import torch
    harness, rnn, W = gpu
    wl = _small_workload(W, SMALL[0])
    model = harness.DeviceModel(wl)
    io = harness.DeviceIO(wl)
    c = wl.cfg
    assert rnn.rnn_forward(model.handle, None, None, None, None, io.y, None, None, c.T, c.B, None) == rnn.RNN_EINVAL
    assert rnn.rnn_forward(model.handle, io.x, None, None, None, None, None, None, c.T, c.B, None) == rnn.RNN_EINVAL
    assert rnn.rnn_forward(model.handle, io.x, None, None, None, io.y, None, None, 0, c.B, None) == rnn.RNN_EINVAL
    assert rnn.rnn_forward(None, io.x, None, None, None, io.y, None, None, c.T, c.B, None) == rnn.RNN_EINVAL
    assert rnn.rnn_model_set_plan(model.handle, 99) == rnn.RNN_EINVAL
    assert rnn.rnn_model_device_bytes(model.handle) > 0
    with pytest.raises(rnn.RnnError):
        rnn.rnn_model_create(5, 1, 8, 8, 1, 0, [np.zeros(1, np.float32)] * 4, 0)
    with pytest.raises(rnn.RnnError):
        rnn.rnn_model_create(0, 1, 8, 6, 1, 1, [np.zeros(1, np.uint16)] * 4, 0)   # H % 8 != 0 for bf16
    model.close()


def test_length_validation(gpu):
    """Out-of-range lengths: clamped on the device by default, RNN_EINVAL under rnn_model_set_validation."""
    import torch
    harness, rnn, W = gpu
    wl = _small_workload(W, SMALL[0])
    model = harness.DeviceModel(wl)
    io = harness.DeviceIO(wl)
    c = wl.cfg
    good = io.lengths.clone()
    st = torch.cuda.current_stream()

    def call(lengths):
        return rnn.rnn_forward(model.handle, io.x, lengths, io.h0, io.c0, io.y, io.hT, io.cT, c.T, c.B, st)

    assert call(good) == rnn.RNN_OK
    torch.cuda.synchronize()
    ref = io.y.clone()
    assert rnn.rnn_model_set_validation(model.handle, 2) == rnn.RNN_EINVAL
    assert rnn.rnn_model_set_validation(model.handle, 1) == rnn.RNN_OK
    assert call(good) == rnn.RNN_OK
    for bad_value in (0, -3, c.T + 1):
        bad = good.clone()
        bad[1] = bad_value
        io.y.fill_(7.0)
        assert call(bad) == rnn.RNN_EINVAL
        torch.cuda.synchronize()
        assert float(io.y.float().min()) == 7.0          # nothing was enqueued
    assert call(None) == rnn.RNN_OK                       # no lengths: nothing to check
    assert rnn.rnn_model_set_validation(model.handle, 0) == rnn.RNN_OK
    bad = good.clone()
    bad[1] = c.T + 5                                      # clamped to T on the device
    assert call(bad) == rnn.RNN_OK
    assert call(good) == rnn.RNN_OK
    torch.cuda.synchronize()
    assert torch.equal(io.y, ref)
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    model.close()


@pytest.mark.parametrize("name", ["lstm_bf16_8layer_h256", "lstm_bf16_inside_sq", "lstm_bf16_b299"])
def test_launch_tag_wraps(gpu, name):
    """The 32-bit launch tag wraps after 2^32 launches: the launch that wraps clears the flag words and the
    tagged words and starts again from tag 1.  Forced here by setting the tag just below the wrap: the
    forwards across it give, bit for bit, what the first forward gave."""
    import torch
    harness, rnn, W = gpu
    wl = _small_workload(W, next(s for s in SMALL if s[0] == name))
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    torch.cuda.synchronize()
    ref = (io.y.clone(), io.hT.clone(), io.cT.clone())
    assert rnn.rnn_model_set_launch_tag(model.handle, 0xFFFFFFFF - 2) == rnn.RNN_OK
    for k in range(8):      # tags ...FFFE, ...FFFF, then the wrap, then 1, 2, ... (several launches per forward)
        io.y.fill_(7.0)
        harness.forward(model, io)
        torch.cuda.synchronize()
        assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK, k
        assert torch.equal(io.y, ref[0]) and torch.equal(io.hT, ref[1]) and torch.equal(io.cT, ref[2]), k
    model.close()


@pytest.mark.parametrize("cell", [0, 1], ids=["lstm", "gru"])
def test_onnx_gate_order(gpu, oracle, cell):
    """Weights whose gate row blocks come in the order of the ONNX operators (LSTM i,o,f,c; GRU z,r,h)
    give, after rnn_model_create_ordered, what the same weights in i,f,g,o / r,z,n order give: checked
    against the oracle (which only knows the latter order) and bit for bit against rnn_model_create."""
    import torch
    harness, rnn, W = gpu
    spec = ("order_test", cell, 2, 2, 40, 128, 7, 9, 1, True, True)
    wl = _small_workload(W, spec)
    c = wl.cfg
    H = c.H
    blocks = [0, 3, 1, 2] if cell == 0 else [1, 0, 2]      # ONNX block j holds our block blocks[j]
    permuted = []
    for w in wl.weights:
        rows = w.reshape(c.G, H, -1) if w.ndim == 2 else w.reshape(c.G, H)
        permuted.append(np.ascontiguousarray(rows[blocks].reshape(w.shape)))
    dev = [harness.to_device_storage(w, c.dtype) for w in permuted]
    handle = rnn.rnn_model_create_ordered(c.cell, c.L, c.I, c.H, c.D, c.dtype, dev, 1, rnn.RNN_ORDER_ONNX)
    ref_model = harness.DeviceModel(wl)
    io_ref, io = harness.DeviceIO(wl), harness.DeviceIO(wl)
    harness.forward(ref_model, io_ref)
    lengths = io.lengths
    assert rnn.rnn_forward(handle, io.x, lengths, io.h0, io.c0, io.y, io.hT, io.cT, c.T, c.B, None) == rnn.RNN_OK
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(handle) == rnn.RNN_OK
    assert torch.equal(io.y, io_ref.y) and torch.equal(io.hT, io_ref.hT)
    _check(harness, wl, io, oracle.forward_workload(wl, nthreads=8))
    with pytest.raises(rnn.RnnError):
        rnn.rnn_model_create_ordered(c.cell, c.L, c.I, c.H, c.D, c.dtype, dev, 1, 7)
    rnn.rnn_model_destroy(handle)
    ref_model.close()


OPT_SPECS = [
    (("lstm_opts_bf16", 0, 2, 2, 40, 128, 9, 21, 1, True, True), 0.5, True),           # tag-in-data kernel, both directions
    (("lstm_opts_f32", 0, 3, 1, 20, 64, 12, 5, 0, True, True), 0.4, True),
    (("lstm_peep_only", 0, 2, 1, 64, 128, 8, 6, 1, True, True), 0.0, True),
    (("lstm_clip_only", 0, 2, 1, 64, 128, 8, 6, 1, True, True), 0.3, False),
    (("gru_clip_bf16", 1, 2, 2, 40, 128, 9, 21, 1, True, True), 0.5, False),
    (("gru_clip_f32", 1, 2, 1, 12, 32, 8, 18, 0, True, True), 0.25, False),
    (("lstm_opts_padded_h72", 0, 2, 2, 24, 72, 6, 5, 1, True, True), 0.6, True),      # 72 -> 128 units: padded peephole weights
    (("lstm_opts_4layer_sq_h1024_b1", 0, 4, 1, 1024, 1024, 7, 1, 1, False, True), 0.15, True),   # the batch-1 latency shape
    (("lstm_opts_inside_sq", 0, 2, 1, 512, 512, 11, 300, 1, True, True), 0.5, True),  # inside-product kernel, two chains
    (("lstm_opts_b300", 0, 1, 1, 64, 512, 6, 300, 1, True, True), 0.5, True),         # flag-vector kernel
    (("gru_clip_b256_bidir", 1, 1, 2, 64, 128, 5, 256, 1, True, True), 0.4, False),   # flag-vector kernel, both directions
    (("lstm_opts_sidebyside_l3", 0, 3, 1, 512, 512, 5, 64, 1, True, True), 0.6, True),  # layers side by side
]


@pytest.mark.parametrize("plan", ["cellwise", "wavefront"])
@pytest.mark.parametrize("spec,clip,peep", OPT_SPECS, ids=lambda v: v[0] if isinstance(v, tuple) else None)
def test_peepholes_and_clipping(gpu, oracle, spec, clip, peep, plan):
    """The optional terms of the ONNX operators, under the cellwise plan and inside the persistent kernels:
    peephole weights and the clipping threshold of the gate arguments, against the oracle with the same terms;
    setting them is refused where they do not exist, and taking them away restores the plain cell bit for bit."""
    import torch
    harness, rnn, W = gpu
    wl = _small_workload(W, spec)
    c = wl.cfg
    if plan == "cellwise" and c.B * c.T > 2000:
        pytest.skip("large batch: the persistent kernels are the point of this shape")
    rng = np.random.default_rng(c.seed + 99)
    ps = [rng.uniform(-4, 4, (3, c.H)).astype(np.float32) for _ in range(c.L * c.D)] if peep else None
    if ps is not None and len(ps) > 1:
        ps[-1] = None                          # a missing entry = zeros
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_CELLWISE if plan == "cellwise" else rnn.RNN_PLAN_WAVEFRONT)
    io_plain, io = harness.DeviceIO(wl), harness.DeviceIO(wl)
    harness.forward(model, io_plain)
    torch.cuda.synchronize()
    if clip:
        assert rnn.rnn_model_set_clip(model.handle, clip) == rnn.RNN_OK
    if ps is not None:
        assert rnn.rnn_model_set_peepholes(model.handle, ps, 0) == rnn.RNN_OK
    harness.forward(model, io)
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    rows = None
    sub = wl
    if c.B > 64:                               # large batches: the oracle recomputes sampled sequences
        rows = np.unique(np.concatenate([np.arange(0, c.B, max(c.B // 20, 1)), [15, 16, 31, 32, c.B - 1]]))
        sub = wl.take_batch(rows)
    sub_ps = ps
    ref = oracle.forward_workload(sub, nthreads=8, peepholes=sub_ps, clip=clip)
    _check(harness, wl, io, ref, rows=rows)
    plain = oracle.forward_workload(sub, nthreads=8)
    moved = float(np.max(np.abs(ref[0] - plain[0])))
    assert moved > 3 * TOL[c.dtype]          # the terms were active: a kernel that ignored them would fail above
    if ps is not None:   # the same from device memory
        dev = [None if q is None else torch.from_numpy(q).cuda() for q in ps]
        torch.cuda.synchronize()
        assert rnn.rnn_model_set_peepholes(model.handle, dev, 1) == rnn.RNN_OK
        y1 = io.y.clone()
        harness.forward(model, io)
        torch.cuda.synchronize()
        assert torch.equal(y1, io.y)
    # back to the plain cell
    assert rnn.rnn_model_set_clip(model.handle, 0.0) == rnn.RNN_OK
    assert rnn.rnn_model_set_peepholes(model.handle, None, 0) == rnn.RNN_OK
    harness.forward(model, io)
    torch.cuda.synchronize()
    assert torch.equal(io.y, io_plain.y) and torch.equal(io.hT, io_plain.hT)
    # refusals
    assert rnn.rnn_model_set_clip(model.handle, -1.0) == rnn.RNN_EINVAL
    assert rnn.rnn_model_set_clip(model.handle, float("nan")) == rnn.RNN_EINVAL
    if c.cell == 1:
        assert rnn.rnn_model_set_peepholes(model.handle, [None] * (c.L * c.D), 0) == rnn.RNN_EUNSUPPORTED
    model.close()


@pytest.mark.parametrize("name,plan", [("lstm_bf16_3layer", "auto"), ("gru_bf16_bidir", "auto"),
                                       ("lstm_bf16_b299", "auto"), ("lstm_bf16_inside_sq", "auto"),
                                       ("lstm_f32_4layer", "auto"), ("gru_f32_bidir", "cellwise"),
                                       ("gru_bf16_padded_h200_bidir", "auto")])
def test_batch_first_layout(gpu, oracle, name, plan):
    """rnn_model_set_batch_first: x as [B, T, I] and y as [B, T, D*H] give, element for element, what the
    time-major call gives (same kernels on a re-laid-out copy), padded positions still +0.0 bits, the state
    tensors unchanged; and one case against the oracle directly."""
    import torch
    harness, rnn, W = gpu
    spec = [s for s in SMALL if s[0] == name][0]
    wl = _small_workload(W, spec)
    c = wl.cfg
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_CELLWISE if plan == "cellwise" else rnn.RNN_PLAN_AUTO)
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    torch.cuda.synchronize()
    assert rnn.rnn_model_set_batch_first(model.handle, 1) == rnn.RNN_OK
    x_bf = io.x.transpose(0, 1).contiguous()
    y_bf = torch.full((c.B, c.T, c.D * c.H), 7.0, dtype=io.y.dtype, device="cuda")
    hT, cT = torch.full_like(io.hT, 7.0), torch.full_like(io.cT, 7.0)
    for _ in range(2):
        assert rnn.rnn_forward(model.handle, x_bf, io.lengths, io.h0, io.c0, y_bf, hT, cT, c.T, c.B, None) == rnn.RNN_OK
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    assert torch.equal(y_bf.transpose(0, 1), io.y)
    assert torch.equal(hT, io.hT) and (c.cell == 1 or torch.equal(cT, io.cT))
    if name == "lstm_bf16_3layer":
        ref = oracle.forward_workload(wl, nthreads=8)
        err = float(np.max(np.abs(y_bf.float().cpu().numpy().astype(np.float64).transpose(1, 0, 2) - ref[0])))
        assert err <= TOL[c.dtype]
    assert rnn.rnn_model_set_batch_first(model.handle, 0) == rnn.RNN_OK
    assert rnn.rnn_model_set_batch_first(model.handle, 2) == rnn.RNN_EINVAL
    y2 = torch.full_like(io.y, 7.0)
    assert rnn.rnn_forward(model.handle, io.x, io.lengths, io.h0, io.c0, y2, hT, cT, c.T, c.B, None) == rnn.RNN_OK
    torch.cuda.synchronize()
    assert torch.equal(y2, io.y)
    model.close()


@pytest.mark.parametrize("spec", [("gru_rb_bf16", 1, 2, 2, 40, 128, 9, 21, 1, True, True),
                                  ("gru_rb_f32", 1, 2, 1, 24, 64, 7, 5, 0, True, True)], ids=lambda s: s[0])
def test_gru_reset_before_product(gpu, oracle, spec):
    """The GRU that applies the reset gate before the candidate's recurrent product (the oracle's
    variant 1, pinned by its own closed-form tests) runs under the cellwise plan."""
    harness, rnn, W = gpu
    wl = _small_workload(W, spec)
    model = harness.DeviceModel(wl)
    assert rnn.rnn_model_set_gru_reset_before(model.handle, 1) == rnn.RNN_OK
    assert rnn.rnn_model_set_plan(model.handle, rnn.RNN_PLAN_WAVEFRONT) == rnn.RNN_EUNSUPPORTED
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    ref = oracle.forward_workload(wl, nthreads=8, gru_variant=1)
    _check(harness, wl, io, ref)
    # the two variants really differ on this input, and switching back gives the default again
    other = oracle.forward_workload(wl, nthreads=8, gru_variant=0)
    assert float(np.max(np.abs(other[0] - ref[0]))) > 5e-2
    # together with a clipping threshold (r, z and the whole argument of n are limited)
    assert rnn.rnn_model_set_clip(model.handle, 0.4) == rnn.RNN_OK
    harness.forward(model, io)
    _check(harness, wl, io, oracle.forward_workload(wl, nthreads=8, gru_variant=1, clip=0.4))
    assert rnn.rnn_model_set_clip(model.handle, 0.0) == rnn.RNN_OK
    assert rnn.rnn_model_set_gru_reset_before(model.handle, 0) == rnn.RNN_OK
    harness.forward(model, io)
    _check(harness, wl, io, other)
    model.close()
    # an LSTM has no such variant
    lstm = harness.DeviceModel(_small_workload(W, SMALL[0]))
    assert rnn.rnn_model_set_gru_reset_before(lstm.handle, 1) == rnn.RNN_EUNSUPPORTED
    assert rnn.rnn_model_set_gru_reset_before(lstm.handle, 0) == rnn.RNN_OK
    lstm.close()


@pytest.mark.parametrize("name,plan", [("lstm_bf16_8layer_h256", "auto"),      # tag-in-data kernel
                                       ("gru_bf16_bidir", "auto"),               # tag-in-data kernel, two launches
                                       ("lstm_bf16_inside_sq", "auto"),          # inside-product kernel, one launch per layer
                                       ("lstm_bf16_sidebyside_l4", "auto"),      # inside-product kernel, layers side by side
                                       ("lstm_f32_fusedflag_l6_h32", "auto"),    # flag-vector kernel
                                       ("lstm_f32_4layer", "cellwise"),
                                       ("lstm_f32_padded_h100", "auto")])
def test_forward_recorded_into_a_graph(gpu, name, plan):
    """rnn_forward recorded into a HIP graph: every replay (on new inputs, with eager forwards and
    synchronisations between the replays) gives bit for bit what the eager call gives on the same inputs."""
    import torch
    harness, rnn, W = gpu
    spec = [s for s in SMALL if s[0] == name][0]
    wl = _small_workload(W, spec)
    c = wl.cfg
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_CELLWISE if plan == "cellwise" else rnn.RNN_PLAN_AUTO)
    io = harness.DeviceIO(wl)
    _say("\n  case %s: capture" % name)
    harness.forward(model, io)               # sizes the workspace; one-time set-up of the kernels
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        harness.forward(model, io)           # on the capturing stream: recorded, not run
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda").manual_seed(c.seed % (2 ** 31))
    for r in range(4):
        # new input values in the same buffers (replays use the recorded pointers)
        io.x.copy_(torch.randn(io.x.shape, generator=gen, device="cuda").to(io.x.dtype))
        if io.h0 is not None:
            io.h0.copy_(0.3 * torch.randn(io.h0.shape, generator=gen, device="cuda"))
        harness.forward(model, io)           # eager, same inputs
        torch.cuda.synchronize()
        want = (io.y.clone(), io.hT.clone(), io.cT.clone())
        for t in (io.y, io.hT, io.cT):
            t.fill_(7.0)
        _say("    replay %d" % r)
        graph.replay()
        if r == 2:
            graph.replay()                   # two replays back to back
        torch.cuda.synchronize()
        assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
        assert torch.equal(io.y, want[0]) and torch.equal(io.hT, want[1])
        assert c.cell == 1 or torch.equal(io.cT, want[2])
    del graph
    model.close()


def test_kernel_runs_a_schedule_of_the_cell_graph(gpu):
    """The persistent kernel's own clock stamps (one per cell, taken when the cell is published), read as
    finish times, form a valid schedule of the cell graph that the host-side scheduler builds: no cell
    finishes before its predecessors.  And the whole grid takes about as many step times as the list
    schedule with one processor per layer predicts (its depth L + T - 1), far from the L * T of one cell
    after another.  Model: the paper's Table 6 shape, 12 layers x 96 steps."""
    import torch
    from paper_2307_11339_amd import schedule
    harness, rnn, W = gpu
    cfg = W.paper_grid()[0]
    wl = W.make_workload(cfg)
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    assert rnn.rnn_model_set_profiling(model.handle, rnn.RNN_PROFILE_STEP_TICKS) == rnn.RNN_OK
    harness.forward(model, io)
    torch.cuda.synchronize()
    n_cells = cfg.L * cfg.D * cfg.T
    rc, ticks = rnn.rnn_model_read_step_ticks(model.handle, n_cells)
    assert rc == rnn.RNN_OK and ticks.min() > 0
    model.close()
    rc, off, idx = schedule.rnn_schedule_grid(cfg.L, cfg.T, cfg.D)
    assert rc == rnn.RNN_OK and off.size == n_cells + 1
    finish = ticks.astype(np.int64)
    for v in range(n_cells):
        for m in idx[off[v]:off[v + 1]]:
            assert finish[m] <= finish[v], "cell %d published before its predecessor %d" % (v, m)
    rc, order = schedule.rnn_schedule_order(off, idx, np.zeros(idx.size), np.ones(n_cells))
    assert rc == rnn.RNN_OK
    rc, _, _, depth = schedule.rnn_schedule_simulate(off, idx, order, cfg.L * cfg.D, np.ones(n_cells), np.zeros(idx.size))
    assert rc == rnn.RNN_OK and depth == cfg.L + cfg.T - 1
    step = float(np.median(np.diff(finish.reshape(cfg.L * cfg.D, cfg.T)[-1])))     # top layer, steady state
    span = float(finish.max() - finish.min())
    _say("    grid of %d cells: %.1f step times measured, %d predicted by the list schedule, %d one after another"
         % (n_cells, span / step, depth, n_cells))
    assert span <= 1.5 * depth * step


def test_workspace_follows_the_plan(gpu):
    """The workspace holds what the plan of the current shape touches; a call of another shape that gets
    another plan grows it, and going back gives the first result again, bit for bit."""
    import torch
    harness, rnn, W = gpu
    by_name = {s[0]: s for s in SMALL}
    wl = _small_workload(W, by_name["lstm_bf16_inside_sq"])      # batch 500: one layer per launch, product inside
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
    io = harness.DeviceIO(wl)
    c = wl.cfg
    assert rnn.rnn_model_reserve(model.handle, c.T, c.B) == rnn.RNN_OK
    bytes_large = rnn.rnn_model_device_bytes(model.handle)
    # no projection buffer (T*B*4H fp32) and no inter-layer output buffer were allocated for this plan
    assert bytes_large < c.T * c.B * 4 * c.H * 4
    harness.forward(model, io)
    torch.cuda.synchronize()
    y_first = io.y.clone()
    # the same model on 3 sequences runs both layers in one launch of the tag-in-data kernel
    small = wl.take_batch(np.arange(3))
    io_small = harness.DeviceIO(small)
    harness.forward(model, io_small)
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    assert rnn.rnn_model_device_bytes(model.handle) > bytes_large          # grew: projection, tagged sequences
    # the same sequences under another plan (another kernel, another summation order): equal within the bf16 tolerance
    assert float((io_small.y.float() - y_first[:, :3].float()).abs().max()) <= 2e-2
    harness.forward(model, io)
    torch.cuda.synchronize()
    assert torch.equal(io.y, y_first)
    model.close()


@pytest.mark.parametrize("kind", ["inside_product", "tagged", "cellwise"])
def test_workspace_keeps_only_live_layers(gpu, oracle, kind):
    """A deeper model needs no more workspace than a shallow one: the state sequences of two launches and two
    inter-layer output buffers are used alternately (only the layer being written and the one being read are
    live), whatever the number of layers.  Checked on the byte count and, for the deep model, against the oracle
    (re-used regions hold another layer's data when a launch starts)."""
    import torch
    harness, rnn, W = gpu
    shape = {"inside_product": dict(I=512, H=512, T=9, B=300), "tagged": dict(I=256, H=256, T=12, B=3),
             "cellwise": dict(I=64, H=128, T=6, B=5)}[kind]
    plan = rnn.RNN_PLAN_CELLWISE if kind == "cellwise" else rnn.RNN_PLAN_WAVEFRONT
    deep_layers = 40 if kind == "tagged" else 7        # tagged: 16 layers per launch, so 3 launches
    shallow_layers = 32 if kind == "tagged" else 2     # two launches already use both halves
    work = {}
    for L in (shallow_layers, deep_layers):
        cfg = W.Config("ws_%s_%d" % (kind, L), W.LSTM, L=L, D=1, dtype=W.BF16, seed=W.BASE_SEED + 60 + L, len_min=2, **shape)
        wl = W.make_workload(cfg, zero_pad_x=False)
        model = harness.DeviceModel(wl, plan=plan)
        weights = rnn.rnn_model_device_bytes(model.handle)
        assert rnn.rnn_model_reserve(model.handle, cfg.T, cfg.B) == rnn.RNN_OK
        work[L] = rnn.rnn_model_device_bytes(model.handle) - weights
        if L == deep_layers:
            io = harness.DeviceIO(wl)
            harness.forward(model, io)
            torch.cuda.synchronize()
            assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
            rows = np.unique(np.linspace(0, cfg.B - 1, 6).astype(int))
            _check(harness, wl, io, oracle.forward_workload(wl.take_batch(rows), nthreads=16), rows=rows)
        model.close()
    # what still grows with the depth: step clocks (8 bytes per layer and step) and the fp32 state of the cellwise plan
    slack = (deep_layers - shallow_layers) * (8 * shape["T"] + 3 * shape["B"] * shape["H"] * 4) + 4096
    assert work[deep_layers] <= work[shallow_layers] + slack, work


@pytest.mark.parametrize("name", ["gru_bf16_inside_t2", "lstm_f32_inside_b501", "lstm_bf16_b299", "lstm_bf16_inside_sq",
                                  "lstm_f32_fusedflag_h32", "gru_f32_fusedflag_h64", "gru_f32_bidir",
                                  "lstm_bf16_sidebyside_l4", "gru_bf16_sidebyside_l2"])
def test_first_call_on_used_memory_equals_later_calls(gpu, name):
    """The kernels exchange states through memory that every address of is written once per launch and
    read with cached loads.  That only works if what a reader's cache line holds besides the data it
    waited for is never needed later in the same launch: the blocked state sequence pads its rows so a
    line never holds sequences of two chains.  Without that, the first call on memory holding anything
    else (or a call after other inputs) read stale values for a few sequences.  Here: workspace memory
    is dirtied first, then the same inputs, other inputs, and the first inputs again must give the
    first call's bits."""
    import torch
    harness, rnn, W = gpu
    by_name = {s[0]: s for s in SMALL}
    junk = [torch.full((32 << 20,), 3.0e4, dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    torch.cuda.synchronize()
    del junk
    torch.cuda.empty_cache()          # hands the memory back to the runtime; the library allocates from it next
    wl = _small_workload(W, by_name[name])
    spec2 = list(by_name[name])
    spec2[0] = name + "_other"
    wl2 = _small_workload(W, tuple(spec2))
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
    io, io2 = harness.DeviceIO(wl), harness.DeviceIO(wl2)
    harness.forward(model, io)
    torch.cuda.synchronize()
    y0, h0 = io.y.clone(), io.hT.clone()
    for _ in range(2):
        harness.forward(model, io)
        torch.cuda.synchronize()
        assert torch.equal(io.y, y0) and torch.equal(io.hT, h0)
    harness.forward(model, io2)        # same weights, other inputs and initial states: leaves other values behind
    torch.cuda.synchronize()
    assert not torch.equal(io2.y, y0)
    harness.forward(model, io)
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    assert torch.equal(io.y, y0) and torch.equal(io.hT, h0)
    model.close()


def test_input_product_placement(gpu):
    """Which kernel performs W_ih x_t, per layer, as the library reports it."""
    harness, rnn, W = gpu
    by_name = {s[0]: s for s in SMALL}
    # first layer narrower than the hidden state: it projects, the layer above multiplies inside
    wl = _small_workload(W, by_name["lstm_bf16_inside"])
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
    c = wl.cfg
    assert [rnn.rnn_model_input_product_placement(model.handle, c.T, c.B, l) for l in range(c.L)] == \
        [(rnn.RNN_OK, 1), (rnn.RNN_OK, 0)]
    # the same model at batch 2 runs both layers in one launch: the first projects, the second is fused
    assert [rnn.rnn_model_input_product_placement(model.handle, c.T, 2, l)[1] for l in range(c.L)] == [1, 0]
    assert rnn.rnn_model_input_product_placement(model.handle, c.T, c.B, c.L)[0] == rnn.RNN_EINVAL
    assert rnn.rnn_model_input_product_placement(model.handle, 0, c.B, 0)[0] == rnn.RNN_EINVAL
    # x and y must be 16-byte aligned
    io = harness.DeviceIO(wl)
    import torch
    xv = io.x.view(-1)[1:]
    assert rnn.rnn_forward(model.handle, xv, io.lengths, io.h0, io.c0, io.y, io.hT, io.cT, 1, 1,
                           torch.cuda.current_stream()) == rnn.RNN_EINVAL
    model.close()
    # square first layer: no projection launch at all
    wl = _small_workload(W, by_name["lstm_bf16_inside_sq"])
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
    c = wl.cfg
    assert [rnn.rnn_model_input_product_placement(model.handle, c.T, c.B, l)[1] for l in range(c.L)] == [0, 0]
    assert rnn.rnn_model_set_plan(model.handle, rnn.RNN_PLAN_CELLWISE) == rnn.RNN_OK
    assert [rnn.rnn_model_input_product_placement(model.handle, c.T, c.B, l)[1] for l in range(c.L)] == [1, 1]
    model.close()
    # small batch, square first layer: the tag-in-data kernel's first layer reads the plain input
    wl = _small_workload(W, by_name["lstm_bf16_3layer_sq_h256"])
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
    c = wl.cfg
    assert [rnn.rnn_model_input_product_placement(model.handle, c.T, c.B, l)[1] for l in range(c.L)] == [0, 0, 0]
    model.close()


# ------------------------------------------------------------------ the five named workloads
def _run_named(gpu, oracle, name, plan, sample=None):
    harness, rnn, W = gpu
    wl = W.make_workload(W.CONFIGS[name])
    _say("\n  workload %s plan %d" % (name, plan))
    model = harness.DeviceModel(wl, plan=plan)
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    import torch
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    if sample is None:
        ref = oracle.forward_workload(wl, nthreads=16)
        _check(harness, wl, io, ref)
    else:
        rows = np.asarray(sample)
        ref = oracle.forward_workload(wl.take_batch(rows), nthreads=16)
        _check(harness, wl, io, ref, rows=rows)
    model.close()
    return io


@pytest.mark.parametrize("plan", [1, 2], ids=["cellwise", "wavefront"])
@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_named_full(gpu, oracle, name, plan):
    _run_named(gpu, oracle, name, plan)


@pytest.mark.parametrize("plan", [1, 2], ids=["cellwise", "wavefront"])
def test_C4_sampled_sequences(gpu, oracle, plan):
    """Full-size C4 on the GPU; the oracle recomputes 6 of the 64 sequences (sequences are
    independent), including the shortest and the longest."""
    harness, rnn, W = gpu
    wl = W.make_workload(W.CONFIGS["C4"])
    rows = sorted({int(np.argmin(wl.lengths)), int(np.argmax(wl.lengths)), 0, 17, 40, 63})
    _run_named(gpu, oracle, "C4", plan, sample=rows)


@pytest.mark.parametrize("index", list(range(13)))
def test_paper_grid_models(gpu, oracle, index):
    """Every model of the paper's own evaluation grid (Table 6: <layers, batch, io size, seq len>: the
    baseline <12, 8, 64, 96> and its twelve one-parameter variants), fp32, all layers in one launch."""
    harness, rnn, W = gpu
    cfg = W.paper_grid()[index]
    wl = W.make_workload(cfg)
    _say("\n  paper grid model %s" % cfg.name)
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_WAVEFRONT)
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    ref = oracle.forward_workload(wl, nthreads=8)
    _check(harness, wl, io, ref)
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    model.close()


def test_C5_sampled_sequences(gpu, oracle):
    """Full-size C5 (the throughput workload, in the launch configuration the benchmark times);
    the oracle recomputes 10 of the 256 sequences through all 8 layers and 512 steps: one in each of
    the eight 32-sequence chains of the launch, plus the last lane of the first 16-sequence tile, the
    first lane of the second and the last lane of the last."""
    _run_named(gpu, oracle, "C5", 0, sample=[0, 15, 16, 36, 72, 109, 145, 182, 218, 255])


def test_long_sequence_on_the_interleaved_chain_kernel(gpu, oracle):
    """1000 steps on the kernel that issues its matrix instructions by hand from the accumulation registers
    (two interleaved chains per workgroup, input product inside): a slip in the spacing of those instructions or
    in the step protocol that shows only now and then has 2000 chain steps per workgroup to show in (the variant
    of the throughput workload: 1024 units, part of W_ih in LDS), against
    the oracle on sampled sequences (first and last lane of a tile, both chains of a workgroup)."""
    import torch
    harness, rnn, W = gpu
    cfg = W.Config("long_T_interleaved", W.LSTM, L=1, D=1, I=1024, H=1024, T=1000, B=128, dtype=W.BF16,
                   seed=W.BASE_SEED + 41, len_min=800)
    prop = torch.cuda.get_device_properties(0)
    rc, plan, sep = rnn.rnn_plan_query(cfg.cell, cfg.L, cfg.I, cfg.H, cfg.D, cfg.dtype, rnn.RNN_PLAN_AUTO, cfg.T, cfg.B,
                                       prop.multi_processor_count, 160 * 1024)
    assert rc == rnn.RNN_OK and plan["chains"] == 2 and sep == [0], (plan, sep)
    wl = W.make_workload(cfg, zero_pad_x=False)
    model = harness.DeviceModel(wl)
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    rows = np.array([0, 15, 47, 64, 127])   # chains of 32 sequences: 0, 0, 1, 2, 3
    ref = oracle.forward_workload(wl.take_batch(rows), nthreads=16)
    _check(harness, wl, io, ref, rows=rows)
    model.close()


@pytest.mark.parametrize("name", ["C2", "C4", "C5"])
def test_one_sequence_through_a_named_model(gpu, oracle, name):
    """The batch-1 latency shapes the benchmark times: sequence 0 of C2, C4 and C5 run as a batch of its
    own (C5: 8 layers of 1024 units at batch 1 take two launches of 4 layers), every element compared."""
    harness, rnn, W = gpu
    wl = W.make_workload(W.CONFIGS[name]).take_batch([0])
    _say("\n  one sequence of %s" % name)
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_AUTO)
    io = harness.DeviceIO(wl)
    harness.forward(model, io)
    ref = oracle.forward_workload(wl, nthreads=16)
    _check(harness, wl, io, ref)
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
    model.close()
