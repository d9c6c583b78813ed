#!/usr/bin/env python3
"""Benchmark of the stacked-RNN forward pass on one MI355X.

A "step" is one rnn_forward of the whole workload batch (projection of every layer plus the
persistent recurrent kernel over all time steps), inputs resident in HBM.  The headline workload
is C5 (8-layer LSTM, input = hidden = 1024, 512 steps, 256 sequences, bf16 with fp32 accumulation);
the other named workloads are reported in the "workloads" field of the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5] [--no-extra] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA (published)
PEAK_F32_TFLOPS = 157.3        # MI355X fp32 vector (published)
PEAK_HBM_GBPS = 8000.0         # MI355X HBM3E (published)
LDS_BYTES_PER_CLK_CU = 128.0   # LDS read bandwidth used for the per-step bound
CLOCK_GHZ = 2.4                # nominal engine clock; the device's own figure is printed beside it
MFMA_BF16_FLOP_PER_CLK_SIMD = 1024
TICK_HZ = 100e6                # device wall clock used by the step ticks


def roofline_constants():
    """The constants every roofline figure of this report uses, beside what the device itself reports."""
    import torch
    prop = torch.cuda.get_device_properties(0)
    cus = prop.multi_processor_count
    clock_ghz = getattr(prop, "clock_rate", 0) / 1e6 if getattr(prop, "clock_rate", 0) else None
    derived = cus * 4 * MFMA_BF16_FLOP_PER_CLK_SIMD * (clock_ghz or CLOCK_GHZ) / 1e3
    return {"device": prop.name, "compute_units": cus, "device_clock_ghz": clock_ghz,
            "lds_bytes_per_workgroup": getattr(prop, "shared_memory_per_block", None),
            "peak_bf16_tflops_used": PEAK_BF16_TFLOPS, "peak_f32_tflops_used": PEAK_F32_TFLOPS,
            "peak_hbm_gbps_used": PEAK_HBM_GBPS,
            "peak_bf16_tflops_from_device": round(derived, 1),   # CUs x 4 SIMDs x 1024 flop/clk x device clock
            "lds_bytes_per_clk_cu_used": LDS_BYTES_PER_CLK_CU, "clock_ghz_used": CLOCK_GHZ}


def matrix_rate_under_load(iterations: int = 20000):
    """Dense bf16 matrix instructions and nothing else (rnn_probe_matrix_rate): on 8 compute units the chip keeps its
    top clock, on all of them it does not; the second rate is what a contraction kernel can reach at most here."""
    import torch
    from paper_2307_11339_amd import rnn
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out = {}
    for name, n in (("few_compute_units", 8), ("all_compute_units", cus)):
        rc, clk, ghz, tf = rnn.rnn_probe_matrix_rate(n, iterations, torch.cuda.current_stream())
        if rc != 0:
            raise RuntimeError("rnn_probe_matrix_rate: status %d" % rc)
        out[name] = {"compute_units": n, "clocks_per_32x32x16_bf16": round(clk, 2), "shader_ghz": round(ghz, 3),
                     "tflops": round(tf, 1), "tflops_scaled_to_chip": round(tf * cus / n, 1)}
    return out


def exchange_floor(steps: int = 4000):
    """One step of the tagged all-gather the small-batch kernels are built on, without their arithmetic
    (rnn_probe_exchange_step), in the group shapes of the named small-batch workloads: 512 words are the h vector of
    1024 bf16 units, 256 words of 512 units."""
    import torch
    from paper_2307_11339_amd import rnn
    out = {}
    for name, (groups, wgs, words) in (("C1_shape_1x32_workgroups_512_words", (1, 32, 512)),
                                       ("C2_shape_2x32_workgroups_256_words", (2, 32, 256)),
                                       ("C3_shape_4x64_workgroups_512_words", (4, 64, 512)),
                                       ("one_group_64_workgroups_512_words", (1, 64, 512)),
                                       ("one_group_8_workgroups_512_words", (1, 8, 512))):
        rc, us, clk = rnn.rnn_probe_exchange_step(groups, wgs, words, steps, torch.cuda.current_stream())
        if rc != 0:
            raise RuntimeError("rnn_probe_exchange_step: status %d" % rc)
        out[name] = {"us_per_step": round(us, 3), "shader_clocks_per_step": round(clk, 1)}
    return out


def host_description():
    model = ""
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                model = ln.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return {"cpu_model": model, "nproc": os.cpu_count() or 1, "usable_cores": usable}


def log(msg: str) -> None:
    sys.stderr.write(msg + "\n")
    sys.stderr.flush()


def algorithmic_flops(cfg):
    """(projection flops per layer list, recurrent flops per layer) counting 2*M*K*N only."""
    rows = cfg.T * cfg.B
    proj = [2.0 * rows * cfg.layer_input(l) * cfg.D * cfg.G * cfg.H for l in range(cfg.L)]
    rec = [2.0 * rows * cfg.H * cfg.D * cfg.G * cfg.H for _ in range(cfg.L)]
    return proj, rec


def W_config(name):
    from paper_2307_11339_amd import workloads as W
    return W.CONFIGS[name]


def W_paper_grid():
    from paper_2307_11339_amd import workloads as W
    return W.paper_grid()


def time_workload(name, steps: int, warmup: int, per_call: int = 0, ticks: bool = False, plan=None, setup=None,
                  reference=None, kernel_events: bool = True):
    """name: one of the named workloads, or a workloads.Config.  plan: an rnn_plan (default: automatic).
    setup(model, io, wl): called before the workspace is sized, to set options of the model.
    reference: (rows, (y, hT, cT)) from the CPU oracle for some sequences of this workload: the device result of
    the last warm-up call is compared with it before anything is timed.
    kernel_events: bracket every kernel of the timed forwards with HIP events on the launch stream (the per-kernel
    averages of the report); without them the timed loop is the bare calls."""
    import numpy as np
    import torch
    from paper_2307_11339_amd import harness, rnn, workloads as W

    cfg = W.CONFIGS[name] if isinstance(name, str) else name
    name = cfg.name
    t0 = time.time()
    wl = W.make_workload(cfg)
    model = harness.DeviceModel(wl) if plan is None else harness.DeviceModel(wl, plan=plan)
    io = harness.DeviceIO(wl)
    if setup is not None:
        setup(model, io, wl)
    assert rnn.rnn_model_reserve(model.handle, cfg.T, cfg.B) == rnn.RNN_OK
    log("[bench] %s: inputs generated and uploaded in %.1f s" % (name, time.time() - t0))
    stream = torch.cuda.current_stream()
    for _ in range(max(warmup, 1 if reference is not None else 0)):
        harness.forward(model, io, stream)
    torch.cuda.synchronize()
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK

    parity = None
    if reference is not None:   # same inputs, same launch configuration as the timed calls, before they run
        rows, (ry, rh, rc) = reference
        y, hT, cT, ybits = harness.results(io)
        err = max(float(np.abs(y[:, rows] - ry).max()), float(np.abs(hT[:, rows] - rh).max()),
                  float(np.abs(cT[:, rows] - rc).max()) if rc is not None else 0.0)
        lengths = wl.lengths if wl.lengths is not None else np.full(cfg.B, cfg.T)
        padded_ok = all(bool(np.all(ybits[int(lengths[b]):, b] == 0)) for b in range(cfg.B))
        tol = 2e-2 if cfg.dtype == 1 else 1e-4
        parity = {"max_abs_err": err, "tolerance": tol, "ok": bool(err <= tol and padded_ok),
                  "padded_positions_all_zero_bits": padded_ok, "sequences_compared": [int(r) for r in rows],
                  "against": "CPU oracle (fp64), y / hT / cT of those sequences, all layers and steps"}
        log("[bench] %s: parity vs oracle on %d sequences: max-abs %.3e (tolerance %.0e)" % (name, len(rows), err, tol))

    # timed region: exactly `steps` forwards; kernel events on the launch stream
    rnn.rnn_model_set_profiling(model.handle, rnn.RNN_PROFILE_KERNELS if kernel_events else 0)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(steps):
        harness.forward(model, io, stream)
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    ms_per_step = (t_end - t_start) * 1e3 / steps
    _, proj_ms, proj_n = rnn.rnn_model_profile_read(model.handle, rnn.RNN_KERNEL_PROJECTION)
    _, rec_ms, rec_n = rnn.rnn_model_profile_read(model.handle, rnn.RNN_KERNEL_RECURRENT)
    rnn.rnn_model_set_profiling(model.handle, 0)
    assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK

    out = {
        "ms_per_step": ms_per_step,
        "seq_per_s": cfg.B / (ms_per_step * 1e-3),
        "projection": {"launches_per_step": proj_n / steps, "avg_ms": proj_ms / max(proj_n, 1)},
        "recurrent": {"launches_per_step": rec_n / steps, "avg_ms": rec_ms / max(rec_n, 1)},
        "device_bytes": rnn.rnn_model_device_bytes(model.handle),
        # per layer: 1 = the input product is a projection launch, 0 = it runs inside the recurrent kernel
        "projection_launched": [rnn.rnn_model_input_product_placement(model.handle, cfg.T, cfg.B, l)[1]
                                for l in range(cfg.L)],
        "parity": parity,
    }
    if per_call > 0:
        # per-call latency: every call bracketed by two events on the launch stream, calls back to back,
        # no kernel events inside, one wait at the end
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(per_call)]
        for a, b in ev:
            a.record(stream)
            harness.forward(model, io, stream)
            b.record(stream)
        torch.cuda.synchronize()
        lat = sorted(a.elapsed_time(b) for a, b in ev)
        out["p50_ms"] = statistics.median(lat)
        out["p90_ms"] = lat[int(0.9 * (len(lat) - 1))]
        out["calls_timed"] = per_call
    if ticks:
        rnn.rnn_model_set_profiling(model.handle, rnn.RNN_PROFILE_STEP_TICKS)
        harness.forward(model, io, stream)
        torch.cuda.synchronize()
        n = cfg.L * cfg.D * cfg.T
        rc, tk = rnn.rnn_model_read_step_ticks(model.handle, n)
        rnn.rnn_model_set_profiling(model.handle, 0)
        if rc == rnn.RNN_OK and tk.min() > 0:
            tk = tk.reshape(cfg.L * cfg.D, cfg.T).astype(np.int64)
            d = np.diff(tk[-1]) / TICK_HZ * 1e6           # top layer: steady-state wavefront
            out["step_us_p50"] = float(np.median(d))
            out["grid_us"] = float((tk.max() - tk.min()) / TICK_HZ * 1e6)
    model.close()
    return cfg, out


def time_cell_variants():
    """The cell variants and layouts beyond the plain time-major cell: what each costs.  Batch-first I/O on the
    bidirectional workload (every plan works on a re-laid-out copy: one more pass over x and y); peephole weights
    and a clipping threshold on the paper's own 12-layer model and on C3, under the cellwise plan and inside the
    persistent kernels, beside the plain cell."""
    import numpy as np
    import torch
    from paper_2307_11339_amd import rnn, workloads as W

    out = {}

    def batch_first(model, io, wl):
        c = wl.cfg
        assert rnn.rnn_model_set_batch_first(model.handle, 1) == rnn.RNN_OK
        io.x = io.x.transpose(0, 1).contiguous()
        io.y = torch.empty((c.B, c.T, c.D * c.H), dtype=io.y.dtype, device="cuda")

    _, r = time_workload("C4", steps=30, warmup=3, setup=batch_first)
    out["C4_batch_first_ms"] = round(r["ms_per_step"], 4)

    def options(model, io, wl):
        c = wl.cfg
        rng = np.random.default_rng(c.seed + 5)
        ps = [rng.uniform(-1, 1, (3, c.H)).astype(np.float32) for _ in range(c.L * c.D)]
        assert rnn.rnn_model_set_peepholes(model.handle, ps, 0) == rnn.RNN_OK
        assert rnn.rnn_model_set_clip(model.handle, 3.0) == rnn.RNN_OK

    base = W.paper_grid()[0]
    _, r = time_workload(base, steps=50, warmup=5)
    out["paper_base_ms"] = round(r["ms_per_step"], 4)
    _, r = time_workload(base, steps=5, warmup=1, plan=rnn.RNN_PLAN_CELLWISE)
    out["paper_base_cellwise_ms"] = round(r["ms_per_step"], 4)
    _, r = time_workload(base, steps=5, warmup=1, plan=rnn.RNN_PLAN_CELLWISE, setup=options)
    out["paper_base_cellwise_peepholes_clip_ms"] = round(r["ms_per_step"], 4)
    # the same terms inside the persistent kernels (a unit's peephole weights and the threshold sit in registers)
    _, r = time_workload(base, steps=50, warmup=5, setup=options)
    out["paper_base_peepholes_clip_ms"] = round(r["ms_per_step"], 4)
    _, r = time_workload("C3", steps=50, warmup=5)
    out["C3_ms"] = round(r["ms_per_step"], 4)
    _, r = time_workload("C3", steps=50, warmup=5, setup=options)
    out["C3_peepholes_clip_ms"] = round(r["ms_per_step"], 4)
    return out


def time_graph_replay(names=("C1", "C2", "C3"), reps: int = 200):
    """The forward pass recorded once into a HIP graph and replayed: ms per call back to back, beside the same
    loop of eager calls (the difference is launch overhead: one graph launch instead of 2-3 kernel launches)."""
    import torch
    from paper_2307_11339_amd import harness, rnn, workloads as W

    out = {}
    for name in names:
        wl = W.make_workload(W.CONFIGS[name])
        model = harness.DeviceModel(wl)
        io = harness.DeviceIO(wl)
        for _ in range(5):
            harness.forward(model, io)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
            harness.forward(model, io)
        torch.cuda.synchronize()

        def loop(fn):
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
            a = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - a) * 1e3 / reps

        eager = loop(lambda: harness.forward(model, io))
        replay = loop(graph.replay)
        assert rnn.rnn_model_check(model.handle) == rnn.RNN_OK
        out[name] = {"eager_ms": round(eager, 4), "graph_replay_ms": round(replay, 4)}
        del graph
        model.close()
    return out


def time_other_widths():
    """Shapes outside the named workloads that exercise the rest of the plan logic: widths that are not 128 times a
    power of two, 2048 units, a width that runs padded, a batch that runs in passes.  ms per forward."""
    from paper_2307_11339_amd import workloads as W

    shapes = {
        "lstm_4x768_T128_B1": dict(L=4, I=768, H=768, T=128, B=1),
        "lstm_2x768_T64_B300": dict(L=2, I=768, H=768, T=64, B=300),
        "lstm_2x2048_T128_B1": dict(L=2, I=2048, H=2048, T=128, B=1),
        "lstm_2x1536_T128_B8": dict(L=2, I=1536, H=1536, T=128, B=8),
        "lstm_2x200_T128_B8_padded_to_256": dict(L=2, I=200, H=200, T=128, B=8),
        "lstm_2x1024_T64_B300_two_passes": dict(L=2, I=1024, H=1024, T=64, B=300),
        "lstm_2x512_T128_B512": dict(L=2, I=512, H=512, T=128, B=512),
    }
    out = {}
    for i, (name, kw) in enumerate(shapes.items()):
        c = W.Config(name, W.LSTM, D=1, dtype=W.BF16, seed=W.BASE_SEED + 300 + i, **kw)
        _, r = time_workload(c, steps=10, warmup=2)
        out[name] = round(r["ms_per_step"], 4)
    return out


def time_projection_gemm(name: str, reps: int = 30, warm: int = 30):
    """The batched input projection X W_ih^T of one layer of the workload over all time steps, as a launch of its
    own (rnn_input_projection).  No named workload needs it any more (their input products run inside the
    recurrent kernels), so it is measured here on its own: it serves every layer whose input is not H/2, H or 2H
    wide, and the cellwise plan."""
    import torch
    from paper_2307_11339_amd import harness, rnn, workloads as W

    cfg = W.CONFIGS[name]
    wl = W.make_workload(cfg.scaled(L=1, T=1, B=1, len_min=None, h0_std=0.0))   # one layer of weights; activations are made here
    model = harness.DeviceModel(wl, plan=rnn.RNN_PLAN_CELLWISE)
    rows, K, N = cfg.T * cfg.B, cfg.I, cfg.D * 4 * cfg.H
    tdt = torch.bfloat16 if cfg.dtype == 1 else torch.float32
    a = torch.randn(rows, K, device="cuda", dtype=torch.float32).to(tdt)
    gx = torch.empty(rows, N, device="cuda", dtype=torch.float32)
    st = torch.cuda.current_stream()
    for _ in range(warm):      # a few launches are not enough: the first tens of milliseconds run measurably slower
        rnn.rnn_input_projection(model.handle, 0, a, gx, rows, st)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(reps):
        rnn.rnn_input_projection(model.handle, 0, a, gx, rows, st)
    e1.record(st)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    model.close()
    flops = 2.0 * rows * K * N
    peak = PEAK_BF16_TFLOPS if cfg.dtype == 1 else PEAK_F32_TFLOPS
    tf = flops / (ms * 1e-3) / 1e12
    return {"shape": {"M": rows, "K": K, "N": N}, "ms": round(ms, 4), "tflops": round(tf, 2),
            "frac_of_mfma_peak": round(tf / peak, 4),
            "output_bytes": rows * N * 4, "output_gbps": round(rows * N * 4 / (ms * 1e-3) / 1e9, 1)}


def cpu_baseline(name: str, n_seq: int):
    """The oracle as it stands, timed on the host cores for a bounded sample of the workload.  Returns the report
    entry and (rows, (y, hT, cT)), the oracle's results for those sequences, for the parity check of the same run."""
    import numpy as np
    from oracle import rnn_oracle
    from paper_2307_11339_amd import workloads as W

    cfg = W.CONFIGS[name]
    wl = W.make_workload(cfg)
    # one sequence in each block of B / n_seq consecutive sequences (for C5: one per 32-sequence chain of the launch)
    rows = np.unique(np.round(np.linspace(0, cfg.B - 1, num=min(n_seq, cfg.B))).astype(int))
    sub = wl.take_batch(rows)
    host = host_description()
    threads = max(1, min(16, host["usable_cores"]))
    rnn_oracle.build()
    t0 = time.perf_counter()
    ref = rnn_oracle.forward_workload(sub, nthreads=threads)
    dt = time.perf_counter() - t0
    # the same code on one thread, on one sequence cut to a few steps when the whole one would take too long
    steps1 = cfg.T
    per_step_flops = sum(2.0 * cfg.G * cfg.H * (cfg.layer_input(l) + cfg.H) * cfg.D for l in range(cfg.L))
    while steps1 > 8 and steps1 * per_step_flops > 12e9:     # about 10 s of scalar fp64
        steps1 //= 2
    one = wl.take_batch(rows[:1])
    one.x = np.ascontiguousarray(one.x[:steps1])
    one.cfg = one.cfg.scaled(T=steps1)
    if one.lengths is not None:
        one.lengths = np.minimum(one.lengths, steps1).astype(np.int32)
    t1 = time.perf_counter()
    rnn_oracle.forward_workload(one, nthreads=1)
    dt1 = time.perf_counter() - t1
    entry = {"value": len(rows) / dt, "unit": "sequences/s", "cores": threads, "kind": "oracle",
             "sample": "%d of the %d sequences of %s through all %d layers and %d steps, fp64, %.1f s"
                       % (len(rows), cfg.B, name, cfg.L, cfg.T, dt),
             "single_thread": {"value": (steps1 / cfg.T) / dt1 if dt1 > 0 else None, "unit": "sequences/s", "cores": 1,
                               "sample": "1 sequence, all %d layers, %d of its %d steps, %.1f s (scaled to whole sequences)"
                                         % (cfg.L, steps1, cfg.T, dt1)},
             "host": host}
    return entry, (rows, ref)


def recorded_traffic(workload: str, kernel_class: str):
    """HBM bytes per launch of the dominant kernel from the committed counter runs (profiles/), or
    None when there is no record for this workload and kernel or the kernel source has changed since."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "traffic_%s_%s.txt" % (workload, kernel_class))
    try:
        rec = json.load(open(path))
        digest = hashlib.sha256(open(os.path.join(ROOT, rec["source"]), "rb").read()).hexdigest()
        return rec["hbm_bytes_per_launch"] if digest == rec["source_sha256"] else None
    except (OSError, KeyError, ValueError):
        return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C5")
    ap.add_argument("--no-extra", action="store_true", help="skip the other named workloads")
    ap.add_argument("--projection-gemm", action="store_true",
                    help="time only the stand-alone input projection of one layer of the workload and exit")
    ap.add_argument("--matrix-rate", action="store_true",
                    help="only measure the dense matrix-instruction rate and shader clock under load")
    ap.add_argument("--exchange-floor", action="store_true",
                    help="only measure a step of the small-batch kernels' exchange without their arithmetic")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="only run a plain device copy of MIB mebibytes five times (reference reading "
                         "for the HBM byte counters of a profiler) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this library runs on one GPU; --gpus %d is not supported "
                         "(sequences are independent: splitting the batch across GPUs needs no kernel change)\n" % args.gpus)
        return 2

    import torch
    from paper_2307_11339_amd import rnn
    rnn.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.projection_gemm:
        print(json.dumps({"projection_gemm": time_projection_gemm(args.workload)}))
        return 0
    if args.exchange_floor:
        print(json.dumps({"exchange_floor": exchange_floor()}))
        return 0
    if args.matrix_rate:
        print(json.dumps({"matrix_rate_under_load": matrix_rate_under_load()}))
        return 0
    if args.copy_calibration > 0:
        n = args.copy_calibration << 20
        src = torch.full((n,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": n, "copies": 5}))
        return 0

    # The oracle goes first: its results for a sample of the sequences are both the CPU baseline (timed) and the
    # reference the device result is compared with before anything is timed.
    cpu_entry, reference = (None, None) if args.no_cpu else cpu_baseline(args.workload, n_seq=8)
    cfg, main_res = time_workload(args.workload, args.steps, args.warmup, reference=reference)
    if main_res["parity"] is not None and not main_res["parity"]["ok"]:
        log("[bench] PARITY FAILED: %r" % (main_res["parity"],))
    proj_flops, rec_flops = algorithmic_flops(cfg)
    # dominant kernel = the class with the larger share of the step
    proj_total = main_res["projection"]["avg_ms"] * main_res["projection"]["launches_per_step"]
    rec_total = main_res["recurrent"]["avg_ms"] * main_res["recurrent"]["launches_per_step"]
    bf16 = cfg.dtype == 1
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_TFLOPS

    def tflops(flops_per_step, kern):
        n = max(kern["launches_per_step"], 1e-9)
        return (flops_per_step / n) / (kern["avg_ms"] * 1e-3) / 1e12 if kern["avg_ms"] > 0 else 0.0

    # an input product that runs inside the recurrent kernel is that kernel's work
    placed = main_res["projection_launched"]
    proj_sep = sum(f for f, sep in zip(proj_flops, placed) if sep == 1)
    proj_in = sum(f for f, sep in zip(proj_flops, placed) if sep != 1)
    proj_tf = tflops(proj_sep, main_res["projection"])
    rec_tf = tflops(sum(rec_flops) + proj_in, main_res["recurrent"])
    dominant = "recurrent" if rec_total >= proj_total else "projection"
    ach = rec_tf if dominant == "recurrent" else proj_tf
    traffic = recorded_traffic(cfg.name, dominant)
    roofline = {"bound": "mfma", "achieved": round(ach, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(ach / peak, 4), "traffic": traffic, "kernel": dominant,
                "avg_ms": round(main_res[dominant]["avg_ms"], 4)}
    # streamed activations of the dominant kernel: HBM bytes per launch (counters, when on record for this kernel
    # source) and algorithmic bytes per launch (x or state in, state out, output, weights once), over its duration
    if dominant == "recurrent" and main_res["recurrent"]["avg_ms"] > 0:
        n_launch = max(main_res["recurrent"]["launches_per_step"], 1.0)
        es = 2 if bf16 else 4
        rows = cfg.T * cfg.B
        # per layer: its input read, its state sequence written and read back by the next step's products
        alg = (sum(rows * cfg.layer_input(l) * es + 2 * rows * cfg.D * cfg.H * es for l in range(cfg.L)) +
               rows * cfg.D * cfg.H * es +
               sum(cfg.D * cfg.G * cfg.H * (cfg.layer_input(l) + cfg.H) * es for l in range(cfg.L))) / n_launch
        sec = main_res["recurrent"]["avg_ms"] * 1e-3
        roofline["hbm"] = {"algorithmic_bytes_per_launch": int(alg), "algorithmic_gbps": round(alg / sec / 1e9, 1),
                           "measured_gbps": round(traffic / sec / 1e9, 1) if traffic else None,
                           "peak_gbps": PEAK_HBM_GBPS,
                           "frac_of_peak": round((traffic or alg) / sec / 1e9 / PEAK_HBM_GBPS, 4)}

    line = {
        "metric": "RNN forward sequences/sec",
        "value": round(main_res["seq_per_s"], 2),
        "unit": "sequences/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(main_res["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: %d-layer %s %s, input %d, hidden %d, seq len %d, batch %d"
                               % (cfg.name, cfg.L, "bidirectional" if cfg.D == 2 else "unidirectional",
                                  "LSTM" if cfg.cell == 0 else "GRU", cfg.I, cfg.H, cfg.T, cfg.B)},
        "roofline": roofline,
        "kernels": {
            "projection": {"avg_ms": round(main_res["projection"]["avg_ms"], 4),
                           "launches_per_step": main_res["projection"]["launches_per_step"],
                           "tflops": round(proj_tf, 2), "frac_of_mfma_peak": round(proj_tf / peak, 4)},
            "recurrent": {"avg_ms": round(main_res["recurrent"]["avg_ms"], 4),
                          "launches_per_step": main_res["recurrent"]["launches_per_step"],
                          "tflops": round(rec_tf, 2), "frac_of_mfma_peak": round(rec_tf / peak, 4)},
        },
        "device_bytes": main_res["device_bytes"],
        "input_product_in_recurrent_kernel": [l for l, sep in enumerate(placed) if sep != 1],
        "parity": main_res["parity"],
        "roofline_constants": roofline_constants(),
    }

    if not args.no_extra:
        extra = {}
        for name in ("C1", "C2", "C3", "C4"):
            if name == args.workload:
                continue
            c, r = time_workload(name, steps=100, warmup=10, per_call=100, ticks=True)
            e = {"seq_per_s": round(r["seq_per_s"], 1), "ms_per_call": round(r["ms_per_step"], 4),
                 "p50_ms": round(r["p50_ms"], 4), "p90_ms": round(r["p90_ms"], 4), "calls_timed": r["calls_timed"],
                 "recurrent_avg_ms": round(r["recurrent"]["avg_ms"], 4),
                 "projection_avg_ms": round(r["projection"]["avg_ms"], 4)}
            if "step_us_p50" in r:
                e["step_us_p50"] = round(r["step_us_p50"], 3)
                e["grid_us"] = round(r["grid_us"], 1)
            if name == "C3":
                # W_hh slice of one workgroup (64 gate rows x 1024 x 2 B) read once per step from LDS
                bound_us = (64 * 1024 * 2) / (LDS_BYTES_PER_CLK_CU * CLOCK_GHZ * 1e9) * 1e6
                e["lds_bound_us_per_step"] = round(bound_us, 3)
                if "step_us_p50" in e:
                    e["step_over_lds_bound"] = round(e["step_us_p50"] / bound_us, 2)
            extra[name] = e
        line["workloads"] = extra

    if not args.no_extra:
        # latency of a single sequence through the shapes that are named with a batch (C1 and C3 have batch 1 as given)
        b1 = {}
        for name in ("C2", "C4", "C5"):
            c1 = W_config(name).scaled(name=name + "/batch1", B=1)
            _, r = time_workload(c1, steps=20, warmup=10, per_call=100)
            b1[name] = {"p50_ms": round(r["p50_ms"], 4), "p90_ms": round(r["p90_ms"], 4),
                        "ms_per_call": round(r["ms_per_step"], 4)}
        line["batch1_latency"] = b1

    if not args.no_extra:
        # the paper's own model grid (Table 6): <layers, batch, io size, seq len>, fp32 LSTM
        grid = {}
        for c in W_paper_grid():
            _, r = time_workload(c, steps=30, warmup=10, per_call=100)
            # latency and device memory (weights + workspace), the two quantities of the paper's Table 6
            grid[c.name] = {"p50_ms": round(r["p50_ms"], 4), "ms_per_call": round(r["ms_per_step"], 4),
                            "device_mb": round(r["device_bytes"] / 1e6, 3)}
        line["paper_grid"] = grid

    if not args.no_extra:
        line["projection_gemm"] = time_projection_gemm(args.workload)
        line["matrix_rate_under_load"] = matrix_rate_under_load()
        line["exchange_floor"] = exchange_floor()
        sustained = line["matrix_rate_under_load"]["all_compute_units"]["tflops"]
        if bf16 and sustained > 0:
            # the same achieved rates against what the chip sustains on matrix instructions alone (its clock drops
            # under that load); the contract figure above stays against the published peak
            line["roofline"]["frac_of_sustained_matrix_rate"] = round(line["roofline"]["achieved"] / sustained, 4)
            line["projection_gemm"]["frac_of_sustained_matrix_rate"] = round(line["projection_gemm"]["tflops"] / sustained, 4)
        line["cell_variants"] = time_cell_variants()
        line["graph_replay"] = time_graph_replay()
        line["other_widths"] = time_other_widths()

    if cpu_entry is not None:
        line["cpu_baseline"] = cpu_entry

    print(json.dumps(line))
    sys.stdout.flush()
    return 0


if __name__ == "__main__":
    sys.exit(main())
