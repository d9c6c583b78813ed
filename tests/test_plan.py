"""Host logic of the library: which execution plan it chooses for a model shape on a GPU with a given
number of compute units and LDS size (include/rnn.h, rnn_plan_query).  Runs without a GPU."""
import random

import pytest

from paper_2307_11339_amd import rnn, workloads as W

CUS, LDS = 256, 160 * 1024      # MI355X


def _query(c, plan=rnn.RNN_PLAN_AUTO, cus=CUS, lds=LDS, T=None, B=None):
    return rnn.rnn_plan_query(c.cell, c.L, c.I, c.H, c.D, c.dtype, plan, T or c.T, B or c.B, cus, lds)


def test_named_workloads():
    """The five named workloads on an MI355X: the plans the measurements in the design notes refer to."""
    expect = {
        # layers per launch, tile (16-row tiles, column tiles, chains), row blocks, column blocks, launches, projections
        "C1": (1, (1, 1, 1), 32, 1, 1, [0]),             # input half as wide as the layer: read by the x waves
        "C2": (2, (4, 1, 1), 32, 1, 1, [0, 0]),
        "C3": (4, (4, 1, 1), 64, 1, 1, [0, 0, 0, 0]),
        "C4": (1, (4, 1, 1), 32, 4, 2, [0, 0]),     # both directions; the upper layer reads [forward, backward] of the lower
        "C5": (1, (4, 2, 2), 64, 8, 8, [0] * 8),
    }
    for name, (lp, tile, nrb, ncb, launches, proj) in expect.items():
        rc, plan, sep = _query(W.CONFIGS[name])
        assert rc == rnn.RNN_OK, name
        assert plan["kind"] == rnn.RNN_PLAN_WAVEFRONT, name
        assert plan["layers_per_launch"] == lp, name
        assert (plan["row_tiles"], plan["col_tiles"], plan["chains"]) == tile, name
        assert (plan["row_blocks"], plan["col_blocks"], plan["launches"]) == (nrb, ncb, launches), name
        assert sep == proj, name


def test_medium_batch_layers_side_by_side():
    """64 sequences, 4 layers of 1024 units: one launch of 4 x 64 workgroups.  With inputs as wide as the layers
    every input product runs inside; with a narrower first layer that layer projects."""
    sq = W.Config("m", W.LSTM, L=4, D=1, I=1024, H=1024, T=128, B=64, dtype=W.BF16, seed=1)
    rc, plan, sep = _query(sq)
    assert rc == rnn.RNN_OK and plan["kind"] == rnn.RNN_PLAN_WAVEFRONT
    assert (plan["layers_per_launch"], plan["row_tiles"], plan["col_tiles"], plan["chains"]) == (4, 4, 2, 2)
    assert (plan["row_blocks"], plan["col_blocks"], plan["launches"]) == (64, 2, 1)
    assert sep == [0, 0, 0, 0]
    # a narrower first layer runs alone behind its projection, the three above it side by side
    rc, plan, sep = _query(sq.scaled(I=64))
    assert rc == rnn.RNN_OK and plan["layers_per_launch"] == 4 and plan["launches"] == 2 and sep == [1, 0, 0, 0]
    # without the LDS for the part of W_ih that does not fit the registers (64 KiB are needed beside the exchange
    # buffer) the layers still share a launch, the first one projects
    rc, plan, sep = _query(sq, lds=48 * 1024)
    assert rc == rnn.RNN_OK and plan["layers_per_launch"] == 4 and plan["launches"] == 1 and sep == [1, 0, 0, 0]


def test_cellwise_requested_or_forced():
    c = W.CONFIGS["C2"]
    rc, plan, sep = _query(c, plan=rnn.RNN_PLAN_CELLWISE)
    assert rc == rnn.RNN_OK and plan["kind"] == rnn.RNN_PLAN_CELLWISE
    assert sep == [1] * c.L and plan["launches"] == c.L
    # a width beyond every persistent kernel: AUTO falls back to cellwise, WAVEFRONT is refused
    odd = W.Config("odd", W.LSTM, L=2, D=1, I=24, H=4096, T=5, B=4, dtype=W.BF16, seed=1)
    rc, plan, _ = _query(odd)
    assert rc == rnn.RNN_OK and plan["kind"] == rnn.RNN_PLAN_CELLWISE
    assert _query(odd, plan=rnn.RNN_PLAN_WAVEFRONT)[0] == rnn.RNN_EUNSUPPORTED
    # a width between two compiled ones is padded up to the next: 72 units run as 128 (row blocks count padded units)
    rc, plan, _ = _query(odd.scaled(H=72))
    assert rc == rnn.RNN_OK and plan["kind"] == rnn.RNN_PLAN_WAVEFRONT
    assert plan["row_blocks"] * plan["row_tiles"] * 4 == 128


def test_fewer_compute_units_mean_more_launches():
    c = W.CONFIGS["C3"]
    rc, plan, sep = _query(c, cus=64, lds=64 * 1024)
    assert rc == rnn.RNN_OK and plan["kind"] == rnn.RNN_PLAN_WAVEFRONT
    assert plan["layers_per_launch"] == 1 and plan["launches"] == 4 and plan["row_blocks"] == 64
    assert sep == [0, 0, 0, 0]          # every launch's first layer reads its plain input itself
    # a GPU too small for one layer of this width
    rc, plan, _ = _query(c, cus=8, lds=64 * 1024)
    assert rc == rnn.RNN_OK and plan["kind"] == rnn.RNN_PLAN_CELLWISE


def test_inside_product_needs_lds_for_the_weights():
    """Large batch, one layer per launch: a quarter of the W_ih slice lives in LDS (32 KiB beside the 32 KiB
    exchange buffer); without that much LDS the layer projects."""
    c = W.CONFIGS["C5"]
    rc, plan, sep = _query(c, lds=48 * 1024)
    assert rc == rnn.RNN_OK and plan["kind"] == rnn.RNN_PLAN_WAVEFRONT
    assert sep == [1] * 8
    rc, plan, sep = _query(c, lds=64 * 1024)
    assert rc == rnn.RNN_OK and sep == [0] * 8


def test_widths_covered_by_the_persistent_kernels():
    """A wave's K quarter is a whole number of MFMA K blocks (32 values in bf16, 4 in fp32); which block counts are
    compiled decides between a persistent kernel and one cell at a time."""
    def kind(H, B, dtype=W.BF16, L=2, D=1, I=None):
        c = W.Config("w", W.LSTM, L=L, D=D, I=H if I is None else I, H=H, T=32, B=B, dtype=dtype, seed=1)
        rc, plan, _ = _query(c)
        assert rc == rnn.RNN_OK
        return plan["kind"]
    for H in (128, 256, 384, 512, 640, 768, 1024):          # small and large batches
        assert kind(H, 1) == rnn.RNN_PLAN_WAVEFRONT and kind(H, 300) == rnn.RNN_PLAN_WAVEFRONT, H
    for H in (1280, 1536, 2048):                            # tag-in-data kernel only: large batches in many passes
        assert kind(H, 1) == rnn.RNN_PLAN_WAVEFRONT and kind(H, 8) == rnn.RNN_PLAN_WAVEFRONT, H
        assert kind(H, 300) == rnn.RNN_PLAN_WAVEFRONT, H
    for H in (64, 192, 896, 1152, 1800):                    # padded up to 128, 256, 1024, 1280, 2048 units
        assert kind(H, 1) == rnn.RNN_PLAN_WAVEFRONT, H
    assert kind(2056, 1) == rnn.RNN_PLAN_CELLWISE           # beyond the widest compiled
    for H in (32, 64, 128, 256, 512):                       # fp32: multiples of 16 up to 512 units
        assert kind(H, 2, dtype=W.F32) == rnn.RNN_PLAN_WAVEFRONT, H
    assert kind(48, 2, dtype=W.F32) == rnn.RNN_PLAN_WAVEFRONT   # as 64
    assert kind(1024, 2, dtype=W.F32) == rnn.RNN_PLAN_CELLWISE


def test_batches_beyond_one_launch_run_in_passes():
    """1024 units: a launch holds 256 sequences (64 row blocks x 4 groups of 2 chains of 32).  A larger batch runs in
    passes of the largest block of sequences that has a plan; the figures describe one pass, the launch count all."""
    c = W.CONFIGS["C5"]
    rc, plan, sep = _query(c, B=1000)
    assert rc == rnn.RNN_OK and plan["kind"] == rnn.RNN_PLAN_WAVEFRONT
    assert (plan["row_tiles"], plan["col_tiles"], plan["chains"], plan["row_blocks"], plan["col_blocks"]) == (4, 2, 2, 64, 8)
    assert plan["launches"] == 8 * 4 and sep == [0] * 8          # 256 + 256 + 256 + 232 sequences
    rc, whole, _ = _query(c, B=256)
    assert whole["launches"] == 8 and whole["col_blocks"] == 8
    # 1536 units: 192 workgroups of 8 units hold two chains of 32 sequences
    wide = W.Config("wide", W.LSTM, L=1, D=1, I=1536, H=1536, T=8, B=40, dtype=W.BF16, seed=1)
    rc, plan, _ = _query(wide)
    assert rc == rnn.RNN_OK and plan["kind"] == rnn.RNN_PLAN_WAVEFRONT
    assert (plan["row_tiles"], plan["col_tiles"], plan["chains"]) == (2, 2, 2)
    assert (plan["row_blocks"], plan["col_blocks"], plan["launches"]) == (192, 2, 1)
    rc, plan, _ = _query(wide.scaled(B=200))
    assert (plan["row_blocks"], plan["col_blocks"], plan["launches"]) == (192, 2, 4)     # 64 + 64 + 64 + 8 sequences
    # with 16 sequences or fewer the tag-in-data kernel, one block
    rc, plan, _ = _query(wide.scaled(B=9))
    assert (plan["row_tiles"], plan["col_tiles"], plan["chains"], plan["row_blocks"], plan["launches"]) == (2, 1, 1, 192, 1)
    # 2048 units: no large-batch tile fits the registers; 256 workgroups of the tag-in-data kernel hold 16 sequences
    rc, plan, _ = _query(wide.scaled(H=2048, I=2048))
    assert (plan["row_tiles"], plan["col_tiles"], plan["chains"]) == (2, 1, 1)
    assert (plan["row_blocks"], plan["col_blocks"], plan["launches"]) == (256, 1, 3)
    # the cellwise plan is never split
    rc, plan, _ = _query(c, plan=rnn.RNN_PLAN_CELLWISE, B=1000)
    assert plan["kind"] == rnn.RNN_PLAN_CELLWISE and plan["launches"] == 8


def test_invariants_over_random_shapes():
    rng = random.Random(20230711)
    seen_kinds = set()
    for _ in range(400):
        dtype = rng.choice([W.F32, W.BF16])
        H = rng.choice([32, 64, 128, 256, 512, 1024]) if rng.random() < 0.8 else 8 * rng.randint(1, 40)
        c = W.Config("r", rng.choice([W.LSTM, W.GRU]), L=rng.randint(1, 16), D=rng.choice([1, 2]),
                     I=8 * rng.randint(1, 64), H=H, T=rng.randint(1, 300), B=rng.choice([1, 2, 8, 17, 64, 100, 256, 500]),
                     dtype=dtype, seed=1)
        cus = rng.choice([64, 128, 256])
        rc, plan, sep = _query(c, cus=cus)
        assert rc == rnn.RNN_OK
        seen_kinds.add(plan["kind"])
        assert len(sep) == c.L and set(sep) <= {0, 1}
        if plan["kind"] == rnn.RNN_PLAN_CELLWISE:
            assert sep == [1] * c.L
            continue
        lp, rt, ct, nch = plan["layers_per_launch"], plan["row_tiles"], plan["col_tiles"], plan["chains"]
        plain = -(-c.L // lp)                           # launches of lp layers each
        first_alone = 1 + -(-(c.L - 1) // lp)           # the first layer alone behind its projection, then lp each
        per_pass = [plain] + ([first_alone] if lp > 1 and c.D == 1 and c.I != c.H and sep[0] == 1 else [])
        held = plan["col_blocks"] * ct * 16             # sequences one pass holds
        if held >= c.B:
            assert plan["launches"] in per_pass
        else:                                           # a batch beyond one launch: passes over blocks of sequences
            assert any(plan["launches"] % k == 0 and plan["launches"] // k >= 2 and (plan["launches"] // k) * held >= c.B
                       for k in per_pass)
        assert c.D == 1 or lp == 1                      # bidirectional layers cannot share a launch
        assert plan["row_blocks"] * rt * 4 >= c.H       # 16 gate rows = 4 hidden units per tile (of the padded width)
        assert plan["row_blocks"] * rt * 4 <= max(2 * c.H, 128)
        assert plan["col_blocks"] % nch == 0
        # all workgroups of a launch are resident at once: at most one per compute unit
        assert lp * c.D * plan["row_blocks"] * (plan["col_blocks"] // nch) <= cus
        # only the first layer of a launch can need a projection launch
        assert all(sep[l] == 0 for l in range(c.L) if l % lp != 0)
    assert seen_kinds == {rnn.RNN_PLAN_CELLWISE, rnn.RNN_PLAN_WAVEFRONT}


def test_errors():
    c = W.CONFIGS["C1"]
    q = lambda **kw: rnn.rnn_plan_query(kw.get("cell", c.cell), kw.get("L", c.L), c.I, kw.get("H", c.H), kw.get("D", c.D),
                                        c.dtype, kw.get("plan", rnn.RNN_PLAN_AUTO), kw.get("T", c.T), kw.get("B", c.B),
                                        kw.get("cus", CUS), LDS)[0]
    assert q() == rnn.RNN_OK
    assert q(cell=7) == rnn.RNN_EINVAL
    assert q(L=0) == rnn.RNN_EINVAL
    assert q(D=3) == rnn.RNN_EINVAL
    assert q(T=0) == rnn.RNN_EINVAL
    assert q(B=0) == rnn.RNN_EINVAL
    assert q(cus=0) == rnn.RNN_EINVAL
    assert q(plan=9) == rnn.RNN_EINVAL
    assert q(H=30) == rnn.RNN_EUNSUPPORTED           # fp32 widths are multiples of 4


def _launches(c, plan=rnn.RNN_PLAN_AUTO, cus=CUS, lds=LDS, T=None, B=None):
    return rnn.rnn_plan_launches(c.cell, c.L, c.I, c.H, c.D, c.dtype, plan, T or c.T, B or c.B, cus, lds)


def _by_layer_numbers(L, D, LP, first_alone):
    """The split written out on layer numbers: launches of LP consecutive layers, after a first layer that runs alone
    when it needs a projection the others do not; groups of a launch in ascending (layer, direction)."""
    launch, group = [], []
    for l in range(L):
        if first_alone:
            r, l0 = (0, 0) if l == 0 else (1 + (l - 1) // LP, 1 + ((l - 1) // LP) * LP)
        else:
            r, l0 = l // LP, (l // LP) * LP
        launch.append(r)
        group += [(l - l0) * D + d for d in range(D)]
    return launch, group


def test_launch_split_comes_out_of_the_scheduler():
    """The launches of a forward pass are the passes of the scheduler's placement of the cell grid (topological
    sorting, then list scheduling with one (layer, direction) per processor and pass, as many processors as a launch
    has room for groups).  For the named workloads, the 13 models of the paper's grid and shapes whose first layer
    runs alone or whose layers do not divide evenly, that placement is the split one would write down on layer
    numbers."""
    cases = [(name, W.CONFIGS[name], None) for name in ("C1", "C2", "C3", "C4", "C5")]
    cases += [(c.name, c, None) for c in W.paper_grid()]
    sq = W.Config("m", W.LSTM, L=4, D=1, I=1024, H=1024, T=128, B=64, dtype=W.BF16, seed=1)
    cases += [("side_by_side", sq, False), ("first_alone", sq.scaled(I=64), True),
              ("first_alone_7", sq.scaled(I=64, L=7), True),
              ("uneven", W.Config("u", W.LSTM, L=7, D=1, I=256, H=256, T=40, B=8, dtype=W.BF16, seed=1), None),
              ("one_step", W.Config("t1", W.GRU, L=5, D=1, I=128, H=128, T=1, B=3, dtype=W.BF16, seed=1), None),
              ("two_directions", W.Config("bi", W.LSTM, L=3, D=2, I=96, H=128, T=33, B=16, dtype=W.BF16, seed=1), None)]
    seen_multi = seen_alone = 0
    for name, c, alone in cases:
        rc, plan, sep = _query(c)
        assert rc == rnn.RNN_OK, name
        rc, launch, group = _launches(c)
        assert rc == rnn.RNN_OK, name
        if plan["kind"] != rnn.RNN_PLAN_WAVEFRONT:
            assert launch == list(range(c.L)), name
            continue
        LP = plan["layers_per_launch"]
        if alone is None:                       # the first layer runs alone iff that explains the launch count
            alone = plan["launches"] == 1 + -(-(c.L - 1) // LP) and plan["launches"] != -(-c.L // LP)
        want_launch, want_group = _by_layer_numbers(c.L, c.D, LP, alone)
        assert launch == want_launch, (name, launch, want_launch)
        assert group == want_group, name
        assert max(launch) + 1 == plan["launches"], name
        seen_multi += LP > 1 and max(launch) > 0
        seen_alone += alone
    assert seen_multi >= 1 and seen_alone >= 2      # the cases do exercise several launches of several layers


def test_launch_split_query_errors():
    c = W.CONFIGS["C2"]
    assert rnn.rnn_plan_launches(c.cell, c.L, c.I, c.H, c.D, c.dtype, 99, c.T, c.B, CUS, LDS)[0] == rnn.RNN_EINVAL
    assert rnn.rnn_plan_launches(c.cell, c.L, c.I, c.H, c.D, c.dtype, rnn.RNN_PLAN_AUTO, 0, c.B, CUS, LDS)[0] == rnn.RNN_EINVAL
    rc, launch, _ = _launches(c, plan=rnn.RNN_PLAN_CELLWISE)
    assert rc == rnn.RNN_OK and launch == list(range(c.L))
