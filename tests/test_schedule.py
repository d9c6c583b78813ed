"""The library's host-side scheduling (include/rnn_schedule.h) against the reference in
oracle/schedule_oracle.py: integer results bit for bit, times exactly (same operations in the same
order on the same doubles).  No GPU needed: these entry points do no device work."""
import random

import numpy as np
import pytest

from oracle import schedule_oracle as S


@pytest.fixture(scope="module")
def sched():
    from paper_2307_11339_amd import _build, rnn, schedule
    import os
    if not os.path.exists(rnn.LIB_PATH):
        _build.build(force=True)
    return schedule, rnn


def _csr(pred):
    off = np.zeros(len(pred) + 1, dtype=np.int32)
    for v, p in enumerate(pred):
        off[v + 1] = off[v] + len(p)
    idx = np.array([m for p in pred for m in p], dtype=np.int32)
    return off, idx


def _flat(per_vertex):
    return np.array([c for row in per_vertex for c in row], dtype=np.float64)


@pytest.mark.parametrize("L,T,D", [(1, 1, 1), (1, 7, 1), (3, 5, 1), (4, 3, 2), (2, 9, 2), (8, 512, 1)])
def test_grid_graph(sched, L, T, D):
    schedule, rnn = sched
    n, pred = S.grid_dag(L, T, D)
    rc, off, idx = schedule.rnn_schedule_grid(L, T, D)
    assert rc == rnn.RNN_OK
    woff, widx = _csr(pred)
    assert np.array_equal(off, woff) and np.array_equal(idx, widx)


def test_grid_graph_errors(sched):
    schedule, rnn = sched
    assert schedule.rnn_schedule_grid(0, 4, 1)[0] == rnn.RNN_EINVAL
    assert schedule.rnn_schedule_grid(2, 4, 3)[0] == rnn.RNN_EINVAL
    assert schedule.rnn_schedule_grid(1 << 16, 1 << 15, 1)[0] == rnn.RNN_EUNSUPPORTED


def _random_case(rng, n_max):
    n = rng.randint(1, n_max)
    pred = [sorted(rng.sample(range(v), rng.randint(0, min(v, 3)))) for v in range(n)]
    comm = [[rng.choice([0.0, 0.5, 2.0, 0.1 * rng.randint(0, 40)]) for _ in p] for p in pred]
    ex = [rng.choice([0.25, 1.0, 3.0, 0.1 * rng.randint(1, 40)]) for _ in range(n)]
    return n, pred, comm, ex


def test_order_and_simulation_on_random_graphs(sched):
    schedule, rnn = sched
    rng = random.Random(2307)
    for trial in range(200):
        n, pred, comm, ex = _random_case(rng, 60)
        off, idx = _csr(pred)
        want = S.topological_order(n, pred, comm, ex)
        rc, order = schedule.rnn_schedule_order(off, idx, _flat(comm), ex)
        assert rc == rnn.RNN_OK and order.tolist() == want
        for P in (1, 2, 5):
            wp, wa, wl = S.simulate(n, pred, want, P, ex, comm)
            rc, proc, aft, lat = schedule.rnn_schedule_simulate(off, idx, order, P, ex, _flat(comm))
            assert rc == rnn.RNN_OK
            assert proc.tolist() == wp and aft.tolist() == wa and lat == wl


def test_resident_placement_on_random_graphs(sched):
    """The library's placement under the residency rule equals the reference vertex by vertex."""
    schedule, rnn = sched
    rng = random.Random(4111)
    for trial in range(200):
        n, pred, comm, ex = _random_case(rng, 60)
        off, idx = _csr(pred)
        order = S.topological_order(n, pred, comm, ex)
        kind = [rng.randint(0, 6) for _ in range(n)]
        for P in (1, 2, 5):
            wp, wr, wa, wl, wn = S.place_resident(n, pred, order, P, ex, comm, kind)
            rc, proc, rnd, aft, lat, npass = schedule.rnn_schedule_place_resident(off, idx, order, P, ex, _flat(comm), kind)
            assert rc == rnn.RNN_OK
            assert proc.tolist() == wp and rnd.tolist() == wr and aft.tolist() == wa and lat == wl and npass == wn
    # errors: an order that is not a permutation, one that is not topological, no processors
    off, idx = _csr([[], [0], [1]])
    ex, cm, kind = [1.0] * 3, [0.0, 0.0], [0, 1, 2]
    assert schedule.rnn_schedule_place_resident(off, idx, [0, 1, 1], 2, ex, cm, kind)[0] == rnn.RNN_EINVAL
    assert schedule.rnn_schedule_place_resident(off, idx, [0, 1, 2], 0, ex, cm, kind)[0] == rnn.RNN_EINVAL
    rc, proc, rnd, aft, lat, npass = schedule.rnn_schedule_place_resident(off, idx, [2, 1, 0], 3, ex, cm, kind)
    wp, wr, wa, wl, wn = S.place_resident(3, [[], [0], [1]], [2, 1, 0], 3, ex, [[], [0.0], [0.0]], kind)
    assert rc == rnn.RNN_OK and rnd.tolist() == wr and npass == wn     # out-of-order vertices simply wait a pass


@pytest.mark.parametrize("L,T,D,LP", [(12, 96, 1, 12), (8, 512, 1, 1), (8, 128, 1, 4), (2, 256, 2, 1), (8, 256, 1, 3)])
def test_resident_placement_on_the_grids_of_the_workloads(sched, L, T, D, LP):
    schedule, rnn = sched
    n, pred = S.grid_dag(L, T, D)
    off, idx = _csr(pred)
    comm = [[0.25] * len(p) for p in pred]
    ex = [1.0] * n
    order = S.topological_order(n, pred, comm, ex)
    kind = [v // T for v in range(n)]
    wp, wr, wa, wl, wn = S.place_resident(n, pred, order, LP * D, ex, comm, kind)
    rc, proc, rnd, aft, lat, npass = schedule.rnn_schedule_place_resident(off, idx, order, LP * D, ex, _flat(comm), kind)
    assert rc == rnn.RNN_OK
    assert proc.tolist() == wp and rnd.tolist() == wr and aft.tolist() == wa and lat == wl and npass == wn
    assert npass == -(-L // LP)


@pytest.mark.parametrize("L,T,D,P", [(12, 96, 1, 12), (8, 512, 1, 8), (2, 256, 2, 4), (4, 128, 1, 2)])
def test_the_grids_of_the_workloads(sched, L, T, D, P):
    """The shapes this repository runs (the paper's Table 6 model, the five named workloads): order and
    schedule equal the reference; with unit cell times and one processor per (layer, direction) the
    latency is the depth of the grid."""
    schedule, rnn = sched
    n, pred = S.grid_dag(L, T, D)
    off, idx = _csr(pred)
    comm = [[0.0] * len(p) for p in pred]
    ex = [1.0] * n
    want = S.topological_order(n, pred, comm, ex)
    rc, order = schedule.rnn_schedule_order(off, idx, _flat(comm), ex)
    assert rc == rnn.RNN_OK and order.tolist() == want
    wp, wa, wl = S.simulate(n, pred, want, P, ex, comm)
    rc, proc, aft, lat = schedule.rnn_schedule_simulate(off, idx, order, P, ex, _flat(comm))
    assert rc == rnn.RNN_OK and proc.tolist() == wp and aft.tolist() == wa and lat == wl
    if P >= L * D:
        assert lat == (L + T - 1 if D == 1 else max(L + T - 1, lat))
    # with communication dearer than execution the chains of the first layer are kept together
    comm2 = [[5.0] * len(p) for p in pred]
    want2 = S.topological_order(n, pred, comm2, ex)
    rc, order2 = schedule.rnn_schedule_order(off, idx, _flat(comm2), ex)
    assert rc == rnn.RNN_OK and order2.tolist() == want2
    assert want2[:T] == list(range(T))


def test_errors(sched):
    schedule, rnn = sched
    off, idx = _csr([[], [0], [1]])
    ex = [1.0, 1.0, 1.0]
    cm = [0.0, 0.0]
    # a cycle (1 <- 2, 2 <- 1)
    coff, cidx = _csr([[], [2], [1]])
    assert schedule.rnn_schedule_order(coff, cidx, cm, ex)[0] == rnn.RNN_EINVAL
    # predecessor index out of range, unsorted predecessors
    assert schedule.rnn_schedule_order(off, np.array([0, 7], dtype=np.int32), cm, ex)[0] == rnn.RNN_EINVAL
    uoff, uidx = _csr([[], [], [1, 0]])
    assert schedule.rnn_schedule_order(uoff, uidx, cm, ex)[0] == rnn.RNN_EINVAL
    # an order that is not topological, a repeated vertex, no processors
    assert schedule.rnn_schedule_simulate(off, idx, [1, 0, 2], 2, ex, cm)[0] == rnn.RNN_EINVAL
    assert schedule.rnn_schedule_simulate(off, idx, [0, 0, 2], 2, ex, cm)[0] == rnn.RNN_EINVAL
    assert schedule.rnn_schedule_simulate(off, idx, [0, 1, 2], 0, ex, cm)[0] == rnn.RNN_EINVAL
    rc, proc, aft, lat = schedule.rnn_schedule_simulate(off, idx, [0, 1, 2], 2, ex, cm)
    assert rc == rnn.RNN_OK and lat == 3.0 and proc.tolist() == [0, 0, 0]
