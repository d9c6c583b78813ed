"""Pins of the scheduling reference (oracle/schedule_oracle.py) against what the paper's definitions and
plain graph theory fix: closed forms on the cell grid, invariants of any valid schedule, brute force on
tiny graphs.  CPU only."""
import itertools
import random

import pytest

from oracle import schedule_oracle as S


def _zeros_like(pred, value=0.0):
    return [[value] * len(p) for p in pred]


def _is_topological(n, pred, order):
    pos = {v: i for i, v in enumerate(order)}
    return sorted(order) == list(range(n)) and all(pos[m] < pos[v] for v in range(n) for m in pred[v])


@pytest.mark.parametrize("L,T,D", [(1, 1, 1), (3, 5, 1), (4, 3, 2), (2, 7, 2)])
def test_grid_dag_structure(L, T, D):
    """Section 2.2, unfolded RNN: cell (l, t) depends on (l, t-1) and on (l-1, t); with two directions the
    layer above needs both directions of the layer below at the same time."""
    n, pred = S.grid_dag(L, T, D)
    assert n == L * D * T
    n_edges = sum(len(p) for p in pred)
    assert n_edges == L * D * (T - 1) + (L - 1) * D * T * D
    for l in range(L):
        for d in range(D):
            for s in range(T):
                v = S.vertex_id(L, T, D, l, d, s)
                want = set()
                if s > 0:
                    want.add(S.vertex_id(L, T, D, l, d, s - 1))
                if l > 0:
                    t = s if d == 0 else T - 1 - s
                    want.add(S.vertex_id(L, T, D, l - 1, 0, t))
                    if D == 2:
                        want.add(S.vertex_id(L, T, D, l - 1, 1, T - 1 - t))
                assert set(pred[v]) == want


def test_breadth_first_order_on_the_grid_is_the_wavefront():
    """Without merges (communication never exceeds execution) the order is breadth first, and on a
    unidirectional grid breadth-first levels are the anti-diagonals l + t: the level never decreases."""
    L, T = 4, 6
    n, pred = S.grid_dag(L, T, 1)
    order = S.topological_order(n, pred, _zeros_like(pred), [1.0] * n)
    assert _is_topological(n, pred, order)
    levels = [(v // T) + (v % T) for v in order]
    assert levels == sorted(levels)
    assert order[0] == 0 and order[-1] == n - 1


def test_merge_rule_keeps_a_chain_together():
    """Two independent chains a0->a1->a2 and b0->b1->b2: breadth first alternates between them; when
    communication exceeds execution every child (one predecessor) follows its parent at once."""
    pred = [[], [0], [1], [], [3], [4]]
    bfs = S.topological_order(6, pred, _zeros_like(pred, 0.5), [1.0] * 6)
    assert bfs == [0, 3, 1, 4, 2, 5]
    dfs = S.topological_order(6, pred, _zeros_like(pred, 2.0), [1.0] * 6)
    assert dfs == [0, 1, 2, 3, 4, 5]
    # a child with two predecessors is never merged, whatever the communication time
    pred = [[], [], [0, 1], [2]]
    order = S.topological_order(4, pred, _zeros_like(pred, 9.0), [1.0] * 4)
    assert order == [0, 1, 2, 3]


def test_order_is_topological_on_random_graphs():
    rng = random.Random(7)
    for trial in range(50):
        n = rng.randint(1, 40)
        pred = [sorted(rng.sample(range(v), rng.randint(0, min(v, 3)))) for v in range(n)]
        comm = [[rng.choice([0.0, 0.5, 2.0]) for _ in p] for p in pred]
        avg = [rng.choice([0.25, 1.0, 3.0]) for _ in range(n)]
        order = S.topological_order(n, pred, comm, avg)
        assert _is_topological(n, pred, order)


def test_cycle_is_reported():
    with pytest.raises(ValueError):
        S.topological_order(3, [[], [2], [1]], [[], [0.0], [0.0]], [1.0] * 3)


@pytest.mark.parametrize("L,T", [(1, 9), (4, 6), (8, 8), (12, 96)])
def test_latency_closed_forms_on_the_grid(L, T):
    """Unit execution time, free communication: one processor needs L*T (the one-cell-at-a-time regime
    of Section 2.2's figure caption), min(L, T) or more processors need the critical path L + T - 1."""
    n, pred = S.grid_dag(L, T, 1)
    order = S.topological_order(n, pred, _zeros_like(pred), [1.0] * n)
    comm = _zeros_like(pred)
    _, aft, lat1 = S.simulate(n, pred, order, 1, [1.0] * n, comm)
    assert lat1 == L * T and sorted(aft) == [float(i) for i in range(1, n + 1)]
    for P in (min(L, T), min(L, T) + 3):
        proc, aft, lat = S.simulate(n, pred, order, P, [1.0] * n, comm)
        assert lat == L + T - 1
        for v in range(n):  # every cell finishes exactly at its depth
            assert aft[v] == (v // T) + (v % T) + 1
    # in between: never better than work / P nor than the critical path, never worse than one processor
    for P in range(1, min(L, T) + 1):
        _, _, lat = S.simulate(n, pred, order, P, [1.0] * n, comm)
        assert max(L + T - 1, -(-n // P)) <= lat <= L * T


def test_schedule_invariants_on_random_graphs():
    """Any list schedule: a vertex starts after its predecessors finish (plus communication across
    processors), a processor runs one vertex at a time, latency is bounded by the critical path below
    and by the serial time plus all communication above."""
    rng = random.Random(11)
    for trial in range(40):
        n = rng.randint(1, 30)
        pred = [sorted(rng.sample(range(v), rng.randint(0, min(v, 3)))) for v in range(n)]
        comm = [[rng.choice([0.0, 0.5, 2.0]) for _ in p] for p in pred]
        ex = [rng.choice([0.5, 1.0, 2.5]) for _ in range(n)]
        order = S.topological_order(n, pred, comm, ex)
        P = rng.randint(1, 4)
        proc, aft, lat = S.simulate(n, pred, order, P, ex, comm)
        start = [aft[v] - ex[v] for v in range(n)]
        for v in range(n):
            for i, m in enumerate(pred[v]):
                assert start[v] >= aft[m] + (comm[v][i] if proc[m] != proc[v] else 0.0) - 1e-12
        for j in range(P):
            iv = sorted((start[v], aft[v]) for v in range(n) if proc[v] == j)
            assert all(iv[i][1] <= iv[i + 1][0] + 1e-12 for i in range(len(iv) - 1))
        depth = [0.0] * n
        for v in range(n):
            depth[v] = ex[v] + max([depth[m] for m in pred[v]], default=0.0)
        assert max(depth) - 1e-12 <= lat <= sum(ex) + sum(map(sum, comm)) + 1e-12
        assert lat == max(aft)


def test_greedy_choice_against_brute_force_on_tiny_graphs():
    """The placement rule (smallest finish time, ties to the lowest index) checked vertex by vertex
    against an exhaustive evaluation of all processors with independently written start-time code."""
    rng = random.Random(3)
    for trial in range(30):
        n = rng.randint(2, 7)
        pred = [sorted(rng.sample(range(v), rng.randint(0, min(v, 2)))) for v in range(n)]
        comm = [[rng.choice([0.0, 1.0, 3.0]) for _ in p] for p in pred]
        ex = [rng.choice([1.0, 2.0]) for _ in range(n)]
        order = list(range(n))
        P = 3
        proc, aft, _ = S.simulate(n, pred, order, P, ex, comm)
        free = [0.0] * P
        for v in order:
            cands = []
            for j in range(P):
                t0 = free[j]
                for m, c in zip(pred[v], comm[v]):
                    t0 = max(t0, aft[m] + (0.0 if proc[m] == j else c))
                cands.append((t0 + ex[v], j))
            assert (aft[v], proc[v]) == min(cands)
            free[proc[v]] = aft[v]


# ---- placement under the residency rule (a processor holds one kind per pass, a kind one processor) ----

def _kinds_of_grid(L, T, D):
    return [v // T for v in range(L * D * T)]          # vertex (l*D + d)*T + s -> kind l*D + d


@pytest.mark.parametrize("L,T,D,LP", [(1, 7, 1, 1), (4, 6, 1, 4), (8, 5, 1, 4), (8, 9, 1, 3), (12, 16, 1, 12),
                                      (3, 6, 2, 1), (2, 5, 2, 2), (8, 40, 1, 1)])
def test_resident_placement_closed_forms_on_the_grid(L, T, D, LP):
    """Unit cells, free communication, P = LP * D processors: a pass holds LP layers and layer l runs in pass l // LP.
    One direction: on processor l % LP, inside a pass every cell finishes at its depth, and the passes add up to the
    sum over passes of (layers in the pass + T - 1).  Two directions: a layer needs the layer below at the same
    TIME, which the backward direction reaches in its last step, so layers follow one another (finish of step s of
    layer l: l * T + s + 1, latency L * T) whatever the pass holds, and the two directions of a layer sit on two
    different processors (which of them gets which is a matter of the order among vertices that are ready together)."""
    n, pred = S.grid_dag(L, T, D)
    comm = _zeros_like(pred)
    order = S.topological_order(n, pred, comm, [1.0] * n)
    proc, pass_of, aft, lat, passes = S.place_resident(n, pred, order, LP * D, [1.0] * n, comm, _kinds_of_grid(L, T, D))
    assert passes == -(-L // LP)
    t0 = 0
    starts = []
    for r in range(passes):
        starts.append(t0)
        t0 += min(LP, L - r * LP) + T - 1
    assert lat == (t0 if D == 1 else L * T)
    for l in range(L):
        for d in range(D):
            for s in range(T):
                v = S.vertex_id(L, T, D, l, d, s)
                assert pass_of[v] == l // LP
                assert proc[v] == proc[S.vertex_id(L, T, D, l, d, 0)]
                if D == 1:
                    assert proc[v] == l % LP
                    assert aft[v] == starts[l // LP] + (l % LP) + s + 1
                else:
                    assert aft[v] == l * T + s + 1
    for r in range(passes):
        kinds = sorted({v // T for v in range(n) if pass_of[v] == r})
        procs = [proc[k * T] for k in kinds]
        assert sorted(procs) == list(range(len(kinds)))          # one processor each, the lowest ones


def test_resident_placement_one_kind_is_serial():
    """All vertices of one kind: everything runs on processor 0 in one pass, one after the other in the given
    order, whatever P is."""
    rng = random.Random(5)
    n = 25
    pred = [sorted(rng.sample(range(v), rng.randint(0, min(v, 3)))) for v in range(n)]
    comm = [[rng.choice([0.0, 1.5]) for _ in p] for p in pred]
    ex = [rng.choice([0.5, 1.0, 2.0]) for _ in range(n)]
    order = S.topological_order(n, pred, comm, ex)
    proc, pass_of, aft, lat, passes = S.place_resident(n, pred, order, 3, ex, comm, [7] * n)
    assert passes == 1 and set(proc) == {0} and set(pass_of) == {0}
    t = 0.0
    for v in order:
        t += ex[v]
        assert aft[v] == pytest.approx(t)
    assert lat == pytest.approx(sum(ex))


def test_resident_placement_worked_example():
    """Four vertices, two kinds, ONE processor: a -> b, a -> c, (b, c) -> d with kinds a, c: 0 and b, d: 1, unit
    times, order a b c d.  Pass 0 places a (the processor now holds kind 0), skips b (kind 1), places c, skips d
    (b is not placed): it ends at 2.  Pass 1 places b in [2, 3] and d in [3, 4].  With two processors there is one
    pass: a on 0 in [0, 1]; b on 1 (empty) from 1 + 0.5 (communication across processors) to 2.5; c on 0 in [1, 2];
    d on processor 1 (its kind lives there): ready when b is done (2.5) and c has arrived (2 + 0.5) -> [2.5, 3.5]."""
    pred = [[], [0], [0], [1, 2]]
    comm = [[], [0.5], [0.5], [0.5, 0.5]]
    kind = [0, 1, 0, 1]
    proc, pass_of, aft, lat, passes = S.place_resident(4, pred, [0, 1, 2, 3], 1, [1.0] * 4, comm, kind)
    assert (passes, pass_of, proc) == (2, [0, 1, 0, 1], [0, 0, 0, 0])
    assert aft == [1.0, 3.0, 2.0, 4.0] and lat == 4.0
    proc, pass_of, aft, lat, passes = S.place_resident(4, pred, [0, 1, 2, 3], 2, [1.0] * 4, comm, kind)
    assert (passes, pass_of, proc) == (1, [0, 0, 0, 0], [0, 1, 0, 1])
    assert aft == [1.0, 2.5, 2.0, 3.5] and lat == 3.5


def test_resident_placement_invariants_on_random_graphs():
    """Every vertex is placed once; it starts after its predecessors (plus communication across processors) and not
    before its pass; a processor runs one vertex at a time and one kind per pass; a kind uses one processor per
    pass; a pass starts when the one before it has ended; a predecessor never sits in a later pass."""
    rng = random.Random(23)
    for trial in range(60):
        n = rng.randint(1, 40)
        pred = [sorted(rng.sample(range(v), rng.randint(0, min(v, 3)))) for v in range(n)]
        comm = [[rng.choice([0.0, 0.5, 2.0]) for _ in p] for p in pred]
        ex = [rng.choice([0.5, 1.0, 2.5]) for _ in range(n)]
        kind = [rng.randint(0, 5) for _ in range(n)]
        order = S.topological_order(n, pred, comm, ex)
        P = rng.randint(1, 4)
        proc, pass_of, aft, lat, passes = S.place_resident(n, pred, order, P, ex, comm, kind)
        assert all(0 <= proc[v] < P and 0 <= pass_of[v] < passes for v in range(n))
        start = [aft[v] - ex[v] for v in range(n)]
        ends = [max([aft[v] for v in range(n) if pass_of[v] == r]) for r in range(passes)]
        begins = [0.0] + ends[:-1]
        for v in range(n):
            assert start[v] >= begins[pass_of[v]] - 1e-12
            for i, m in enumerate(pred[v]):
                assert pass_of[m] <= pass_of[v]
                assert start[v] >= aft[m] + (comm[v][i] if proc[m] != proc[v] else 0.0) - 1e-12
        for r in range(passes):
            assert min(start[v] for v in range(n) if pass_of[v] == r) >= begins[r] - 1e-12
            for j in range(P):
                mine = [v for v in range(n) if pass_of[v] == r and proc[v] == j]
                assert len({kind[v] for v in mine}) <= 1
                iv = sorted((start[v], aft[v]) for v in mine)
                assert all(iv[i][1] <= iv[i + 1][0] + 1e-12 for i in range(len(iv) - 1))
            for k in set(kind):
                assert len({proc[v] for v in range(n) if pass_of[v] == r and kind[v] == k}) <= 1
        assert lat == max(aft)
        # with as many processors as kinds nothing ever waits for a second pass
        _, _, _, _, one = S.place_resident(n, pred, order, 6, ex, comm, kind)
        assert one == 1
