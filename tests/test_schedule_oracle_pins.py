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
