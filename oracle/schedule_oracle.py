"""Plain, slow reference for the host-side scheduling of the cell graph.  TEST INFRASTRUCTURE ONLY:
imported by tests/ (and nothing in the product path); shares no code with the library.

What it follows in the paper (Section 3: the computation graph G = (V, E), predecessor and successor
sets, earliest start time EST and earliest finish time EFT of a vertex on a processor, the latency
L = the largest actual finish time; Section 4.1: Algorithm "Topological Sorting" and the text
around it):

  grid_dag        the unrolled RNN of Section 2.2 as a graph: one vertex per cell (layer, direction,
                  step), an edge from the cell of the previous step of the same layer and direction,
                  and edges from the cells of the layer below at the same time (all directions).
  topological_order
                  the sorting algorithm of Section 4.1.  The printed pseudo-code initialises a ready
                  queue with the vertices without predecessors, pops the first element, appends it
                  to the order when all its predecessors are marked and pushes it back otherwise; it
                  never enqueues a successor and has no merge step, although the text describes one.
                  Reading used here: after appending a vertex, every successor that is not yet
                  queued is pushed to the back of the queue (breadth first), except that a
                  successor with exactly one predecessor whose communication time from that
                  predecessor exceeds its average execution time is appended to the order at once,
                  before anything else (depth first: locality), and the rule is applied again to
                  that successor's own successors.
  simulate        list scheduling of the vertices in a given order on P processors with the EST /
                  EFT rules of Section 3: a vertex can start on processor j when j is free and every
                  predecessor has finished, plus the communication time of the edge when the
                  predecessor ran on another processor (reading: the printed formula adds the
                  communication time of every edge; with processors that share one memory an edge
                  inside a processor costs nothing, the usual convention of list scheduling, and
                  with one processor the printed formula would otherwise delay a chain by its
                  edges); it is placed on the processor with the smallest EFT, ties to the lowest
                  index.  Latency = the largest finish time.

  place_resident  the same list scheduling under a residency rule, the form of the paper's memory
                  constraint (Section 3, Equation 4: what a device holds is bounded) that the
                  persistent kernels impose: every vertex has a kind (the weights it needs: its layer
                  and direction), a processor (a group of compute units) holds the weights of ONE kind
                  for the length of a launch and a kind lives on ONE processor.  Reading used here:
                  the vertices are taken in the given order in passes (a pass is a launch); in a pass
                  a vertex is placed when all its predecessors are placed and its kind's processor,
                  or else a processor that holds nothing yet, exists: on its kind's processor if the
                  kind has one, otherwise on the empty processor with the smallest EFT (ties to the
                  lowest index), which then holds that kind; a vertex that cannot be placed waits
                  for the next pass, which starts, with all processors empty, when the last vertex
                  of this pass has finished (launches on one stream run one after the other).

Every function is a direct transcription of these definitions with Python lists and loops.
"""
from __future__ import annotations

from collections import deque
from typing import List, Sequence, Tuple


def vertex_id(L: int, T: int, D: int, l: int, d: int, s: int) -> int:
    """Vertex of layer l, direction d, s-th step in that direction's processing order."""
    return (l * D + d) * T + s


def grid_dag(L: int, T: int, D: int) -> Tuple[int, List[List[int]]]:
    """Returns (n, pred) with pred[v] the sorted list of predecessors of vertex v.
    Direction 0 processes time t = s, direction 1 processes time t = T-1-s."""
    n = L * D * T
    pred: List[List[int]] = [[] for _ in range(n)]
    for l in range(L):
        for d in range(D):
            for s in range(T):
                v = vertex_id(L, T, D, l, d, s)
                if s > 0:
                    pred[v].append(vertex_id(L, T, D, l, d, s - 1))
                if l > 0:
                    t = s if d == 0 else T - 1 - s
                    for d2 in range(D):
                        s2 = t if d2 == 0 else T - 1 - t
                        pred[v].append(vertex_id(L, T, D, l - 1, d2, s2))
                pred[v].sort()
    return n, pred


def successors(n: int, pred: Sequence[Sequence[int]]) -> List[List[int]]:
    succ: List[List[int]] = [[] for _ in range(n)]
    for v in range(n):
        for m in pred[v]:
            succ[m].append(v)
    return succ  # ascending by construction


def topological_order(n: int, pred: Sequence[Sequence[int]], comm: Sequence[Sequence[float]],
                      avg_exec: Sequence[float]) -> List[int]:
    """comm[v][i] = communication time of the edge pred[v][i] -> v; avg_exec[v] = execution time of
    v averaged over the devices."""
    succ = successors(n, pred)
    marked = [False] * n
    queued = [False] * n
    order: List[int] = []
    q = deque()
    for v in range(n):
        if len(pred[v]) == 0:
            q.append(v)
            queued[v] = True

    def append_with_merges(v: int) -> None:
        # depth first: append v; then, for its successors in ascending order, a mergeable one is
        # appended (with its own merges) before the next successor is looked at, any other one is
        # queued.  Written with an explicit stack of (vertex, index of the next successor).
        marked[v] = True
        order.append(v)
        stack = [[v, 0]]
        while stack:
            u, i = stack[-1]
            if i == len(succ[u]):
                stack.pop()
                continue
            stack[-1][1] = i + 1
            c = succ[u][i]
            if marked[c]:
                continue
            if len(pred[c]) == 1 and comm[c][0] > avg_exec[c]:
                marked[c] = True
                queued[c] = True
                order.append(c)
                stack.append([c, 0])
            elif not queued[c]:
                q.append(c)
                queued[c] = True

    guard = 0
    while q:
        v = q.popleft()
        if marked[v]:
            continue
        if all(marked[m] for m in pred[v]):
            append_with_merges(v)
            guard = 0
        else:
            q.append(v)
            guard += 1
            if guard > len(q) + 1:
                raise ValueError("the graph has a cycle")
    if len(order) != n:
        raise ValueError("the graph has a cycle or unreachable vertices")
    return order


def simulate(n: int, pred: Sequence[Sequence[int]], order: Sequence[int], P: int, exec_time: Sequence[float],
             comm: Sequence[Sequence[float]]):
    """Returns (proc[v], aft[v], latency)."""
    avail = [0.0] * P
    proc = [-1] * n
    aft = [0.0] * n
    for v in order:
        best_j, best_eft = -1, 0.0
        for j in range(P):
            est = avail[j]
            for i, m in enumerate(pred[v]):
                if proc[m] < 0:
                    raise ValueError("the order is not topological")
                ready = aft[m] + (comm[v][i] if proc[m] != j else 0.0)
                if ready > est:
                    est = ready
            eft = est + exec_time[v]
            if best_j < 0 or eft < best_eft:
                best_j, best_eft = j, eft
        proc[v] = best_j
        aft[v] = best_eft
        avail[best_j] = best_eft
    latency = 0.0
    for v in range(n):
        if aft[v] > latency:
            latency = aft[v]
    return proc, aft, latency


def place_resident(n: int, pred: Sequence[Sequence[int]], order: Sequence[int], P: int,
                   exec_time: Sequence[float], comm: Sequence[Sequence[float]], kind: Sequence[int]):
    """Returns (proc[v], pass_of[v], aft[v], latency, number of passes)."""
    proc = [-1] * n
    pass_of = [-1] * n
    aft = [0.0] * n
    waiting = list(order)
    if sorted(waiting) != list(range(n)):
        raise ValueError("the order is not a permutation of the vertices")
    start = 0.0
    r = 0
    while waiting:
        avail = [start] * P
        holds = [None] * P            # kind held by each processor in this pass
        left = []
        end = start
        for v in waiting:
            if any(pass_of[m] < 0 for m in pred[v]):
                left.append(v)
                continue
            if kind[v] in holds:
                allowed = [holds.index(kind[v])]
            else:
                allowed = [j for j in range(P) if holds[j] is None]
            if not allowed:
                left.append(v)
                continue
            best_j, best_eft = -1, 0.0
            for j in allowed:
                est = avail[j]
                for i, m in enumerate(pred[v]):
                    ready = aft[m] + (comm[v][i] if proc[m] != j else 0.0)
                    if ready > est:
                        est = ready
                eft = est + exec_time[v]
                if best_j < 0 or eft < best_eft:
                    best_j, best_eft = j, eft
            proc[v] = best_j
            pass_of[v] = r
            aft[v] = best_eft
            avail[best_j] = best_eft
            holds[best_j] = kind[v]
            if best_eft > end:
                end = best_eft
        if len(left) == len(waiting):
            raise ValueError("the order is not topological")
        waiting = left
        start = end
        r += 1
    return proc, pass_of, aft, max(aft) if n else 0.0, r
