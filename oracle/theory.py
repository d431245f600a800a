"""CPU oracle, part 1: graph theory of rollouts (Sec. 3 and App. A1).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the
GPU library is checked against.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path never does.
It shares no code with the GPU library.

Everything here works on plain integers: ``n_nodes`` and a list of edges
``(src, tgt)`` plus, where a rollout pattern is involved, a list ``R`` of 0/1
bits parallel to the edge list.

Pins (tests/test_oracle_theory.py): inference factors printed for the
skip+recurrent example net (Sec. 4: 3 sequential, 1 streaming); three most
sequential patterns of an input-fed 3-cycle (Fig. 2 caption); Lemma 1 bounds,
which coincide (16) for the example net; the two definitions of the inference
tableau (Eq. 5) computed by two unrelated algorithms; Theorem 1 on random
graphs; rejection of the input-less 4-cycle of Fig. A1.
"""
from __future__ import annotations

from itertools import product
from typing import List, Sequence, Tuple

EdgeList = Sequence[Tuple[int, int]]


class GraphError(ValueError):
    """Not a network: no edges, bad ids, or not input-connected (Sec. 3, definition of a network)."""


class RolloutError(ValueError):
    """Rollout pattern invalid: its rollout windows contain a cycle (Sec. 3, definition of validity)."""


def input_set(n_nodes: int, edges: EdgeList) -> List[int]:
    """I_N: all nodes without incoming edges (Eq. 1).  A self-edge is an incoming edge."""
    has_in = {t for (_, t) in edges}
    return [v for v in range(n_nodes) if v not in has_in]


def check_network(n_nodes: int, edges: EdgeList) -> None:
    """Definition of a network: 0 < |E| < inf, directed, input-connected, i.e.
    every node is the end of a path that starts in I_N."""
    if n_nodes <= 0 or len(edges) == 0:
        raise GraphError("a network needs nodes and at least one edge")
    for (s, t) in edges:
        if not (0 <= s < n_nodes and 0 <= t < n_nodes):
            raise GraphError(f"edge ({s},{t}) names a node outside 0..{n_nodes - 1}")
    inputs = input_set(n_nodes, edges)
    reached = set(inputs)
    frontier = list(inputs)
    while frontier:
        u = frontier.pop()
        for (s, t) in edges:
            if s == u and t not in reached:
                reached.add(t)
                frontier.append(t)
    # input nodes count as reached (they are where every such path starts)
    missing = [v for v in range(n_nodes) if v not in reached]
    if missing:
        raise GraphError(f"nodes {missing} are not reachable from the input set {inputs}")


def window_edges(n_nodes: int, edges: EdgeList, R: Sequence[int], W: int):
    """E_W of Eq. 2: ((i,u),(j,v)) with (u,v) in E and j = i + R((u,v)), both frames in 0..W."""
    out = []
    for (e, (u, v)) in enumerate(edges):
        for i in range(0, W + 1):
            j = i + R[e]
            if j <= W:
                out.append(((i, u), (j, v)))
    return out


def is_valid(n_nodes: int, edges: EdgeList, R: Sequence[int], W: int = 1) -> bool:
    """Validity by the definition itself: build the rollout window R_W and test it
    for cycles (repeatedly strip nodes without incoming window edges)."""
    for r in R:
        if r not in (0, 1):
            raise RolloutError("R(e) must be 0 or 1")
    ew = window_edges(n_nodes, edges, R, W)
    nodes = {(i, v) for i in range(W + 1) for v in range(n_nodes)}
    indeg = {nv: 0 for nv in nodes}
    succ = {nv: [] for nv in nodes}
    for (a, b) in ew:
        indeg[b] += 1
        succ[a].append(b)
    stack = [nv for nv in nodes if indeg[nv] == 0]
    removed = 0
    while stack:
        a = stack.pop()
        removed += 1
        for b in succ[a]:
            indeg[b] -= 1
            if indeg[b] == 0:
                stack.append(b)
    return removed == len(nodes)


def check_rollout(n_nodes: int, edges: EdgeList, R: Sequence[int]) -> None:
    if len(R) != len(edges):
        raise RolloutError("pattern length differs from edge count")
    if not is_valid(n_nodes, edges, R, 1):
        raise RolloutError("rollout window contains a cycle")


def tableau_longest_path(n_nodes: int, edges: EdgeList, R: Sequence[int], W: int):
    """Inference tableau, first form of Eq. 5: T((i,v)) = length of the longest
    path in R_W ending at (i,v) whose first edge does not end in frame 0.
    Computed by memoised recursion over the (acyclic) window."""
    ew = [(a, b) for (a, b) in window_edges(n_nodes, edges, R, W) if b[0] != 0]
    preds = {}
    for (a, b) in ew:
        preds.setdefault(b, []).append(a)
    memo = {}

    def longest(nv):
        if nv in memo:
            return memo[nv]
        best = 0
        for a in preds.get(nv, []):
            best = max(best, 1 + longest(a))
        memo[nv] = best
        return best

    import sys
    sys.setrecursionlimit(max(10000, sys.getrecursionlimit()))
    T = [[0] * n_nodes for _ in range(W + 1)]
    for i in range(W + 1):
        for v in range(n_nodes):
            T[i][v] = longest((i, v))
    return T


def tableau_update_steps(n_nodes: int, edges: EdgeList, R: Sequence[int], W: int):
    """Inference tableau, second form of Eq. 5: the number of applications of the
    update step U (Eq. 3-4) to S_init after which (i,v) is first marked computed.
    S_init marks frame 0 and the input nodes of every frame."""
    inputs = set(input_set(n_nodes, edges))
    ew = window_edges(n_nodes, edges, R, W)
    preds = {}
    for (a, b) in ew:
        preds.setdefault(b, []).append(a)
    S = {(i, v): 1 if (v in inputs or i == 0) else 0 for i in range(W + 1) for v in range(n_nodes)}
    T = {nv: (0 if S[nv] else None) for nv in S}
    n = 0
    while not all(S.values()):
        n += 1
        new = dict(S)
        for nv in S:
            if S[nv] == 0 and all(S[a] == 1 for a in preds.get(nv, [])):
                new[nv] = 1
                T[nv] = n
        if new == S:
            raise RolloutError("update steps do not reach the full state")
        S = new
    return [[T[(i, v)] for v in range(n_nodes)] for i in range(W + 1)]


def inference_factor(n_nodes: int, edges: EdgeList, R: Sequence[int]) -> int:
    """F(R) = max of the tableau over the window of size 1 (Eq. 6)."""
    T = tableau_longest_path(n_nodes, edges, R, 1)
    return max(max(row) for row in T)


def levels(n_nodes: int, edges: EdgeList, R: Sequence[int]) -> List[int]:
    """T_{R_1}((1,v)) for every node: the update step of a frame at which v is
    computed; 0 for input nodes."""
    return tableau_longest_path(n_nodes, edges, R, 1)[1]


def equally_model_parallel(n_nodes: int, edges: EdgeList, R1: Sequence[int], R2: Sequence[int]) -> bool:
    """R1 and R2 agree on every edge that does not leave an input node (Sec. 3)."""
    inputs = set(input_set(n_nodes, edges))
    return all(a == b for (a, b, (u, _)) in zip(R1, R2, edges) if u not in inputs)


def all_valid_patterns(n_nodes: int, edges: EdgeList):
    """Brute-force enumeration of the valid rollout patterns (2^|E| candidates)."""
    return [R for R in product((0, 1), repeat=len(edges)) if is_valid(n_nodes, edges, R, 1)]


def simple_cycles(n_nodes: int, edges: EdgeList):
    """All minimal cycles as tuples of edge indices (brute force, tiny graphs)."""
    found = set()
    out_edges = {}
    for ei, (s, t) in enumerate(edges):
        out_edges.setdefault(s, []).append(ei)

    def walk(start, node, path, seen_nodes):
        for ei in out_edges.get(node, []):
            t = edges[ei][1]
            if t == start:
                cyc = tuple(path + [ei])
                k = cyc.index(min(cyc))
                found.add(cyc[k:] + cyc[:k])
            elif t not in seen_nodes and t > start:
                walk(start, t, path + [ei], seen_nodes | {t})

    for v in range(n_nodes):
        walk(v, v, [], {v})
    return sorted(found)


def lemma1_bounds(n_nodes: int, edges: EdgeList):
    """(lower_forward, lower_cycles, upper) of Lemma 1: 2^|E_forward|, the best
    product of (2^|p|-1) over sets of pairwise edge-disjoint minimal cycles, and
    2^(|E|-|E_rec|)."""
    cycles = simple_cycles(n_nodes, edges)
    in_cycle = set()
    for c in cycles:
        in_cycle.update(c)
    n_forward = len(edges) - len(in_cycle)
    n_rec = sum(1 for (s, t) in edges if s == t)
    best = 1
    m = len(cycles)
    for mask in range(1 << m):
        chosen = [cycles[i] for i in range(m) if mask >> i & 1]
        used = set()
        ok = True
        for c in chosen:
            if used & set(c):
                ok = False
                break
            used |= set(c)
        if ok:
            p = 1
            for c in chosen:
                p *= (2 ** len(c) - 1)
            best = max(best, p)
    return 2 ** n_forward, best, 2 ** (len(edges) - n_rec)


def shortest_path_length(n_nodes: int, edges: EdgeList, target: int) -> int:
    """Number of edges on the shortest path from any input node to ``target``."""
    inputs = input_set(n_nodes, edges)
    dist = {v: 0 for v in inputs}
    frontier = list(inputs)
    while frontier:
        nxt = []
        for u in frontier:
            for (s, t) in edges:
                if s == u and t not in dist:
                    dist[t] = dist[u] + 1
                    nxt.append(t)
        frontier = nxt
    return dist[target]
