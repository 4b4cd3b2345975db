"""Oracle for the host-side planner pieces.  TEST INFRASTRUCTURE ONLY: the product never imports it.

Plain Python, written from the paper's description, small and slow on purpose:

* Section 3.2, "Scheduling validation and completion", and Section 3.3, "Dependency
  materialization": data dependencies are found by intersecting the index masks of produced and
  consumed vTensors of the same pTensor; together with the happen-before relations (op-order) they
  form a dependency graph; a schedule is feasible iff that graph is acyclic; where a consumer may
  take its data from any one of several replicated producers the alternatives are enumerated and
  one acyclic choice is enough; a topological sort completes the order.
* Section 5, "RVD representation" and "Communication primitive search over RVD graph": a layout
  R(i)V(j)D(k1..kn) of one tensor over a device group; every collective is a transition rule
  between layouts; edges are weighted with the time of the primitive and Dijkstra's algorithm
  gives the cheapest chain of primitives from the producers' layout to the consumers'.

Readings (the figure that lists the primitives is not part of the text):
* the six same-group primitives are taken to be all-reduce (V -> R), all-gather (D -> R),
  reduce-scatter (V -> D), all-to-all (D on one axis -> D on another), schunk (R -> D, a local
  slice, named in Section 6.5) and vchunk (R -> V, local: one replica keeps the value, the others
  contribute zero).  Each acts on groups of g devices, g > 1 a divisor of the factor it consumes.
* edge weight = alpha + bytes over the busiest link / link bandwidth for a directly connected group
  (every device talks to each of its g - 1 peers at once, over a link of its own): with m the bytes
  of one device's vTensor BEFORE the primitive, reduce-scatter and all-to-all send a 1/g slice
  (m / g) over every link, all-gather sends the whole piece (m), all-reduce is a reduce-scatter
  followed by an all-gather of the slices (2 m / g); the local primitives cost a fixed small time.  All times are integer nanoseconds computed with integer arithmetic, so that two
  implementations agree exactly.
* ties are broken towards fewer primitives (alpha > 0 does that) and then towards the
  lexicographically smallest sequence of (primitive, axis, axis2, g) so that the result is unique.
"""
from __future__ import annotations

import heapq
import itertools
from dataclasses import dataclass

# ----------------------------------------------------------------------------------------------
# dependencies and schedule validation
# ----------------------------------------------------------------------------------------------


@dataclass(frozen=True)
class VTensor:
    """One vTensor: which operator touches it, which pTensor it is a view of, and its mask: a
    half-open index range per dimension (the value-split index plays no part in a dependency)."""
    op: int
    tensor: int
    lo: tuple
    hi: tuple


def intersect(a: VTensor, b: VTensor):
    """The overlapped portion of two views of the same pTensor, or None."""
    if a.tensor != b.tensor or len(a.lo) != len(b.lo):
        return None
    lo = tuple(max(x, y) for x, y in zip(a.lo, b.lo))
    hi = tuple(min(x, y) for x, y in zip(a.hi, b.hi))
    if any(l >= h for l, h in zip(lo, hi)):
        return None
    return lo, hi


def data_dependencies(produced, consumed):
    """All (producer op, consumer op) pairs whose masks intersect, sorted, without duplicates."""
    edges = set()
    for p in produced:
        for c in consumed:
            if p.op != c.op and intersect(p, c) is not None:
                edges.add((p.op, c.op))
    return sorted(edges)


def has_cycle(n, edges):
    """Depth-first search with three colours."""
    adj = [[] for _ in range(n)]
    for a, b in edges:
        adj[a].append(b)
    colour = [0] * n

    def visit(u):
        colour[u] = 1
        for v in adj[u]:
            if colour[v] == 1:
                return True
            if colour[v] == 0 and visit(v):
                return True
        colour[u] = 2
        return False

    return any(colour[u] == 0 and visit(u) for u in range(n))


def topo_order(n, edges):
    """The topological order that always takes the smallest ready operator (unique)."""
    indeg = [0] * n
    adj = [[] for _ in range(n)]
    for a, b in set(edges):
        adj[a].append(b)
        indeg[b] += 1
    ready = [u for u in range(n) if indeg[u] == 0]
    heapq.heapify(ready)
    order = []
    while ready:
        u = heapq.heappop(ready)
        order.append(u)
        for v in adj[u]:
            indeg[v] -= 1
            if indeg[v] == 0:
                heapq.heappush(ready, v)
    return order if len(order) == n else None


def validate_schedule(n, fixed_edges, alternatives=()):
    """fixed_edges: data dependencies and happen-before pairs that must all hold.
    alternatives: groups of edges of which exactly one is chosen (a consumer that may read any one
    of several replicated producers).  Tries the choices in lexicographic order of their indices
    and returns (feasible, choice, order) for the first acyclic one."""
    alternatives = [list(g) for g in alternatives]
    for choice in itertools.product(*[range(len(g)) for g in alternatives]):
        edges = list(fixed_edges) + [alternatives[i][c] for i, c in enumerate(choice)]
        if not has_cycle(n, edges):
            return True, tuple(choice), topo_order(n, edges)
    return False, None, None


# ----------------------------------------------------------------------------------------------
# RVD
# ----------------------------------------------------------------------------------------------

ALL_REDUCE, ALL_GATHER, REDUCE_SCATTER, ALL_TO_ALL, SCHUNK, VCHUNK = range(6)
PRIMITIVE_NAMES = ("all-reduce", "all-gather", "reduce-scatter", "all-to-all", "schunk", "vchunk")


@dataclass(frozen=True)
class CostModel:
    """alpha_ns: nanoseconds per primitive; link_bytes_per_us: bytes per microsecond of one
    point-to-point link; local_ns: nanoseconds of a primitive that moves nothing between devices."""
    alpha_ns: int = 10000
    link_bytes_per_us: int = 153000
    local_ns: int = 1000


def divisors(x):
    return [g for g in range(2, x + 1) if x % g == 0]


def device_bytes(state, tensor_bytes):
    """Bytes of one device's vTensor in layout `state` = (r, v, d1, .., dn)."""
    n = int(tensor_bytes)
    for d in state[2:]:
        n //= d
    return n


def transitions(state):
    """Every (primitive, axis, axis2, g, next_state) one primitive away.  axis / axis2 are tensor
    axes (0-based) or -1 where they do not apply."""
    r, v, d = state[0], state[1], list(state[2:])
    out = []
    for g in divisors(v):
        out.append((ALL_REDUCE, -1, -1, g, (r * g, v // g, *d)))
        for a in range(len(d)):
            nd = d.copy()
            nd[a] *= g
            out.append((REDUCE_SCATTER, a, -1, g, (r, v // g, *nd)))
    for a in range(len(d)):
        for g in divisors(d[a]):
            nd = d.copy()
            nd[a] //= g
            out.append((ALL_GATHER, a, -1, g, (r * g, v, *nd)))
            for b in range(len(d)):
                if b != a:
                    nb = nd.copy()
                    nb[b] *= g
                    out.append((ALL_TO_ALL, a, b, g, (r, v, *nb)))
    for g in divisors(r):
        out.append((VCHUNK, -1, -1, g, (r // g, v * g, *d)))
        for a in range(len(d)):
            nd = d.copy()
            nd[a] *= g
            out.append((SCHUNK, a, -1, g, (r // g, v, *nd)))
    return out


def edge_time(prim, g, state, tensor_bytes, cm: CostModel):
    m = device_bytes(state, tensor_bytes)
    if prim in (SCHUNK, VCHUNK):
        return cm.local_ns
    if prim == ALL_GATHER:
        return cm.alpha_ns + m * 1000 // cm.link_bytes_per_us
    pieces = 2 if prim == ALL_REDUCE else 1
    return cm.alpha_ns + pieces * ((m // g) * 1000 // cm.link_bytes_per_us)


def rvd_search(src, dst, tensor_bytes, cm: CostModel = CostModel()):
    """Dijkstra from layout src to layout dst (same device count).  Returns (time, steps) with
    steps = [(primitive, axis, axis2, g, state_after)], or None when dst cannot be reached."""
    if len(src) != len(dst):
        return None
    prod = lambda s: s[0] * s[1] * _prod(s[2:])
    if prod(src) != prod(dst):
        return None
    best = {src: (0, ())}
    heap = [(0, (), src)]
    while heap:
        t, path, s = heapq.heappop(heap)
        if best.get(s, (None, None)) != (t, path):
            continue
        if s == dst:
            steps, cur = [], src
            for prim, a, b, g in path:
                cur = next(ns for p2, a2, b2, g2, ns in transitions(cur) if (p2, a2, b2, g2) == (prim, a, b, g))
                steps.append((prim, a, b, g, cur))
            return t, steps
        for prim, a, b, g, ns in transitions(s):
            nt = t + edge_time(prim, g, s, tensor_bytes, cm)
            npath = path + ((prim, a, b, g),)
            if ns not in best or (nt, npath) < best[ns]:
                best[ns] = (nt, npath)
                heapq.heappush(heap, (nt, npath, ns))
    return None


def _prod(xs):
    p = 1
    for x in xs:
        p *= x
    return p


def path_time(src, steps, tensor_bytes, cm: CostModel = CostModel()):
    """Time of a given chain of (primitive, axis, axis2, g); None if a step is not a legal transition."""
    t, cur = 0, src
    for prim, a, b, g in steps:
        nxt = [ns for p2, a2, b2, g2, ns in transitions(cur) if (p2, a2, b2, g2) == (prim, a, b, g)]
        if not nxt:
            return None, None
        t += edge_time(prim, g, cur, tensor_bytes, cm)
        cur = nxt[0]
    return t, cur
