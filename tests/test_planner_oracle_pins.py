"""Pins for oracle/planner.py against what the paper and the mathematics fix (no GPU, no product code)."""
import itertools
import random

import pytest

from oracle import planner as P


# ---- dependency materialization example (Section 3.3): A1, A2 produce the left and right halves,
# ---- B1 consumes the top half; the overlaps are the top-left and the top-right quarter
def test_materialization_example_overlaps():
    R, C = 8, 6
    a1 = P.VTensor(op=0, tensor=0, lo=(0, 0), hi=(R, C // 2))
    a2 = P.VTensor(op=1, tensor=0, lo=(0, C // 2), hi=(R, C))
    b1 = P.VTensor(op=2, tensor=0, lo=(0, 0), hi=(R // 2, C))
    assert P.intersect(a1, b1) == ((0, 0), (R // 2, C // 2))
    assert P.intersect(a2, b1) == ((0, C // 2), (R // 2, C))
    assert P.intersect(a1, a2) is None
    assert P.data_dependencies([a1, a2], [b1]) == [(0, 2), (1, 2)]
    # a consumer of the bottom-right quarter depends on A2 only; another pTensor never matches
    b2 = P.VTensor(op=3, tensor=0, lo=(R // 2, C // 2), hi=(R, C))
    other = P.VTensor(op=4, tensor=1, lo=(0, 0), hi=(R, C))
    assert P.data_dependencies([a1, a2], [b2, other]) == [(1, 3)]


def _brute_force_orders(n, edges):
    return [p for p in itertools.permutations(range(n)) if all(p.index(a) < p.index(b) for a, b in edges)]


@pytest.mark.parametrize("seed", range(40))
def test_acyclic_iff_an_order_exists_and_the_order_is_the_smallest(seed):
    rng = random.Random(seed)
    n = rng.randint(1, 6)
    m = rng.randint(0, 9)
    edges = [(rng.randrange(n), rng.randrange(n)) for _ in range(m)]
    edges = [(a, b) for a, b in edges if a != b] + ([(0, 0)] if seed % 13 == 5 else [])
    orders = _brute_force_orders(n, edges)
    assert P.has_cycle(n, edges) == (len(orders) == 0)
    order = P.topo_order(n, edges)
    if orders:
        assert tuple(order) == min(orders)  # always taking the smallest ready operator = lexicographic minimum
    else:
        assert order is None


def test_replicated_producers_one_acyclic_choice_is_enough():
    # ops: 0, 1 = replicas producing the same tensor; 2 = consumer; happen-before 2 -> 0 (op-order)
    # taking the data from replica 0 would close a cycle, replica 1 is fine
    ok, choice, order = P.validate_schedule(3, fixed_edges=[(2, 0)], alternatives=[[(0, 2), (1, 2)]])
    assert ok and choice == (1,) and order == [1, 2, 0]
    # with 2 -> 1 as well no choice works
    ok, choice, order = P.validate_schedule(3, fixed_edges=[(2, 0), (2, 1)], alternatives=[[(0, 2), (1, 2)]])
    assert not ok and choice is None and order is None
    # brute force over both alternatives agrees
    for fixed in ([(2, 0)], [(2, 0), (2, 1)], []):
        feasible = any(_brute_force_orders(3, fixed + [e]) for e in [(0, 2), (1, 2)])
        assert P.validate_schedule(3, fixed, [[(0, 2), (1, 2)]])[0] == feasible


def test_coshard_chunk_order_on_one_device():
    # Section 2 / 3.2: k forward chunks then k backward chunks on one device; backward chunk c reads
    # what forward chunk c produced (recompute aside), op-order chains the chunks
    k = 4
    fwd = [P.VTensor(op=c, tensor=0, lo=(c * 3,), hi=(c * 3 + 3,)) for c in range(k)]
    bwd = [P.VTensor(op=k + c, tensor=0, lo=(c * 3,), hi=(c * 3 + 3,)) for c in range(k)]
    data = P.data_dependencies(fwd, bwd)
    assert data == [(c, k + c) for c in range(k)]
    chain = [(c, c + 1) for c in range(2 * k - 1)]
    ok, _, order = P.validate_schedule(2 * k, data + chain)
    assert ok and order == list(range(2 * k))
    # an op-order that puts backward chunk 0 before forward chunk 0 contradicts the data dependency
    ok, _, _ = P.validate_schedule(2 * k, data + chain + [(k, 0)])
    assert not ok
    # with no op-order at all the completion is still a valid order
    ok, _, order = P.validate_schedule(2 * k, data)
    assert ok and all(order.index(a) < order.index(b) for a, b in data)


# ---- RVD (Section 5)
def test_rvd_example_counts_and_path():
    src, mid, dst = (1, 2, 1, 2), (2, 1, 1, 2), (2, 1, 2, 1)
    assert src[0] * src[1] * src[2] * src[3] == 4  # R(1)V(2)D(1,2) stands for 4 vTensors
    # the chain the paper gives: all-reduce over every 2 tensors, then all-to-all over every two
    steps = [(P.ALL_REDUCE, -1, -1, 2), (P.ALL_TO_ALL, 1, 0, 2)]
    t1, s1 = P.path_time(src, steps[:1], 1 << 20)
    assert s1 == mid
    t2, s2 = P.path_time(src, steps, 1 << 20)
    assert s2 == dst and t2 > t1 > 0
    # an illegal step (no value split left to reduce) is rejected
    assert P.path_time(mid, [(P.ALL_REDUCE, -1, -1, 2)], 1 << 20) == (None, None)


def test_every_transition_keeps_the_device_count_and_has_an_inverse_kind():
    for state in [(1, 2, 1, 2), (2, 1, 2, 1), (4, 2, 1), (1, 1, 8), (8, 1, 1), (2, 2, 2, 2)]:
        n = state[0] * state[1] * P._prod(state[2:])
        for prim, a, b, g, ns in P.transitions(state):
            assert ns[0] * ns[1] * P._prod(ns[2:]) == n and all(x >= 1 for x in ns)
            back = {(p2, ns2) for p2, _, _, _, ns2 in P.transitions(ns)}
            inverse = {P.ALL_REDUCE: P.VCHUNK, P.VCHUNK: P.ALL_REDUCE, P.ALL_GATHER: P.SCHUNK, P.SCHUNK: P.ALL_GATHER,
                       P.ALL_TO_ALL: P.ALL_TO_ALL}.get(prim)
            if inverse is not None:
                assert (inverse, state) in back


def _cheapest_by_enumeration(src, dst, nbytes, cm, depth):
    best = None

    def walk(state, t, seen, n):
        nonlocal best
        if state == dst and (best is None or t < best):
            best = t
        if n == depth:
            return
        for prim, a, b, g, ns in P.transitions(state):
            if ns not in seen:
                walk(ns, t + P.edge_time(prim, g, state, nbytes, cm), seen | {ns}, n + 1)

    walk(src, 0, {src}, 0)
    return best


@pytest.mark.parametrize("src,dst", [((1, 2, 1, 2), (2, 1, 2, 1)), ((1, 4, 1), (1, 1, 4)), ((4, 1, 1), (1, 1, 4)),
                                     ((1, 1, 4, 2), (1, 1, 2, 4)), ((2, 2, 2), (8, 1, 1)), ((1, 8, 1), (8, 1, 1)),
                                     ((1, 1, 2, 2), (4, 1, 1, 1)), ((2, 1, 1, 4), (1, 2, 4, 1))])
@pytest.mark.parametrize("nbytes", [1 << 12, 1 << 24])
def test_dijkstra_matches_exhaustive_enumeration(src, dst, nbytes):
    cm = P.CostModel()
    found = P.rvd_search(src, dst, nbytes, cm)
    best = _cheapest_by_enumeration(src, dst, nbytes, cm, depth=4)
    if best is None:
        assert found is None or len(found[1]) > 4
    else:
        assert found is not None and found[0] == best
        t, end = P.path_time(src, [s[:4] for s in found[1]], nbytes, cm)
        assert (t, end) == (found[0], dst)


def test_closed_forms_single_primitive_cases():
    # the same-size categories of the micro-benchmark table (Section 6.5): one primitive each
    cm, nbytes = P.CostModel(), 16 << 20
    t, steps = P.rvd_search((1, 8, 1), (8, 1, 1), nbytes, cm)      # value split -> replicated: one all-reduce
    assert [s[0] for s in steps] == [P.ALL_REDUCE] and steps[0][3] == 8
    assert t == cm.alpha_ns + 2 * ((nbytes // 8) * 1000 // cm.link_bytes_per_us)
    t, steps = P.rvd_search((1, 8, 1), (1, 1, 8), nbytes, cm)      # value split -> partitioned: reduce-scatter
    assert [s[0] for s in steps] == [P.REDUCE_SCATTER] and t == cm.alpha_ns + (nbytes // 8) * 1000 // cm.link_bytes_per_us
    t, steps = P.rvd_search((1, 1, 8), (8, 1, 1), nbytes, cm)      # partitioned -> replicated: all-gather
    assert [s[0] for s in steps] == [P.ALL_GATHER] and t == cm.alpha_ns + (nbytes // 8) * 1000 // cm.link_bytes_per_us
    t, steps = P.rvd_search((8, 1, 1), (1, 1, 8), nbytes, cm)      # replicated -> partitioned: a local slice
    assert [s[0] for s in steps] == [P.SCHUNK] and t == cm.local_ns
    assert P.rvd_search((8, 1, 1), (8, 1, 1), nbytes, cm) == (0, [])
    assert P.rvd_search((8, 1, 1), (4, 1, 1), nbytes, cm) is None  # different device counts: not the same group


def test_the_examples_cheaper_chain_under_the_link_model():
    # under the direct-link model reduce-scatter + all-gather moves less than the example's
    # all-reduce + all-to-all (2/3 of it); both are legal chains to the same layout
    src, dst, nbytes, cm = (1, 2, 1, 2), (2, 1, 2, 1), 1 << 26, P.CostModel()
    t_paper, _ = P.path_time(src, [(P.ALL_REDUCE, -1, -1, 2), (P.ALL_TO_ALL, 1, 0, 2)], nbytes, cm)
    t_found, steps = P.rvd_search(src, dst, nbytes, cm)
    assert [s[0] for s in steps] == [P.REDUCE_SCATTER, P.ALL_GATHER] and t_found < t_paper
    m = nbytes // 2
    assert t_paper == 2 * cm.alpha_ns + 2 * ((m // 2) * 1000 // cm.link_bytes_per_us) + (m // 2) * 1000 // cm.link_bytes_per_us


# ---- the paper's printed examples as fixtures (tests/golden/, each with its citation)
def _golden(name):
    import json
    import os
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)) as fh:
        return json.load(fh)


def test_golden_rvd_worked_example():
    gold = _golden("rvd_worked_example.json")
    names = {n: i for i, n in enumerate(P.PRIMITIVE_NAMES)}
    state = tuple(gold["producer"])
    assert state[0] * state[1] * P._prod(state[2:]) == gold["vtensors_represented"]
    for step in gold["steps"]:
        options = [ns for prim, a, b, g, ns in P.transitions(state)
                   if prim == names[step["primitive"]] and g == step["over_every"] and ns == tuple(step["layout_after"])]
        assert len(options) == 1, step
        state = options[0]
    assert state == tuple(gold["consumer"])


def test_golden_materialization_example():
    gold = _golden("materialization_example.json")
    R, C = 10, 14
    region = {"left half": ((0, 0), (R, C // 2)), "right half": ((0, C // 2), (R, C)), "top half": ((0, 0), (R // 2, C)),
              "top-left part": ((0, 0), (R // 2, C // 2)), "top-right part": ((0, C // 2), (R // 2, C))}
    ops = {}
    for i, (name, where) in enumerate(list(gold["producers"].items()) + list(gold["consumer"].items())):
        lo, hi = region[where]
        ops[name] = P.VTensor(op=i, tensor=0, lo=lo, hi=hi)
    for pair, where in gold["overlaps"].items():
        a, b = pair.split(" and ")
        assert P.intersect(ops[a], ops[b]) == region[where]


def test_golden_microbenchmark_same_group_categories_take_one_primitive():
    gold = _golden("rvd_microbenchmark_categories.json")
    import re
    expected = {("R", "R"): [], ("R", "D"): [P.SCHUNK], ("V", "R"): [P.ALL_REDUCE], ("V", "D"): [P.REDUCE_SCATTER],
                ("D", "R"): [P.ALL_GATHER], ("D", "D"): []}
    assert len(gold["categories"]) * len(gold["configurations"]) == 18
    for cat in gold["categories"]:
        which = lambda text, sym: [m.group(1) for m in re.finditer(r"([RVD])\((%s)\)" % sym, text)][0]
        src_kind, dst_kind = which(cat["producers"], "i"), which(cat["consumers"], "j")
        for i, j in gold["configurations"]:
            layout = lambda kind, n: {"R": (n, 1, 1), "V": (1, n, 1), "D": (1, 1, n)}[kind]
            found = P.rvd_search(layout(src_kind, i), layout(dst_kind, j), 1 << 24)
            if i != j:
                assert found is None  # different group sizes: not a same-group search
            else:
                assert [s[0] for s in found[1]] == expected[(src_kind, dst_kind)]
