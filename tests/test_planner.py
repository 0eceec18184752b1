"""The planning steps of Sections 4.2-4.3: the oracle against what the paper fixes (its worked
2 -> 8 example of Fig. 5, closed forms, invariants, brute force), then the library's C
functions against the oracle, bit for bit, over a sweep of sizes.  No GPU."""
import ctypes as C
import itertools
import math

import pytest

from oracle import planner_oracle as po
from paper_2502_09922_amd import binding as b


# ---- the oracle against the paper -----------------------------------------------------------
def test_fig5_worked_example_two_to_eight():
    """Fig. 5 / Section 4.2: 4 blocks, 2 sub-groups.  Sub-group 1 receives blocks 1-2 then 3-4,
    sub-group 2 blocks 3-4 then 1-2 (0-based here); destination nodes 3,4,5 and 6,7,8 form
    the pipelines (3,6), (4,7), (5,8)."""
    assert po.kway_order(4, 2, 0) == [0, 1, 2, 3]
    assert po.kway_order(4, 2, 1) == [2, 3, 0, 1]
    assert po.subgroup_sizes(8, 2) == [4, 4]
    dest = {0: [3, 4, 5], 1: [6, 7, 8]}  # node numbers of the figure
    pipes = po.pipelines([3, 3])
    assert [[dest[g][j] for g, j in p] for p in pipes] == [[3, 6], [4, 7], [5, 8]]
    # a pipeline member from sub-group i runs chunk i first: stages in block order
    assert [po.chunk_span(4, 2, i) for i in range(2)] == [(0, 2), (2, 4)]


@pytest.mark.parametrize("bk", [(4, 2), (16, 4), (32, 8), (7, 3), (5, 5), (3, 5), (1, 1), (34, 4)])
def test_kway_orders_are_shifted_permutations_and_complete_a_model_after_one_chunk(bk):
    nb, k = bk
    size = math.ceil(nb / k)
    orders = [po.kway_order(nb, k, g) for g in range(k)]
    for g, o in enumerate(orders):
        assert sorted(o) == list(range(nb))               # every block exactly once
        lo, hi = po.chunk_span(nb, k, g)
        assert o[: hi - lo] == list(range(lo, hi))        # own chunk first, in block order
    # group g's order is group 0's rotated by g chunks
    for g in range(k):
        lo, _ = po.chunk_span(nb, k, g)
        assert orders[g] == orders[0][lo:] + orders[0][:lo]
    # after ceil(b/k) steps the sub-groups together hold every block (first full instance)
    assert set(itertools.chain.from_iterable(o[:size] for o in orders)) == set(range(nb))
    # chunks tile [0, b) in order
    spans = [po.chunk_span(nb, k, i) for i in range(k)]
    assert spans[0][0] == 0 and spans[-1][1] == nb
    assert all(spans[i][1] == spans[i + 1][0] for i in range(k - 1))
    assert all(hi - lo <= size for lo, hi in spans)


def test_subgroup_sizes_are_even():
    for n in range(1, 40):
        for k in range(1, n + 1):
            s = po.subgroup_sizes(n, k)
            assert sum(s) == n and max(s) - min(s) <= 1 and s == sorted(s, reverse=True)
            if n % k == 0:
                assert s == [n // k] * k


def brute_pipelines(sizes):
    """Round by round: take the next free node of every sub-group that still has one; when
    only one sub-group is left, all its free nodes form the last pipeline."""
    left = [list(range(n)) for n in sizes]
    out = []
    while any(left):
        live = [g for g in range(len(sizes)) if left[g]]
        if len(live) == 1:
            out.append([(live[0], j) for j in left[live[0]]])
            left[live[0]] = []
        else:
            out.append([(g, left[g].pop(0)) for g in live])
    return out


def test_pipeline_generation_invariants_and_brute_force():
    for sizes in itertools.product(range(0, 5), repeat=3):
        pipes = po.pipelines(list(sizes))
        flat = [n for p in pipes for n in p]
        assert sorted(flat) == sorted((g, j) for g, n in enumerate(sizes) for j in range(n))
        assert pipes == brute_pipelines(sizes)
        for p in pipes:
            groups = [g for g, _ in p]
            # across sub-groups: one node of each, in sub-group order; else a single sub-group
            assert len(set(groups)) == len(groups) and groups == sorted(groups) or len(set(groups)) == 1
    # equal sub-groups (the case the paper prefers): exactly L pipelines of k nodes each
    assert po.pipelines([3, 3, 3, 3]) == [[(g, t) for g in range(4)] for t in range(3)]
    assert po.pipelines([3, 1]) == [[(0, 0), (1, 0)], [(0, 1), (0, 2)]]


def test_multicast_step_count_closed_form():
    assert po.multicast_steps(4, 4) == 4 + 2 - 1
    assert po.multicast_steps(16, 8) == 16 + 3 - 1
    assert po.multicast_steps(16, 5) == 16 + 3 - 1   # ceil(log2 5) = 3
    assert po.multicast_steps(1, 2) == 1
    for n in range(1, 70):
        assert po.multicast_steps(8, n) == 8 + math.ceil(math.log2(n)) - 1


def replay(b_, n_nodes, steps):
    """Plays a multicast schedule; checks that it is executable and returns who holds what."""
    n = n_nodes.bit_length() - 1
    have = [set() for _ in range(n_nodes)]
    have[0] = set(range(b_))
    for s, sends in enumerate(steps):
        got = []
        for u, (v, k) in sends.items():
            assert v == u ^ (1 << (s % n)), "partners walk the hypercube dimensions"
            assert k in have[u], "a node can only send what it holds at the start of the step"
            assert k not in have[v], "no block is sent to a node that already holds it"
            got.append((v, k))
        assert len({v for v, _ in got}) == len(got), "at most one block received per step"
        for v, k in got:
            have[v].add(k)
    return have


@pytest.mark.parametrize("n_nodes", [2, 4, 8, 16, 32])
def test_multicast_schedule_meets_the_step_count_of_section_4_2(n_nodes):
    """Section 4.2: a binomial-pipeline multicast of b blocks to N nodes takes b + log2 N - 1
    steps.  The oracle's schedule must be executable (senders hold what they send, one block
    in and one out per node and step), complete, free of redundant transfers, and exactly that
    long -- which is also the fewest steps possible: the last block cannot leave node 0 before
    step b - 1 and a block needs log2 N more steps to reach N nodes by doubling."""
    n = n_nodes.bit_length() - 1
    for nb in list(range(1, 12)) + [32, 34]:
        steps = po.multicast_schedule(nb, n_nodes)
        assert len(steps) == nb + n - 1 == po.multicast_steps(nb, n_nodes)
        have = replay(nb, n_nodes, steps)
        assert all(h == set(range(nb)) for h in have)
        assert sum(len(x) for x in steps) == nb * (n_nodes - 1)
        for s in range(nb):  # the source injects block s at step s
            assert steps[s][0][1] == s


def test_multicast_schedule_special_cases():
    # one block: the classic binomial tree, holders double every step
    steps = po.multicast_schedule(1, 16)
    holders = {0}
    for s, sends in enumerate(steps):
        assert set(sends) == holders
        holders |= {v for v, _ in sends.values()}
        assert len(holders) == 2 ** (s + 1)
    # two nodes: the source sends block s at step s, nothing else happens
    assert po.multicast_schedule(5, 2) == [{0: (1, s)} for s in range(5)]


def test_no_schedule_is_shorter_brute_force():
    """Exhaustive search over ALL schedules (any node may send any block it holds to any node,
    one block out and one in per node and step) for 4 nodes: none completes in fewer than
    b + 1 steps, so the oracle's schedule is optimal there."""
    def fewest(nb, n_nodes):
        start = tuple([frozenset(range(nb))] + [frozenset()] * (n_nodes - 1))
        full = frozenset(range(nb))
        frontier, seen, steps = {start}, {start}, 0
        while True:
            if any(all(h == full for h in st) for st in frontier):
                return steps
            nxt = set()
            for st in frontier:
                options = []
                for u in range(n_nodes):
                    opts = [None] + [(v, k) for v in range(n_nodes) if v != u for k in st[u] - st[v]]
                    options.append(opts)
                for choice in itertools.product(*options):
                    dests = [c[0] for c in choice if c]
                    if len(set(dests)) != len(dests):
                        continue
                    new = [set(h) for h in st]
                    for c in choice:
                        if c:
                            new[c[0]].add(c[1])
                    t = tuple(frozenset(h) for h in new)
                    if t not in seen:
                        seen.add(t)
                        nxt.add(t)
            frontier, steps = nxt, steps + 1
    for nb in (1, 2, 3):
        assert fewest(nb, 4) == nb + 1 == len(po.multicast_schedule(nb, 4))
    assert fewest(2, 2) == 2


# ---- the library against the oracle ------------------------------------------------------------
def c_multicast(nb, n_nodes):
    cap = nb + 8
    dest, blk = (C.c_int32 * (cap * n_nodes))(), (C.c_int32 * (cap * n_nodes))()
    n = C.c_int()
    assert b.ls_plan_multicast_schedule(nb, n_nodes, dest, blk, cap, C.byref(n)) == 0
    out = []
    for s in range(n.value):
        step = {}
        for u in range(n_nodes):
            d, k = dest[s * n_nodes + u], blk[s * n_nodes + u]
            assert (d < 0) == (k < 0)
            if d >= 0:
                step[u] = (d, k)
        out.append(step)
    return out


def test_library_multicast_schedule_matches_the_oracle_bit_for_bit():
    for n_nodes in (2, 4, 8, 16, 64):
        for nb in list(range(1, 20)) + [63, 64, 65, 130]:
            assert c_multicast(nb, n_nodes) == po.multicast_schedule(nb, n_nodes), (nb, n_nodes)


def test_library_multicast_schedule_rejects_bad_arguments():
    arr = (C.c_int32 * 64)()
    n = C.c_int()
    for nb, nn in ((0, 4), (4, 1), (4, 3), (4, 6), (4, 0), (-1, 4)):
        assert b.ls_plan_multicast_schedule(nb, nn, arr, arr, 16, C.byref(n)) == b.LS_ERR_INVALID_ARG
    assert b.ls_plan_multicast_schedule(4, 4, None, arr, 16, C.byref(n)) == b.LS_ERR_INVALID_ARG
    assert b.ls_plan_multicast_schedule(4, 4, arr, arr, 4, C.byref(n)) == b.LS_ERR_OOM  # 5 steps needed


def c_kway(nb, k, g):
    arr = (C.c_int32 * max(nb, 1))()
    assert b.ls_plan_kway_order(nb, k, g, arr) == 0
    return list(arr[:nb])


def c_pipelines(sizes):
    k, total = len(sizes), sum(sizes)
    sz = (C.c_int32 * max(k, 1))(*sizes)
    grp, idx = (C.c_int32 * max(total, 1))(), (C.c_int32 * max(total, 1))()
    start = (C.c_int32 * (total + 1))()
    n = C.c_int()
    assert b.ls_plan_pipelines(sz, k, grp, idx, start, total, C.byref(n)) == 0
    return [[(grp[i], idx[i]) for i in range(start[p], start[p + 1])] for p in range(n.value)]


def test_library_planner_matches_the_oracle_bit_for_bit():
    for nb in range(1, 40):
        for k in range(1, 10):
            for g in range(k):
                assert c_kway(nb, k, g) == po.kway_order(nb, k, g), (nb, k, g)
            lo, hi = C.c_int(), C.c_int()
            for i in range(k):
                assert b.ls_plan_chunk_span(nb, k, i, C.byref(lo), C.byref(hi)) == 0
                assert (lo.value, hi.value) == po.chunk_span(nb, k, i)
    for n in range(1, 40):
        for k in range(1, n + 1):
            arr = (C.c_int32 * k)()
            assert b.ls_plan_subgroup_sizes(n, k, arr) == 0
            assert list(arr) == po.subgroup_sizes(n, k)
        assert b.ls_plan_multicast_steps(8, n) == po.multicast_steps(8, n)
    for sizes in itertools.product(range(0, 5), repeat=3):
        assert c_pipelines(list(sizes)) == po.pipelines(list(sizes)), sizes
    assert c_pipelines([3, 3]) == po.pipelines([3, 3])
    assert c_pipelines([7, 2, 5, 2, 9]) == po.pipelines([7, 2, 5, 2, 9])


def test_library_planner_rejects_bad_arguments():
    arr = (C.c_int32 * 8)()
    assert b.ls_plan_kway_order(0, 1, 0, arr) == b.LS_ERR_INVALID_ARG
    assert b.ls_plan_kway_order(4, 0, 0, arr) == b.LS_ERR_INVALID_ARG
    assert b.ls_plan_kway_order(4, 2, 2, arr) == b.LS_ERR_INVALID_ARG
    assert b.ls_plan_kway_order(4, 2, 0, None) == b.LS_ERR_INVALID_ARG
    assert b.ls_plan_subgroup_sizes(3, 4, arr) == b.LS_ERR_INVALID_ARG
    assert b.ls_plan_multicast_steps(0, 4) == b.LS_ERR_INVALID_ARG
    sz = (C.c_int32 * 2)(3, 3)
    n = C.c_int()
    start = (C.c_int32 * 8)()
    assert b.ls_plan_pipelines(sz, 2, arr, arr, start, 5, C.byref(n)) == b.LS_ERR_OOM  # 6 nodes, room for 5
