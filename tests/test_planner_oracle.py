"""Pins for the integer planner oracle (oracle/planner.py), Sec. 5 of the paper.

Pinned against: the paper's Table 2 at its grid points, hand-worked
interpolation and a hand-worked three-node plan, Eq. 4-5 as inequalities,
brute-force optimal schedules on tiny instances (the 4/3 - 1/(3m) bound of
longest-first list scheduling), exact-tiling invariants, and a CPU replay of
the emitted task list that must reproduce the definition oracle.
"""
import itertools
import random

import numpy as np
import pytest

from oracle import attention as A
from oracle import method as M
from oracle import planner as P
from golden_tables import load_table2
from workloads import (HeadConfig, make_workload, two_level_forest, three_level_forest,
                       random_forest, unshared_forest, concat_forests, Forest, DTYPE_BF16, DTYPE_FP16)

TABLE2 = load_table2()
LINEAR = {"row_grid": [1], "len_grid": [100, 200], "cost": [[100, 200]]}   # cost = max(n, 100)


def test_table2_values_at_grid_points():
    """Sec. 5.2, Table 2: every printed entry is returned at its own (n_q, n)."""
    assert TABLE2["row_grid"] == [1, 2, 5, 10, 20, 50, 100]
    assert TABLE2["len_grid"] == [512, 1024, 2048, 4096, 8192, 16384]
    assert P.c_est(TABLE2, 1, 512) == 36 and P.c_est(TABLE2, 100, 16384) == 746
    assert P.c_est(TABLE2, 10, 4096) == 126 and P.c_est(TABLE2, 50, 1024) == 109
    for ri, r in enumerate(TABLE2["row_grid"]):
        for ni, n in enumerate(TABLE2["len_grid"]):
            assert P.c_est(TABLE2, r, n) == TABLE2["cost"][ri][ni]


def test_interpolation_lies_between_neighbours_and_clamps():
    rng = random.Random(0)
    rg, ng, c = TABLE2["row_grid"], TABLE2["len_grid"], TABLE2["cost"]
    for _ in range(500):
        ri, ni = rng.randrange(len(rg) - 1), rng.randrange(len(ng) - 1)
        r, n = rng.randint(rg[ri], rg[ri + 1]), rng.randint(ng[ni], ng[ni + 1])
        corners = [c[ri][ni], c[ri + 1][ni], c[ri][ni + 1], c[ri + 1][ni + 1]]
        assert min(corners) <= P.c_est(TABLE2, r, n) <= max(corners)
    assert P.c_est(TABLE2, 1, 16) == 36            # below the grid: launch-dominated, clamped
    assert P.c_est(TABLE2, 1, 32768) == 283 + 2 * (283 - 156)   # above: continue the last segment


def test_interpolation_hand_worked_rounding():
    t = {"row_grid": [1, 3], "len_grid": [10, 20], "cost": [[10, 20], [30, 41]]}
    assert P.c_est(t, 2, 15) == 25                 # 505/20 = 25.25
    t["cost"][1][1] = 42
    assert P.c_est(t, 2, 15) == 26                 # 510/20 = 25.5, half rounds up
    assert P.c_est(t, 1, 30) == 30                 # extrapolated along n
    assert P.c_est(t, 5, 10) == 50                 # extrapolated along rows
    assert P.c_est(t, 1, 5) == 10                  # clamped
    assert P.c_est({"row_grid": [4], "len_grid": [8], "cost": [[7]]}, 99, 1) == 7


def test_slices_tile_exactly():
    for n in list(range(1, 200)) + [4096, 131072, 32769]:
        for align in (16, 32, 256):
            for b in (1, 2, 3, 5, 8, 33, 1000):
                count, length, last = P.slices(n, b, align)
                assert length % align == 0 and 0 < last <= length
                assert (count - 1) * length + last == n
                assert count <= max(1, b)
                assert P.slices(n, count, align)[0] == count      # normal form is stable


def _brute_opt(costs, m):
    best = None
    for assign in itertools.product(range(m), repeat=len(costs)):
        loads = [0] * m
        for c, s in zip(costs, assign):
            loads[s] += c
        ms = max(loads)
        best = ms if best is None else min(best, ms)
    return best


def test_longest_first_schedule_against_brute_force_optimum():
    rng = random.Random(1)
    for _ in range(120):
        m = rng.randint(2, 3)
        t = rng.randint(1, 7)
        costs = [rng.randint(1, 30) for _ in range(t)]
        sub = [(c, i, 0) for i, c in enumerate(costs)]
        ms, slot_of, lists = P.lpt(sub, m)
        opt = _brute_opt(costs, m)
        assert opt <= ms
        assert 3 * m * ms <= (4 * m - 1) * opt
        assert ms >= max(max(costs), -(-sum(costs) // m))
        assert sorted(i for l in lists for i in l) == list(range(t))
        for s, l in enumerate(lists):
            assert all(slot_of[i] == s for i in l)
    # ties go to the lowest slot id and the order inside a slot is assignment order
    ms, slot_of, lists = P.lpt([(5, 0, 0), (5, 1, 0), (5, 2, 0), (1, 3, 0)], 3)
    assert slot_of == [0, 1, 2, 0] and lists[0] == [0, 3] and ms == 6


def test_hand_worked_three_node_plan():
    """Root of 1200 tokens under two requests, two 100-token leaves, 4 slots, cost = tokens.

    Total load 1400 -> cost_l = 350 (Eq. 4); root bound ceil(1200/350) = 4 slices (Eq. 5);
    makespans for 1..4 root slices: 1200, 600, 400, 400 -> 3 slices (tie to the coarser).
    """
    f = two_level_forest(1200, [100, 100])
    p = P.plan(f.parent, f.node_len, f.req_node, group=1, num_slots=4, align=100,
               max_rows=64, share=True, table=LINEAR)
    assert p["cost_l"] == 350
    assert [it["ub"] for it in p["items"]] == [4, 1, 1]
    assert [it["b"] for it in p["items"]] == [3, 1, 1]
    assert p["makespan"] == 400
    assert [(t["node"], t["kv_begin"], t["kv_len"]) for t in p["tasks"]] == \
        [(0, 0, 400), (0, 400, 400), (0, 800, 400), (1, 0, 100), (2, 0, 100)]
    assert [t["slot"] for t in p["tasks"]] == [0, 1, 2, 3, 3]
    assert [t["part_row_base"] for t in p["tasks"]] == [0, 2, 4, 6, 7]
    assert p["slot_off"] == [0, 1, 2, 3, 5] and p["slot_tasks"] == [0, 1, 2, 3, 4]
    assert p["node_q"] == [0, 1, 0, 1] and p["node_q_off"] == [0, 2, 3, 4]
    assert p["req_part_off"] == [0, 4, 8]
    assert p["req_part"] == [0, 2, 4, 6, 1, 3, 5, 7]
    assert p["part_rows"] == 8


def _check_invariants(f, p, group, m, align, slack=False):
    n_q = np.zeros(f.num_nodes, dtype=np.int64)
    for r in range(f.num_requests):
        for n in f.path(r):
            n_q[n] += 1
    # slices of one item tile [0, len) in order, on aligned boundaries
    by_item = {}
    for t in p["tasks"]:
        by_item.setdefault(t["item"], []).append(t)
    for j, ts in by_item.items():
        pos = 0
        for t in ts:
            assert t["kv_begin"] == pos and t["kv_begin"] % align == 0 and t["kv_len"] > 0
            pos += t["kv_len"]
        assert pos == f.node_len[p["items"][j]["node"]]
    # every (request, head-of-group, token) is covered once
    covered = sum(t["n_req"] * group * t["kv_len"] for t in p["tasks"])
    assert covered == int((f.node_len.astype(np.int64) * n_q).sum()) * group
    # schedule: each task in exactly one slot, loads give the makespan, lower bounds hold
    assert sorted(p["slot_tasks"]) == list(range(len(p["tasks"])))
    loads = [sum(p["tasks"][i]["cost"] for i in p["slot_tasks"][p["slot_off"][s]:p["slot_off"][s + 1]])
             for s in range(m)]
    assert max(loads) == p["makespan"]
    total = sum(t["cost"] for t in p["tasks"])
    assert p["makespan"] >= max(-(-total // m), max(t["cost"] for t in p["tasks"]))
    # Eq. 5 as printed: b_k <= ceil(C_est / cost_l).  Only under the library's slack extension may a
    # node whose cost is at least a quarter of cost_l exceed it, and then by one slice.
    for it in p["items"]:
        over = 1 if slack and 4 * it["cost"] >= p["cost_l"] else 0
        assert 1 <= it["b"] <= it["ub"] <= max(1, -(-it["cost"] // p["cost_l"])) + over
    # Eq. 4 at cost_l: the division it induces fits m slots on average, the next finer T does not
    def tot(T):
        return sum(P.division_cost(p["table"], it["rows"], it["len"],
                                   min(-(-it["cost"] // T), it["max_b"]), align) for it in p["items"])
    assert tot(p["cost_l"]) <= m * p["cost_l"]
    if p["cost_l"] > 1:
        assert tot(p["cost_l"] - 1) > m * (p["cost_l"] - 1)
    # partial rows: disjoint, dense
    rows = sorted((t["part_row_base"], t["n_req"] * group) for t in p["tasks"])
    pos = 0
    for base, cnt in rows:
        assert base == pos
        pos += cnt
    assert pos == p["part_rows"]


FORESTS = {
    "docqa": lambda: two_level_forest(10000, [50] * 24),
    "three": lambda: three_level_forest(2048, [8192] * 4, 5, [37 + 13 * i for i in range(20)]),
    "random": lambda: random_forest(40, 5, 2.0, 512, 1.0, 16, 32768, seed=8),
    "mixed": lambda: concat_forests(two_level_forest(30000, [100] * 9), unshared_forest([7000, 8000, 50])),
}


@pytest.mark.parametrize("name", sorted(FORESTS))
@pytest.mark.parametrize("share", [True, False])
@pytest.mark.parametrize("m,align,max_rows,group", [(8, 256, 64, 4), (3, 32, 16, 8), (64, 64, 64, 1)])
@pytest.mark.parametrize("slack,diagonal", [(False, False), (True, False), (False, True), (True, True)])
def test_plan_invariants(name, share, m, align, max_rows, group, slack, diagonal):
    """With both extensions off the bound asserted is the printed Eq. 5, with no slack term."""
    f = FORESTS[name]()
    p = P.plan(f.parent, f.node_len, f.req_node, group, m, align, max_rows, share, TABLE2,
               slack=slack, diagonal=diagonal)
    p["table"] = TABLE2
    _check_invariants(f, p, group, m, align, slack=slack)
    if not slack and not diagonal:
        # extensions only ever add candidates to the search: the printed solver's makespan is an upper bound
        q = P.plan(f.parent, f.node_len, f.req_node, group, m, align, max_rows, share, TABLE2, diagonal=True)
        assert q["makespan"] <= p["makespan"]


def test_docqa_leaves_are_not_divided():
    """Sec. 5.1: Eq. 5 leaves tasks far below the average cost (the per-request questions) whole."""
    f = FORESTS["docqa"]()
    p = P.plan(f.parent, f.node_len, f.req_node, 4, 16, 32, 64, True, LINEAR)
    assert all(it["b"] == 1 for it in p["items"] if it["len"] == 50)
    assert max(it["b"] for it in p["items"] if it["len"] == 10000) > 1


def test_flat_plan_gives_every_request_its_own_tasks():
    f = two_level_forest(640, [33, 70, 5])
    p = P.plan(f.parent, f.node_len, f.req_node, 4, 4, 32, 64, False, LINEAR)
    assert all(it["n_req"] == 1 for it in p["items"])
    assert sum(1 for it in p["items"] if it["node"] == 0) == 3


def test_requests_ending_inside_the_tree_and_unused_nodes():
    f = Forest(np.array([-1, 0, 0, -1]), np.array([300, 40, 50, 77]), np.array([1, 0, 1]))
    p = P.plan(f.parent, f.node_len, f.req_node, 2, 2, 32, 64, True, LINEAR)
    assert {it["node"] for it in p["items"]} == {0, 1}        # nodes 2 and 3 have no request
    assert p["node_q"] == [0, 1, 2, 0, 2]
    p["table"] = LINEAR
    _check_invariants(f, p, 2, 2, 32)


@pytest.mark.parametrize("bad", [
    (np.array([0]), np.array([4]), np.array([0])),           # self parent
    (np.array([1, 0]), np.array([4, 4]), np.array([0])),     # cycle
    (np.array([-1]), np.array([0]), np.array([0])),          # empty node
    (np.array([-1]), np.array([4]), np.array([1])),          # request beyond the forest
    (np.array([5]), np.array([4]), np.array([0])),           # parent out of range
])
def test_malformed_forests_are_rejected(bad):
    with pytest.raises(ValueError):
        P.plan(bad[0], bad[1], bad[2], 1, 2, 32, 64, True, LINEAR)


@pytest.mark.parametrize("share", [True, False])
@pytest.mark.parametrize("dtype,hq,hkv,max_rows", [(DTYPE_BF16, 8, 2, 8), (DTYPE_FP16, 2, 2, 64)])
def test_cpu_replay_of_the_task_list_equals_the_definition(share, dtype, hq, hkv, max_rows):
    """Run the emitted tasks (PAC per task, POR per request) in fp64: must be the oracle's output."""
    f = three_level_forest(90, [130, 40], 3, [5, 33, 64, 1, 17, 48])
    head = HeadConfig(hq, hkv, 16, dtype, page_size=16)
    w = make_workload("replay", f, head, seed=77, poison=True)
    table = {"row_grid": [1, 64], "len_grid": [16, 256], "cost": [[20, 100], [40, 300]]}
    p = P.plan(f.parent, f.node_len, f.req_node, head.group, 40, 16, max_rows, share, table)
    assert any(it["b"] > 1 for it in p["items"])
    tasks = [(t["node"], t["kv_begin"], t["kv_len"], t["q_off"], t["n_req"], t["part_row_base"])
             for t in p["tasks"]]
    got = M.replay_tasks(w, tasks, p["node_q"], p["req_part_off"], p["req_part"])
    ref, _ = A.decode_attention_workload(w)
    assert np.max(np.abs(got - ref)) < 1e-13


# ---- carrying a plan over to new lengths (task division only every few decoding steps) -----------

def test_refresh_hand_worked():
    """The three-node plan above after growth: root 1200 -> 1250, leaves 100 -> 101 and 100 -> 164.

    Slices keep their boundaries (0, 400, 800): the root's last slice becomes 450 tokens; slot loads
    with cost = tokens: 400, 400, 450, 101 + 164 -> makespan 450.
    """
    f = two_level_forest(1200, [100, 100])
    p = P.plan(f.parent, f.node_len, f.req_node, group=1, num_slots=4, align=100,
               max_rows=64, share=True, table=LINEAR)
    q = P.refresh(p, LINEAR, [1250, 101, 164])
    assert [(t["node"], t["kv_begin"], t["kv_len"], t["cost"]) for t in q["tasks"]] == \
        [(0, 0, 400, 400), (0, 400, 400, 400), (0, 800, 450, 450), (1, 0, 101, 101), (2, 0, 164, 164)]
    assert [t["slot"] for t in q["tasks"]] == [t["slot"] for t in p["tasks"]]
    assert [it["len"] for it in q["items"]] == [1250, 101, 164]
    assert q["makespan"] == 450
    for k in ("slot_off", "slot_tasks", "node_q", "node_q_off", "req_part", "req_part_off", "part_rows", "cost_l"):
        assert q[k] == p[k]
    # the original plan is not touched
    assert p["tasks"][2]["kv_len"] == 400 and p["makespan"] == 400
    # unchanged lengths: identity
    same = P.refresh(p, LINEAR, [1200, 100, 100])
    assert same["tasks"] == p["tasks"] and same["makespan"] == p["makespan"]
    # shrinking the root to the start of its last slice leaves that slice empty
    with pytest.raises(ValueError):
        P.refresh(p, LINEAR, [800, 100, 100])
    assert P.refresh(p, LINEAR, [801, 100, 100])["tasks"][2]["kv_len"] == 1


@pytest.mark.parametrize("name", sorted(FORESTS))
def test_refresh_keeps_the_invariants(name):
    f = FORESTS[name]()
    group, m, align = 4, 8, 256
    p = P.plan(f.parent, f.node_len, f.req_node, group, m, align, 64, True, TABLE2)
    p["table"] = TABLE2
    rng = np.random.Generator(np.random.PCG64(5))
    grown = f.node_len + rng.integers(0, 40, size=f.num_nodes)
    q = P.refresh(p, TABLE2, grown)
    q["table"] = TABLE2
    g = Forest(f.parent, grown.astype(np.int32), f.req_node)
    # every invariant of a plan except those of the search (cost_l, bounds) holds for the carried plan
    by_item = {}
    for t in q["tasks"]:
        by_item.setdefault(t["item"], []).append(t)
    for j, ts in by_item.items():
        pos = 0
        for t in ts:
            assert t["kv_begin"] == pos and t["kv_len"] > 0
            assert t["cost"] == P.c_est(TABLE2, q["items"][j]["rows"], t["kv_len"])
            pos += t["kv_len"]
        assert pos == g.node_len[q["items"][j]["node"]]
    loads = [sum(q["tasks"][i]["cost"] for i in q["slot_tasks"][q["slot_off"][s]:q["slot_off"][s + 1]])
             for s in range(m)]
    assert max(loads) == q["makespan"]
    assert [(t["kv_begin"], t["slot"], t["part_row_base"]) for t in q["tasks"]] == \
        [(t["kv_begin"], t["slot"], t["part_row_base"]) for t in p["tasks"]]


def test_fixed_slice_count_is_the_naive_even_division():
    """Granularity study: every node cut evenly into n slices (fewer when it is too short)."""
    f = two_level_forest(1200, [100, 250])
    p = P.plan(f.parent, f.node_len, f.req_node, group=1, num_slots=4, align=100,
               max_rows=64, share=True, table=LINEAR, fixed_slices=3)
    assert [it["b"] for it in p["items"]] == [3, 1, 3]
    assert [(t["node"], t["kv_begin"], t["kv_len"]) for t in p["tasks"]] == \
        [(0, 0, 400), (0, 400, 400), (0, 800, 400), (1, 0, 100), (2, 0, 100), (2, 100, 100), (2, 200, 50)]
    # longest first onto 4 slots: 400, 400, 400 | 100, 100, 100, 50 -> 350
    assert p["makespan"] == 400
    _check_invariants_of_division(f, p, 1, 4, 100)
    one = P.plan(f.parent, f.node_len, f.req_node, 1, 4, 100, 64, True, LINEAR, fixed_slices=1)
    assert [it["b"] for it in one["items"]] == [1, 1, 1] and one["makespan"] == 1200


def _check_invariants_of_division(f, p, group, m, align):
    by_item = {}
    for t in p["tasks"]:
        by_item.setdefault(t["item"], []).append(t)
    for j, ts in by_item.items():
        pos = 0
        for t in ts:
            assert t["kv_begin"] == pos and t["kv_begin"] % align == 0 and t["kv_len"] > 0
            pos += t["kv_len"]
        assert pos == f.node_len[p["items"][j]["node"]]
    loads = [sum(p["tasks"][i]["cost"] for i in p["slot_tasks"][p["slot_off"][s]:p["slot_off"][s + 1]])
             for s in range(m)]
    assert max(loads) == p["makespan"]


def test_best_candidate_plan_hand_worked():
    """Two requests under a 100-token root, 100-token leaves, group 8, 2 slots, cost = rows * tokens.

    Shared plan (16-row tiles cover both requests): root 16 * 100 = 1600, leaves 800 each -> loads
    1600 | 1600 -> 1600.  Flat: four tasks of 800 -> 1600 as well: the tie goes to the shared plan.
    With a table that charges rows beyond 8 triple, the shared root costs 8*100 + 3*8*100 = 3200
    -> makespan 3200 and the flat plan (1600) wins.
    """
    f = two_level_forest(100, [100, 100])
    prop = {"row_grid": [1, 17], "len_grid": [1, 101], "cost": [[1, 101], [17, 1717]]}          # rows * tokens
    steep = {"row_grid": [8, 16], "len_grid": [1, 101], "cost": [[8, 808], [32, 3232]]}
    for table, want_share, want_ms in ((prop, True, 1600), (steep, False, 1600)):
        p = P.plan_best(f.parent, f.node_len, f.req_node, 8, 100, 16, {"narrow": table, "wide": table},
                        lambda wide: 2)
        assert (p["share"], p["makespan"]) == (want_share, want_ms)


def test_half_width_row_tiles_hand_worked():
    """64 requests end at one 100-token node, group 1, row tiles of at most 64, cost = rows * tokens.

    On 2 slots: one 64-row task costs 6400 and leaves a slot idle; two 32-row tiles cost 3200 each, one
    per slot -> 3200; four 16-row tiles -> two per slot, 3200; the flat plan, 64 tasks of 100 -> 3200.
    The three ties go to the earliest candidate, the 32-row tiles.  On 1 slot all four come to 6400
    and the tie goes to the 64-row plan.
    """
    f = Forest(np.array([-1]), np.array([100]), np.zeros(64, dtype=np.int32))
    prop = {"row_grid": [1, 65], "len_grid": [1, 101], "cost": [[1, 101], [65, 6565]]}          # rows * tokens
    for slots, want_rows, want_ms in ((2, 32, 3200), (1, 64, 6400)):
        p = P.plan_best(f.parent, f.node_len, f.req_node, 1, 100, 64, {"narrow": prop, "wide": prop},
                        lambda wide: slots)
        assert (p["share"], p["max_rows"], p["makespan"]) == (True, want_rows, want_ms)
        assert len(p["tasks"]) == 64 // want_rows


def test_slice_bound_slack_hand_worked():
    """Eight 1000-token contexts and a 100-token one on 4 slots, cost = tokens, slices of 100 tokens.

    Total 8100 -> cost_l = 2025; every quotient is 1.  The printed bound keeps all nodes whole: two
    long contexts per slot and the short one on top, makespan 2100.  With one slice of slack for
    nodes of at least cost_l / 4 = 507 (the long ones; not the short one) the search may halve a long
    context; it does so for none, because two per slot already is the best packing, and the short
    node stays whole in any case.
    """
    f = unshared_forest([1000] * 8 + [100])
    p = P.plan(f.parent, f.node_len, f.req_node, group=1, num_slots=4, align=100,
               max_rows=64, share=True, table=LINEAR, slack=True)
    assert p["cost_l"] == 2025
    assert [it["ub"] for it in p["items"]] == [2] * 8 + [1]
    assert p["makespan"] == 2100
    strict = P.plan(f.parent, f.node_len, f.req_node, group=1, num_slots=4, align=100,
                    max_rows=64, share=True, table=LINEAR)
    assert strict["cost_l"] == 2025 and [it["ub"] for it in strict["items"]] == [1] * 9      # Eq. 5 as printed
    assert strict["makespan"] == 2100
    # three contexts of 1000 on 2 slots: whole -> 2000; the slack lets one be halved -> 1500
    g = unshared_forest([1000] * 3)
    q = P.plan(g.parent, g.node_len, g.req_node, group=1, num_slots=2, align=100,
               max_rows=64, share=True, table=LINEAR, slack=True)
    assert q["cost_l"] == 1500 and [it["ub"] for it in q["items"]] == [2, 2, 2]
    assert q["makespan"] == 1500 and sorted(it["b"] for it in q["items"]) == [1, 1, 2]
    # the printed bound: ceil(1000 / 1500) = 1 slice each, nothing to search, two contexts on one slot
    q0 = P.plan(g.parent, g.node_len, g.req_node, group=1, num_slots=2, align=100,
                max_rows=64, share=True, table=LINEAR)
    assert q0["cost_l"] == 1500 and [it["ub"] for it in q0["items"]] == [1, 1, 1] and q0["makespan"] == 2000


def test_diagonal_of_the_grid_hand_worked():
    """Two 1200-token contexts on 8 slots, cost = tokens, slices on multiples of 20 tokens.

    Total 2400 -> cost_l = 300; quotient 4, bound 5 with the slack.  Node by node from (5, 5): with the
    other node in 5 slices of 240, the first node in 3 slices of 400 gives 8 tasks on 8 slots, makespan
    400; 4 slices (4 x 300 + 5 x 240: nine tasks, one slot holds 240 + 240) or 5 slices give 480, so 3 is
    kept; then the second node: 3, 4 or 5 slices all leave the makespan at 400, the first of them, 3, is
    kept.  That point, (3, 3), is one no single move improves.  The diagonal point of target cost_l,
    (4, 4), packs 8 slices of 300 onto the 8 slots: makespan 300, which is the lower bound.
    """
    f = unshared_forest([1200, 1200])
    # Sec. 5.1 as printed: bound 4 each; from (4, 4): first node 3 slices of 400 beside 4 of 300 -> 7 tasks
    # on 8 slots, makespan 400; 4 slices -> 8 x 300 on 8 slots, 300: kept; second node likewise stays at 4
    p0 = P.plan(f.parent, f.node_len, f.req_node, group=1, num_slots=8, align=20,
                max_rows=64, share=True, table=LINEAR)
    assert p0["cost_l"] == 300 and [it["ub"] for it in p0["items"]] == [4, 4]
    assert [it["b"] for it in p0["items"]] == [4, 4] and p0["makespan"] == 300
    # with the slack alone the pass starts from (5, 5) and stops at (3, 3), as worked out above
    p1 = P.plan(f.parent, f.node_len, f.req_node, group=1, num_slots=8, align=20,
                max_rows=64, share=True, table=LINEAR, slack=True)
    assert [it["ub"] for it in p1["items"]] == [5, 5] and [it["b"] for it in p1["items"]] == [3, 3]
    assert p1["makespan"] == 400
    p = P.plan(f.parent, f.node_len, f.req_node, group=1, num_slots=8, align=20,
               max_rows=64, share=True, table=LINEAR, slack=True, diagonal=True)
    assert p["cost_l"] == 300
    assert [it["ub"] for it in p["items"]] == [5, 5]
    assert [it["b"] for it in p["items"]] == [4, 4]
    assert p["makespan"] == 300 and len(p["tasks"]) == 8
    assert sorted(t["kv_len"] for t in p["tasks"]) == [300] * 8



def test_cpu_replay_with_visibility_masks_equals_the_definition():
    """Plan a forest whose drafted-token nodes carry masks, run the emitted tasks on the CPU (Alg. 2 with
    the mask of Sec. 4.1 per task, Alg. 3 per request): the definition oracle's output.  Masked nodes get
    row tiles of at most 16 rows and are never divided."""
    from workloads import draft_masked_forest
    f = draft_masked_forest(90, [130, 40, 333], 21, seed=6)
    head = HeadConfig(8, 2, 16, DTYPE_BF16, page_size=16)
    w = make_workload("replay-masked", f, head, seed=78, poison=True)
    table = {"row_grid": [1, 64], "len_grid": [16, 256], "cost": [[20, 100], [40, 300]]}
    masked = {int(f.req_node[r]) for r in range(f.num_requests) if f.visible(r) is not None}
    p = P.plan(f.parent, f.node_len, f.req_node, head.group, 40, 16, 64, True, table, masked_nodes=masked)
    assert any(it["b"] > 1 for it in p["items"])
    for it in p["items"]:
        if it["node"] in masked:
            assert it["rows"] <= 16 and it["b"] == 1 and it["ub"] == 1
    tasks = [(t["node"], t["kv_begin"], t["kv_len"], t["q_off"], t["n_req"], t["part_row_base"])
             for t in p["tasks"]]
    got = M.replay_tasks(w, tasks, p["node_q"], p["req_part_off"], p["req_part"])
    ref, _ = A.decode_attention_workload(w)
    assert np.max(np.abs(got - ref)) < 1e-13
    p["table"] = table
    _check_invariants(f, p, head.group, 40, 16)
