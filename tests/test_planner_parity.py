"""The library's planner (C++) against the independent integer re-derivation, bit for bit.

The paper gives the solver in prose (Sec. 5); the exact plan is therefore
pinned only by the two implementations agreeing, while the oracle itself is
pinned to the paper in test_planner_oracle.py.
"""
import random

import numpy as np
import pytest

import paper_2505_17694_amd as C
from oracle import planner as P
from golden_tables import load_table2
from workloads import (two_level_forest, three_level_forest, random_forest, unshared_forest,
                       concat_forests, degenerate_forest, full_kary_forest, draft_tree_forest, draft_masked_forest, Forest,
                       HeadConfig, build_paged_kv)
from workloads.configs import config_forest, config_head, CONFIG_NAMES

TABLE2 = load_table2()


def _tuple(t):
    return (t["row_grid"], t["len_grid"], t["cost"])


def _default_table(wide=1):
    rg, lg, c = C.codec_default_cost_table(wide)
    return {"row_grid": rg, "len_grid": lg, "cost": c}


def _lib_plan(f, head, m, align, max_rows, share, table, extensions=0):
    paged = build_paged_kv(f, head, seed=1)
    st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                   head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                   head.page_size, head.scale, m, align, max_rows, int(share),
                                   _tuple(table) if table is not None else None, extensions=extensions)
    assert st == C.CODEC_OK, C.codec_status_string(st)
    st, view = C.codec_plan_export(plan)
    assert st == C.CODEC_OK
    C.codec_plan_destroy(plan)
    return view


def _compare(view, ref):
    assert view["cost_l"] == ref["cost_l"]
    assert view["makespan"] == ref["makespan"]
    assert view["part_rows"] == ref["part_rows"]
    assert len(view["items"]) == len(ref["items"])
    for a, b in zip(view["items"], ref["items"]):
        for k in ("node", "q_off", "n_req", "rows", "len", "ub", "b", "cost"):
            assert a[k] == b[k], (k, a, b)
    assert len(view["tasks"]) == len(ref["tasks"])
    for a, b in zip(view["tasks"], ref["tasks"]):
        for k in ("item", "node", "kv_begin", "kv_len", "q_off", "n_req", "part_row_base", "slot", "cost"):
            assert a[k] == b[k], (k, a, b)
    for k in ("slot_off", "slot_tasks", "node_q_off", "node_q", "req_part_off", "req_part"):
        assert list(view[k]) == list(ref[k]), k


def test_cost_estimate_matches_oracle_everywhere():
    rng = random.Random(3)
    for table in (TABLE2, _default_table(0), _default_table(1),
                  {"row_grid": [1, 3], "len_grid": [10, 20], "cost": [[10, 20], [30, 42]]},
                  {"row_grid": [4], "len_grid": [8], "cost": [[7]]}):
        for _ in range(400):
            r, n = rng.randint(1, 300), rng.choice([rng.randint(1, 600), rng.randint(1, 200000)])
            assert C.codec_cost_estimate(_tuple(table), r, n) == P.c_est(table, r, n)
    assert C.codec_cost_estimate(None, 16, 256) == P.c_est(_default_table(0), 16, 256)
    assert C.codec_cost_estimate(None, 200, 5000) == P.c_est(_default_table(1), 200, 5000)
    # the paper's Table 2 at its own grid points through the C ABI
    assert C.codec_cost_estimate(_tuple(TABLE2), 10, 4096) == 126
    assert C.codec_cost_estimate(_tuple(TABLE2), 100, 16384) == 746


def test_built_in_tables_are_the_profilers_output():
    """The tables the library plans with are generated from the profiler's JSON at build time: every
    grid point and cost of codec_default_cost_table equals the file (no hand copy in between)."""
    import json
    import os
    path = os.path.join(os.path.dirname(C.LIB_PATH), "cost_table_mi355x.json")
    with open(path) as f:
        tables = json.load(f)
    for wide, key in ((0, "narrow"), (1, "wide")):
        got = _default_table(wide)
        assert got["row_grid"] == tables[key]["row_grid"]
        assert got["len_grid"] == tables[key]["len_grid"]
        assert got["cost"] == tables[key]["cost"]
    # the jump between the stream path (16 rows) and the dense path (17 rows) is a grid line of its own
    assert 16 in tables["wide"]["row_grid"] and 17 in tables["wide"]["row_grid"]
    i17, j32 = tables["wide"]["row_grid"].index(17), tables["wide"]["len_grid"].index(32)
    assert C.codec_cost_estimate(None, 17, 32) == tables["wide"]["cost"][i17][j32]


FORESTS = {
    "docqa": lambda: two_level_forest(10000, [50] * 24),
    "three": lambda: three_level_forest(2048, [8192] * 4, 5, [37 + 13 * i for i in range(20)]),
    "random": lambda: random_forest(60, 5, 2.0, 512, 1.0, 16, 32768, seed=8),
    "mixed": lambda: concat_forests(two_level_forest(30000, [100] * 9), unshared_forest([7000, 8000, 50])),
    "degenerate": lambda: degenerate_forest(6, 3000, 200),
    "binary": lambda: full_kary_forest(2, 5, lambda lvl: 4000 // lvl),
    "drafted": lambda: draft_tree_forest(700, [3000, 45, 1200], 9, seed=4),
    "inner_request": lambda: Forest(np.array([-1, 0, 0, -1]), np.array([300, 40, 50, 77]), np.array([1, 0, 1])),
}


@pytest.mark.parametrize("name", sorted(FORESTS))
@pytest.mark.parametrize("share", [True, False])
@pytest.mark.parametrize("m,align,max_rows,hq,hkv,table", [
    (8, 256, 64, 32, 8, "table2"), (3, 32, 16, 8, 1, "default"), (64, 64, 256, 8, 8, "table2"),
    (17, 32, 7, 28, 4, "default"), (32, 256, 130, 64, 8, "default")])
@pytest.mark.parametrize("extensions", [0, 1, 2, 3])
def test_library_plan_equals_rederivation(name, share, m, align, max_rows, hq, hkv, table, extensions):
    """extensions = 0 is the solver of Sec. 5.1 as printed; bit 0 the slack over Eq. 5, bit 1 the diagonal."""
    f = FORESTS[name]()
    head = HeadConfig(hq, hkv, 128)
    view = _lib_plan(f, head, m, align, max_rows, share, TABLE2 if table == "table2" else None, extensions)
    # without a caller's table the library takes the built-in one of the kernel variant the plan needs
    wide = max(it["rows"] for it in view["items"]) > 16
    tab = TABLE2 if table == "table2" else _default_table(wide)
    ref = P.plan(f.parent, f.node_len, f.req_node, head.group, m, align, max_rows, share, tab,
                 slack=bool(extensions & 1), diagonal=bool(extensions & 2))
    _compare(view, ref)
    if extensions == 0:             # Eq. 5 as printed, on the library's own numbers, no slack term
        for it in view["items"]:
            assert 1 <= it["b"] <= it["ub"] <= max(1, -(-it["cost"] // view["cost_l"]))


@pytest.mark.parametrize("name", CONFIG_NAMES)
@pytest.mark.parametrize("share", [True, False])
@pytest.mark.parametrize("extensions", [0, 3])
def test_measured_configurations_with_library_defaults(name, share, extensions):
    """Full-size forests of the measured configurations, default options of the library: the printed
    solver (extensions = 0) and the one the benchmark's headline runs (both extensions)."""
    f, head = config_forest(name), config_head(name)
    view = _lib_plan(f, head, 0, 0, 0, share, None, extensions)
    # library defaults: 256-token alignment, row tiles of 256, and as many slots as workgroups that
    # run at once (one per CU if any task holds more than 16 rows, else two)
    widest = max(it["rows"] for it in view["items"])
    m = (256 if widest > 16 else 512) // head.num_kv_heads
    assert view["num_slots"] == m
    ref = P.plan(f.parent, f.node_len, f.req_node, head.group, m, 256, 256, share,
                 _default_table(widest > 16), slack=bool(extensions & 1), diagonal=bool(extensions & 2))
    _compare(view, ref)
    if extensions == 0:
        for it in view["items"]:
            assert 1 <= it["b"] <= it["ub"] <= max(1, -(-it["cost"] // view["cost_l"]))


# ---- codec_plan_refresh_lengths against the oracle's refresh ---------------------------------------

def _grow_paged(f, head, grown, seed):
    g = Forest(f.parent, np.asarray(grown, dtype=np.int32), f.req_node)
    return g, build_paged_kv(g, head, seed=seed)


@pytest.mark.parametrize("name", sorted(FORESTS))
@pytest.mark.parametrize("share", [True, False])
def test_refresh_matches_oracle(name, share):
    f = FORESTS[name]()
    head = HeadConfig(32, 8, 128, 1)
    m, align, max_rows = 16, 64, 64
    table = _default_table(1)
    paged = build_paged_kv(f, head, seed=1)
    st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                   head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                   head.page_size, head.scale, m, align, max_rows, int(share), _tuple(table))
    assert st == C.CODEC_OK
    ref = P.plan(f.parent, f.node_len, f.req_node, 4, m, align, max_rows, share, table)
    rng = np.random.Generator(np.random.PCG64(11))
    lens = f.node_len.astype(np.int64)
    before = C.codec_plan_device_bytes(plan)
    for step in range(4):
        lens = lens + rng.integers(0, 3 if step < 3 else 70, size=f.num_nodes)
        g, gp = _grow_paged(f, head, lens, seed=2 + step)
        assert C.codec_plan_refresh_lengths(plan, g.node_len, gp.node_page_off, gp.page_ids) == C.CODEC_OK
        ref = P.refresh(ref, table, lens)
        st, view = C.codec_plan_export(plan)
        assert st == C.CODEC_OK
        _compare(view, ref)
    assert C.codec_plan_device_bytes(plan) >= before
    C.codec_plan_destroy(plan)


def test_refresh_error_paths_leave_the_plan_unchanged():
    f = two_level_forest(5000, [300, 40, 77])
    head = HeadConfig(8, 2, 128, 0)
    paged = build_paged_kv(f, head, seed=1)
    st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                   8, 2, 128, 0, 16, head.scale, 8, 32, 64, 1, None)
    assert st == C.CODEC_OK
    _, before = C.codec_plan_export(plan)
    assert max(it["b"] for it in before["items"]) > 1
    root_last = max(t["kv_begin"] for t in before["tasks"] if t["node"] == 0)
    bad = f.node_len.copy()
    bad[0] = root_last                              # the root's last slice would be empty
    assert C.codec_plan_refresh_lengths(plan, bad, paged.node_page_off, paged.page_ids) == C.CODEC_ERR_INVALID_ARGUMENT
    zero = f.node_len.copy()
    zero[1] = 0
    assert C.codec_plan_refresh_lengths(plan, zero, paged.node_page_off, paged.page_ids) == C.CODEC_ERR_INVALID_TREE
    longer = f.node_len.copy()
    longer[2] += 64                                 # pages of the old layout do not cover it
    assert C.codec_plan_refresh_lengths(plan, longer, paged.node_page_off, paged.page_ids) == C.CODEC_ERR_INVALID_TREE
    assert C.codec_plan_refresh_lengths(None, f.node_len, paged.node_page_off, paged.page_ids) == C.CODEC_ERR_INVALID_ARGUMENT
    _, after = C.codec_plan_export(plan)
    assert after["tasks"] == before["tasks"] and after["makespan"] == before["makespan"]
    C.codec_plan_destroy(plan)


@pytest.mark.parametrize("name", sorted(FORESTS))
@pytest.mark.parametrize("fixed", [1, 2, 7, 64])
def test_fixed_slice_count_matches_oracle(name, fixed):
    f = FORESTS[name]()
    head = HeadConfig(32, 8, 128, 1)
    m, align, max_rows = 16, 64, 64
    table = _default_table(1)
    paged = build_paged_kv(f, head, seed=1)
    st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                   head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                   head.page_size, head.scale, m, align, max_rows, 1, _tuple(table),
                                   fixed_slices=fixed)
    assert st == C.CODEC_OK
    st, view = C.codec_plan_export(plan)
    C.codec_plan_destroy(plan)
    _compare(view, P.plan(f.parent, f.node_len, f.req_node, 4, m, align, max_rows, True, table, fixed_slices=fixed))


# ---- share = 2: best of the candidate plans ------------------------------------------------------

BEST_CASES = {
    # heavy sharing: the 256-row plan wins
    "docqa": (lambda: two_level_forest(20000, [64] * 48), HeadConfig(32, 8, 128, 1)),
    # a quarter of every context shared: the long private leaves decide, small row tiles or flat win
    "quarter": (lambda: two_level_forest(30720, [92160] * 16), HeadConfig(32, 8, 128, 1)),
    "nothing": (lambda: unshared_forest([40000] * 12), HeadConfig(32, 8, 128, 1)),
    "random": (lambda: random_forest(60, 5, 2.0, 512, 1.0, 16, 32768, seed=8), HeadConfig(64, 8, 128, 1)),
    "mha": (lambda: three_level_forest(2048, [8192] * 4, 5, [37 + 13 * i for i in range(20)]), HeadConfig(8, 8, 128, 0)),
}


# A table under which tasks of more than 16 rows are dear (as on a device without a fast wide kernel):
# cost = len * rows for up to 16 rows, forty times that above.  It makes the candidates with small row
# tiles, or the flat plan, win where the built-in tables pick the 256-row plan.
DEAR_WIDE = {"row_grid": [1, 16, 17, 256], "len_grid": [32, 65536],
             "cost": [[32 * 1, 65536 * 1], [32 * 16, 65536 * 16], [32 * 17 * 40, 65536 * 17 * 40],
                      [32 * 256 * 40, 65536 * 256 * 40]]}


@pytest.mark.parametrize("table", ["builtin", "dear_wide"])
@pytest.mark.parametrize("name", sorted(BEST_CASES))
def test_best_candidate_plan_matches_oracle(name, table):
    make, head = BEST_CASES[name]
    f = make()
    group = head.num_q_heads // head.num_kv_heads
    paged = build_paged_kv(f, head, seed=1)
    custom = None if table == "builtin" else DEAR_WIDE
    st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                   head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                   head.page_size, head.scale, share=2,
                                   cost_table=_tuple(custom) if custom else None)
    assert st == C.CODEC_OK
    st, view = C.codec_plan_export(plan)
    C.codec_plan_destroy(plan)
    tables = ({"narrow": _default_table(0), "wide": _default_table(1)} if custom is None
              else {"narrow": custom, "wide": custom})
    ref = P.plan_best(f.parent, f.node_len, f.req_node, group, 256, 256, tables,
                      lambda wide: (256 if wide else 512) // head.num_kv_heads)
    assert (view["share"], view["max_rows"]) == (int(ref["share"]), ref["max_rows"])
    _compare(view, ref)
    if name == "docqa" and custom is None:
        assert (view["share"], view["max_rows"]) == (1, 256)
    if name in ("docqa", "quarter", "random") and custom is not None:
        assert (view["share"], view["max_rows"]) != (1, 256)


# ---- run-time queue (schedule = 1): structure of the entries ---------------------------------------

@pytest.mark.parametrize("name", sorted(BEST_CASES))
@pytest.mark.parametrize("slots", [0, 4])
def test_run_time_queue_entries(name, slots):
    """The queue holds every task once; an entry of several tasks holds short ones only (at most 16 rows
    and 2048 tokens, at most 4 of them); entries come in order of decreasing cost (a bundle counts as the
    sum of its tasks); when the tasks that are not short leave workgroups free, the bundles are just
    large enough for every entry to have a workgroup of its own."""
    make, head = BEST_CASES[name]
    f = make()
    group = head.num_q_heads // head.num_kv_heads
    paged = build_paged_kv(f, head, seed=1)
    st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                   head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                   head.page_size, head.scale, num_slots=slots, schedule=1)
    assert st == C.CODEC_OK
    st, v = C.codec_plan_export(plan)
    C.codec_plan_destroy(plan)
    assert v["schedule"] == 1
    off, q, tasks = list(v["queue_off"]), list(v["queue_tasks"]), v["tasks"]
    assert sorted(q) == list(range(len(tasks))) and off[0] == 0 and off[-1] == len(tasks)
    short = [t["n_req"] * group <= 16 and t["kv_len"] <= 2048 for t in tasks]
    costs = []
    for e in range(len(off) - 1):
        members = q[off[e]:off[e + 1]]
        assert 1 <= len(members) <= 4
        if len(members) > 1:
            assert all(short[i] for i in members)
        costs.append(sum(tasks[i]["cost"] for i in members))
    assert costs == sorted(costs, reverse=True)
    n_long = short.count(False)
    m = v["num_slots"]
    if n_long < m and -(-short.count(True) // (m - n_long)) <= 4:
        assert len(off) - 1 <= m


def test_half_width_row_tiles_match_oracle():
    """share = 2 with an explicit max_rows: the candidate with row tiles of half that width exists and wins
    where the oracle says so (the hand-worked case of the oracle's pins, through the library)."""
    f = Forest(np.array([-1]), np.array([100]), np.zeros(64, dtype=np.int32))
    head = HeadConfig(2, 2, 128, 0)
    paged = build_paged_kv(f, head, seed=1)
    prop = {"row_grid": [1, 65], "len_grid": [1, 101], "cost": [[1, 101], [65, 6565]]}
    for slots, want_rows in ((2, 32), (1, 64)):
        st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                       head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                       head.page_size, head.scale, num_slots=slots, split_align=256,
                                       max_rows=64, share=2, cost_table=_tuple(prop))
        assert st == C.CODEC_OK
        st, view = C.codec_plan_export(plan)
        C.codec_plan_destroy(plan)
        ref = P.plan_best(f.parent, f.node_len, f.req_node, 1, 256, 64, {"narrow": prop, "wide": prop},
                          lambda wide: slots)
        assert (view["share"], view["max_rows"]) == (1, want_rows) == (int(ref["share"]), ref["max_rows"])
        _compare(view, ref)


def test_schedule_option_is_checked():
    f = two_level_forest(100, [5, 9])
    head = HeadConfig(8, 8, 128, 0)
    paged = build_paged_kv(f, head, seed=1)
    for bad in (3, -1):
        st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                       head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                       head.page_size, head.scale, schedule=bad)
        assert st == C.CODEC_ERR_INVALID_ARGUMENT and plan is None
    for bad in (4, -1):
        st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                       head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                       head.page_size, head.scale, extensions=bad)
        assert st == C.CODEC_ERR_INVALID_ARGUMENT and plan is None



@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4", "cfg5c"])
def test_automatic_schedule_follows_the_entry_count(name):
    """schedule = 2 resolves to the run-time queue from six entries per slot on, to the static
    schedule below; everything else in the plan is the same in the three modes."""
    f, head = config_forest(name), config_head(name)
    paged = build_paged_kv(f, head, seed=1)
    views = {}
    for schedule in (0, 1, 2):
        st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                       head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                       head.page_size, head.scale, schedule=schedule)
        assert st == C.CODEC_OK
        st, views[schedule] = C.codec_plan_export(plan)
        C.codec_plan_destroy(plan)
    entries = len(views[2]["queue_off"]) - 1
    assert views[0]["schedule"] == 0 and views[1]["schedule"] == 1
    assert views[2]["schedule"] == (1 if entries >= 6 * views[2]["num_slots"] else 0)
    assert views[2]["schedule"] == {"cfg2": 0, "cfg3": 0, "cfg4": 1, "cfg5c": 0}[name]
    for key in ("tasks", "slot_off", "slot_tasks", "queue_off", "queue_tasks", "makespan"):
        assert _same(views[0][key], views[2][key]) and _same(views[1][key], views[2][key]), key


def _same(a, b):
    if isinstance(a, list):
        return a == b
    return np.array_equal(np.asarray(a), np.asarray(b))


def test_single_launch_option():
    """fused = 2 resolves by the estimated makespan (40 us with the built-in tables) and the number of query
    rows per KV head (at most 64); 3 and -1 are refused."""
    picked = {}
    for name in ("cfg1", "cfg2", "cfg3", "cfg5c"):
        f, head = config_forest(name), config_head(name)
        paged = build_paged_kv(f, head, seed=1)
        for fused in (0, 1, 2):
            st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                           head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                           head.page_size, head.scale, fused=fused, extensions=3)
            assert st == C.CODEC_OK
            st, v = C.codec_plan_export(plan)
            C.codec_plan_destroy(plan)
            if fused < 2:
                assert v["fused"] == fused
            else:
                small = f.num_requests * (head.num_q_heads // head.num_kv_heads) <= 64
                assert v["fused"] == (1 if v["makespan"] < 40000 and small else 0)
                picked[name] = v["fused"]
    assert picked == {"cfg1": 1, "cfg2": 0, "cfg3": 0, "cfg5c": 0}
    f, head = config_forest("cfg1"), config_head("cfg1")
    paged = build_paged_kv(f, head, seed=1)
    for bad in (3, -1):
        st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                       head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                                       head.page_size, head.scale, fused=bad)
        assert st == C.CODEC_ERR_INVALID_ARGUMENT and plan is None


# ---- visibility masks (multi-token decoding) ------------------------------------------------------

def _masked_nodes(f):
    return {int(f.req_node[r]) for r in range(f.num_requests) if f.req_mask_off[r + 1] > f.req_mask_off[r]}


@pytest.mark.parametrize("share", [1, 0])
@pytest.mark.parametrize("hq,hkv,drafted", [(32, 8, 64), (8, 8, 5), (16, 1, 33), (12, 4, 40)])
def test_plans_with_visibility_masks_match_oracle(share, hq, hkv, drafted):
    """A node that ends masked requests gets row tiles of at most 16 rows and stays whole; everything
    else is planned as ever.  Bit-exact against the re-derivation, for the printed solver and both extensions."""
    f = draft_masked_forest(700, [3000, 45, 1200, 9000], drafted, seed=4)
    head = HeadConfig(hq, hkv, 128)
    paged = build_paged_kv(f, head, seed=1)
    for ext in (0, 3):
        st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                       hq, hkv, 128, head.dtype, head.page_size, head.scale, 16, 64, 0, share,
                                       extensions=ext, req_mask_off=f.req_mask_off, req_mask=f.req_mask)
        assert st == C.CODEC_OK, C.codec_status_string(st)
        st, view = C.codec_plan_export(plan)
        C.codec_plan_destroy(plan)
        wide = max(it["rows"] for it in view["items"]) > 16
        ref = P.plan(f.parent, f.node_len, f.req_node, head.group, 16, 64, 256, bool(share), _default_table(wide),
                     slack=bool(ext & 1), diagonal=bool(ext & 2), masked_nodes=_masked_nodes(f))
        _compare(view, ref)
        for it in view["items"]:
            if it["node"] in _masked_nodes(f):
                assert it["rows"] <= 16 and it["b"] == 1


def test_malformed_masks_are_rejected():
    f = draft_masked_forest(0, [100], 40, seed=2)          # two words per drafted request
    head = HeadConfig(8, 2, 128)
    paged = build_paged_kv(f, head, seed=1)

    def create(off, words, hq=8, hkv=2):
        return C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                   hq, hkv, 128, head.dtype, head.page_size, head.scale,
                                   req_mask_off=off, req_mask=words)[0]
    assert create(f.req_mask_off, f.req_mask) == C.CODEC_OK
    short = f.req_mask_off.copy()
    short[2:] -= 1                                           # request 1 is left with one word for 40 tokens
    assert create(short, f.req_mask[1:]) == C.CODEC_ERR_INVALID_TREE
    blind = f.req_mask.copy()
    blind[0:2] = 0                                           # request 1 sees none of its node's tokens
    assert create(f.req_mask_off, blind) == C.CODEC_ERR_INVALID_TREE
    beyond = f.req_mask.copy()
    beyond[0:2] = [0, 1 << 20]                               # only a bit past the node's 40 tokens is set
    assert create(f.req_mask_off, beyond) == C.CODEC_ERR_INVALID_TREE
    shifted = f.req_mask_off + 1
    assert create(shifted, np.concatenate([[0], f.req_mask])) == C.CODEC_ERR_INVALID_TREE
    assert create(f.req_mask_off, f.req_mask, hq=64, hkv=2) == C.CODEC_ERR_UNSUPPORTED      # group 32 > 16


def test_refresh_keeps_masked_nodes_as_they_are():
    f = draft_masked_forest(0, [100, 60], 8, seed=2)
    head = HeadConfig(8, 2, 128)
    paged = build_paged_kv(f, head, seed=1)
    st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                                   8, 2, 128, head.dtype, head.page_size, head.scale,
                                   req_mask_off=f.req_mask_off, req_mask=f.req_mask)
    assert st == C.CODEC_OK
    grown = f.node_len.copy()
    grown[0] += 5                                            # a context grows: fine
    g = Forest(f.parent, grown, f.req_node)
    gp = build_paged_kv(g, head, seed=1)
    assert C.codec_plan_refresh_lengths(plan, grown, gp.node_page_off, gp.page_ids) == C.CODEC_OK
    grown[1] += 1                                            # a drafted-token node grows: its masks no longer fit
    g = Forest(f.parent, grown, f.req_node)
    gp = build_paged_kv(g, head, seed=1)
    assert C.codec_plan_refresh_lengths(plan, grown, gp.node_page_off, gp.page_ids) == C.CODEC_ERR_INVALID_ARGUMENT
    C.codec_plan_destroy(plan)


# ---- head dimensions 64 and 256: capped row tiles, the narrow kernel variant's table and slot count ----
@pytest.mark.parametrize("head_dim", [64, 256])
@pytest.mark.parametrize("name", ["docqa", "three", "random", "binary"])
@pytest.mark.parametrize("hq,hkv", [(32, 8), (8, 8), (16, 1)])
@pytest.mark.parametrize("share", [1, 0, 2])
def test_other_head_dimensions_plan(head_dim, name, hq, hkv, share):
    """With 64 (256) channels a task holds at most 32 (16) rows whatever max_rows asks for, and the plan
    takes the slot count and cost table of the kernel variant that runs such tasks."""
    f = FORESTS[name]()
    head = HeadConfig(hq, hkv, head_dim)
    group = hq // hkv
    view = _lib_plan(f, head, 0, 0, 0, share, None, 3)
    cap = max(group, P.max_task_rows(head_dim) // group * group)
    assert max(t["n_req"] * group for t in view["tasks"]) <= cap
    m = 512 // hkv
    assert view["num_slots"] == m
    if share == 2:
        tables = {"narrow": _default_table(0), "wide": _default_table(1)}
        ref = P.plan_best(f.parent, f.node_len, f.req_node, group, 256, 256, tables, lambda wide: (256 if wide else 512) // hkv,
                          slack=True, diagonal=True, head_dim=head_dim)
        assert (view["share"], view["max_rows"]) == (int(ref["share"]), ref["max_rows"])
    else:
        ref = P.plan(f.parent, f.node_len, f.req_node, group, m, 256, cap, bool(share), _default_table(0),
                     slack=True, diagonal=True)
    _compare(view, ref)
