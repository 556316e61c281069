"""Integer re-derivation of the workload balancer.  TEST INFRASTRUCTURE ONLY.

Follows Sec. 5 of the paper: per-node cost from a profiled table with
interpolation (Sec. 5.2, Eq. 6-7), no split along the query dimension beyond a
row-tile cap (Sec. 5.1 fixes b_q = 1; the cap is this build's addition for
query sets that do not fit one workgroup), a lower bound cost_l of the makespan
found by binary search on the average-load inequality (Eq. 4), the per-node
upper bound on the number of KV slices (Eq. 5), a grid search over each node's
slice count, and greedy longest-first scheduling onto m slots (Eq. 3).

With ``slack`` and ``diagonal`` off (the defaults) this is the solver of Sec.
5.1 as printed: b_k <= ceil(C_est / cost_l) (Eq. 5) and one node-by-node pass
of the grid search.  The two flags mirror the library's extensions, which are
not in the paper:
``slack``: a node whose cost is at least a quarter of cost_l may take one slice
more than the quotient of Eq. 5 (64 contexts of 0.4 average loads each on 32
slots: two per slot, or three); every other node keeps the printed bound.
``diagonal``: after the pass, nine more points of the grid are evaluated (every
node at its Eq. 5 quotient for a common target cost_l * (1 + k/8), k = 0 .. 8,
capped by its bound) and the best point seen is kept.

The paper gives the solver in prose; where it is silent this file fixes:
integer costs; round-half-up bilinear interpolation, clamped below the grid
and linearly extrapolated above it; slice boundaries on multiples of
``align`` tokens with equal-length slices except the last; the grid search as
one pass node by node, in order of decreasing node cost with ties to the
smaller slice count; ties in the schedule to the lower slot id.
Python integers are unbounded, so no intermediate can overflow.
"""
from __future__ import annotations

import heapq
from typing import Dict, List, Sequence


def _ceil_div(a: int, b: int) -> int:
    return -((-a) // b)


def locate(grid: Sequence[int], x: int):
    """Bracket x on an ascending grid -> (i0, i1, num, den); weight of i1 is num/den."""
    k = len(grid)
    if k == 1 or x <= grid[0]:
        return 0, 0, 0, 1
    if x >= grid[k - 1]:
        return k - 2, k - 1, x - grid[k - 2], grid[k - 1] - grid[k - 2]
    i = 0
    while grid[i + 1] <= x:
        i += 1
    return i, i + 1, x - grid[i], grid[i + 1] - grid[i]


def c_est(table: Dict, rows: int, n: int) -> int:
    """C_est(rows, n): estimated cost of one partial attention task (Eq. 6)."""
    r0, r1, ar, dr = locate(table["row_grid"], rows)
    n0, n1, an, dn = locate(table["len_grid"], n)
    c = table["cost"]
    num = ((dr - ar) * (dn - an) * c[r0][n0] + ar * (dn - an) * c[r1][n0]
           + (dr - ar) * an * c[r0][n1] + ar * an * c[r1][n1])
    den = dr * dn
    if num <= 0:
        return 1
    return max(1, (num + den // 2) // den)


def slices(n: int, b: int, align: int):
    """Cut n tokens into about b slices on multiples of align -> (count, length, last length)."""
    length = align * _ceil_div(_ceil_div(n, b), align)
    count = _ceil_div(n, length)
    return count, length, n - (count - 1) * length


def division_cost(table, rows: int, n: int, b: int, align: int) -> int:
    count, length, last = slices(n, b, align)
    return (count - 1) * c_est(table, rows, length) + c_est(table, rows, last)


def lpt(sub: List[tuple], m: int):
    """Greedy longest-first schedule of (cost, item, chunk) onto m slots.

    Returns (makespan, slot of each subtask in input order, per-slot lists of
    input indices in assignment order).
    """
    order = sorted(range(len(sub)), key=lambda i: (-sub[i][0], sub[i][1], sub[i][2]))
    heap = [(0, s) for s in range(m)]
    slot_of = [0] * len(sub)
    lists: List[List[int]] = [[] for _ in range(m)]
    for i in order:
        load, s = heapq.heappop(heap)
        slot_of[i] = s
        lists[s].append(i)
        heapq.heappush(heap, (load + sub[i][0], s))
    return max(l for l, _ in heap), slot_of, lists


def build_index(parent, node_len, req_node):
    """Prefix paths (root first) and per-node ascending request lists; validates the forest."""
    n_nodes = len(parent)
    for i in range(n_nodes):
        if not (-1 <= parent[i] < n_nodes) or parent[i] == i:
            raise ValueError("bad parent")
        if node_len[i] < 1:
            raise ValueError("empty node")
    paths, node_q = [], [[] for _ in range(n_nodes)]
    for r, leaf in enumerate(req_node):
        if not (0 <= leaf < n_nodes):
            raise ValueError("bad req_node")
        p, n = [], int(leaf)
        while n != -1:
            if len(p) >= n_nodes:
                raise ValueError("cycle")
            p.append(n)
            n = int(parent[n])
        p.reverse()
        paths.append(p)
        for n in p:
            node_q[n].append(r)
    return paths, node_q


def plan(parent, node_len, req_node, group: int, num_slots: int, align: int,
         max_rows: int, share: bool, table: Dict, fixed_slices: int = 0,
         slack: bool = False, diagonal: bool = False, masked_nodes=()) -> Dict:
    """``masked_nodes``: nodes that end a request with a visibility mask (Sec. 4.1).  The library runs
    masks in its 16-row task shape only, so such a node gets row tiles of at most 16 rows and is not
    divided along KV (its bound and slice count are 1)."""
    masked_nodes = set(int(n) for n in masked_nodes)
    parent = [int(x) for x in parent]
    node_len = [int(x) for x in node_len]
    req_node = [int(x) for x in req_node]
    m = num_slots
    paths, node_q = build_index(parent, node_len, req_node)
    n_nodes = len(parent)

    node_q_off = [0]
    node_q_flat: List[int] = []
    for n in range(n_nodes):
        node_q_flat += node_q[n]
        node_q_off.append(len(node_q_flat))

    # work items: (node, request range); a flat plan gives every request its own item
    qpt_all = max(1, max_rows // group) if share else 1
    qpt_of = [min(qpt_all, max(1, 16 // group)) if n in masked_nodes else qpt_all for n in range(n_nodes)]
    items = []
    first_item_of_node = [0] * n_nodes
    for n in range(n_nodes):
        first_item_of_node[n] = len(items)
        nq = len(node_q[n])
        qpt = qpt_of[n]
        for a in range(0, nq, qpt):
            cnt = min(qpt, nq - a)
            items.append({"node": n, "q_off": node_q_off[n] + a, "n_req": cnt,
                          "rows": cnt * group, "len": node_len[n]})
    for it in items:
        it["cost"] = c_est(table, it["rows"], it["len"])
        it["max_b"] = 1 if it["node"] in masked_nodes else _ceil_div(it["len"], align)

    def b_of(it, T):
        return min(_ceil_div(it["cost"], T), it["max_b"])

    def ok(T):
        tot = sum(division_cost(table, it["rows"], it["len"], b_of(it, T), align) for it in items)
        return tot <= m * T

    cost_l = 0
    if items:
        lo = 1
        hi = max(max(it["cost"] for it in items),
                 _ceil_div(sum(it["cost"] for it in items), m))
        while lo < hi:
            mid = (lo + hi) // 2
            if ok(mid):
                hi = mid
            else:
                lo = mid + 1
        cost_l = lo

    for it in items:
        want = b_of(it, cost_l)                                   # Eq. 5: the quotient
        if slack and 4 * it["cost"] >= cost_l:
            want = min(want + 1, it["max_b"])                     # extension: one slice over the printed bound
        it["ub"] = slices(it["len"], want, align)[0]
        it["b"] = it["ub"]

    def subtasks():
        sub = []
        for j, it in enumerate(items):
            count, length, last = slices(it["len"], it["b"], align)
            for c in range(count):
                ln = length if c < count - 1 else last
                sub.append((c_est(table, it["rows"], ln), j, c, c * length, ln))
        return sub

    order = sorted((j for j in range(len(items)) if items[j]["ub"] > 1),
                   key=lambda j: (-items[j]["cost"], j))
    if fixed_slices > 0:
        # the naive strategy the paper compares with (impact of division granularity): the same
        # slice count for every node, no bound, no search
        order = []
        for it in items:
            it["b"] = slices(it["len"], min(fixed_slices, it["max_b"]), align)[0]
    for j in order:
        it = items[j]
        best_b, best_ms, seen = None, None, set()
        for b in range(1, it["ub"] + 1):
            count = slices(it["len"], b, align)[0]
            if count in seen:
                continue
            seen.add(count)
            it["b"] = count
            ms = lpt(subtasks(), m)[0]
            if best_ms is None or ms < best_ms:
                best_b, best_ms = count, ms
        it["b"] = best_b

    if diagonal and fixed_slices == 0 and items:
        # extension: the pass above moves one node at a time; the search also looks along the diagonal of the grid:
        # every node at its Eq. 5 quotient for one common target cost_l * (1 + k/8), k = 0 .. 8, capped by
        # its bound; the best point seen is kept (ties: the earlier one)
        best_ms = lpt(subtasks(), m)[0]
        best_bs = [it["b"] for it in items]
        for k in range(9):
            target = max(1, cost_l + cost_l * k // 8)
            for it in items:
                it["b"] = slices(it["len"], min(it["ub"], b_of(it, target)), align)[0]
            ms = lpt(subtasks(), m)[0]
            if ms < best_ms:
                best_ms, best_bs = ms, [it["b"] for it in items]
        for it, b in zip(items, best_bs):
            it["b"] = b

    sub = subtasks()
    makespan, slot_of, lists = lpt(sub, m) if sub else (0, [], [[] for _ in range(m)])

    tasks = []
    base = 0
    first_task_of_item = []
    for i, (cost, j, c, kv_begin, kv_len) in enumerate(sub):
        it = items[j]
        if c == 0:
            first_task_of_item.append(i)
        tasks.append({"item": j, "node": it["node"], "kv_begin": kv_begin, "kv_len": kv_len,
                      "q_off": it["q_off"], "n_req": it["n_req"], "part_row_base": base,
                      "cost": cost, "slot": slot_of[i]})
        base += it["rows"]

    slot_off, slot_tasks = [0], []
    for s in range(m):
        slot_tasks += lists[s]
        slot_off.append(len(slot_tasks))

    req_part_off, req_part = [0], []
    for r, p in enumerate(paths):
        for n in p:
            qi = node_q[n].index(r)
            qpt = qpt_of[n]
            j = first_item_of_node[n] + qi // qpt
            it = items[j]
            t0 = first_task_of_item[j]
            for c in range(it["b"]):
                req_part.append(tasks[t0 + c]["part_row_base"] + (qi % qpt) * group)
        req_part_off.append(len(req_part))

    return {"items": items, "cost_l": cost_l, "tasks": tasks, "makespan": makespan,
            "slot_off": slot_off, "slot_tasks": slot_tasks,
            "node_q_off": node_q_off, "node_q": node_q_flat,
            "req_part_off": req_part_off, "req_part": req_part,
            "part_rows": base, "paths": paths}


def refresh(plan_out: Dict, table: Dict, new_node_len) -> Dict:
    """Carry a plan over to new node lengths without dividing or scheduling again.

    The paper divides tasks only every few decoding steps (Implementation section, task division
    module) while every step appends a token to each request's last node.  Between two plannings the division and the
    slot assignment are kept: a node's slices keep their boundaries, its last slice takes up the
    change in length, costs and the makespan are re-estimated for the new lengths.  Returns a new
    dict with the same keys as ``plan``; raises ValueError when a last slice would become empty.
    """
    new_node_len = [int(x) for x in new_node_len]
    out = dict(plan_out)
    items = [dict(it) for it in plan_out["items"]]
    tasks = [dict(t) for t in plan_out["tasks"]]
    first = {}
    for i, t in enumerate(tasks):
        first.setdefault(t["item"], i)
    for j, it in enumerate(items):
        n = new_node_len[it["node"]]
        b = it["b"]
        t0 = first[j]
        start = tasks[t0 + b - 1]["kv_begin"]
        if n < 1 or n - start < 1:
            raise ValueError("node %d: length %d leaves its last slice empty" % (it["node"], n))
        it["len"] = n
        it["cost"] = c_est(table, it["rows"], n)
        last = tasks[t0 + b - 1]
        last["kv_len"] = n - start
        last["cost"] = c_est(table, it["rows"], last["kv_len"])
    m = len(plan_out["slot_off"]) - 1
    loads = [sum(tasks[i]["cost"] for i in plan_out["slot_tasks"][plan_out["slot_off"][s]:plan_out["slot_off"][s + 1]])
             for s in range(m)]
    out["items"], out["tasks"] = items, tasks
    out["makespan"] = max(loads) if loads else 0
    return out


def max_task_rows(head_dim: int) -> int:
    """Most rows of a task: the dense task shape (up to 256 rows, the wide kernel variant) exists for
    128 channels; the stream shape holds 32 rows of 64 channels and 16 of 256."""
    return {128: 256, 64: 32, 256: 16}[head_dim]


def plan_best(parent, node_len, req_node, group: int, align: int, max_rows: int, tables: Dict,
              num_slots_of, slack: bool = False, diagonal: bool = False, masked_nodes=(),
              head_dim: int = 128) -> Dict:
    """share = 2 of the library: the candidate with the lowest estimated makespan, ties to the earlier.

    Candidates: the prefix-shared plan with row tiles of ``max_rows``; with row tiles of half that (if
    more than 16 rows); with row tiles of at most 16 rows (query-dimension splits, b_q > 1 in the terms
    of Sec. 5.1); the flat plan.
    ``tables`` = {"narrow": .., "wide": ..} and ``num_slots_of(wide)`` give each candidate the table and
    slot count of the kernel variant its widest task selects, as the library does (the wide variant
    exists for 128 channels; with 64 or 256 the row tiles are capped by max_task_rows).
    """
    cap = max(group, max_task_rows(head_dim) // group * group)      # every candidate's row tiles
    cands = [(True, max_rows)]
    half = max_rows // 2 // group * group
    if half > 16 and half >= group:
        cands.append((True, half))
    small = 16 // group * group if group <= 16 else 0
    if small >= group and small < max_rows:
        cands.append((True, small))
    cands.append((False, max_rows))
    best = None
    for share, rows in cands:
        rows = min(rows, cap)
        paths, node_q = build_index([int(x) for x in parent], [int(x) for x in node_len], [int(x) for x in req_node])
        qpt_all = max(1, rows // group) if share else 1
        tile = [min(qpt_all, max(1, 16 // group)) if n in set(masked_nodes) else qpt_all for n in range(len(node_q))]
        widest = max((min(tile[n], len(q) - a) * group for n, q in enumerate(node_q)
                      for a in range(0, len(q), tile[n])), default=0)
        wide = widest > 16 and head_dim == 128
        p = plan(parent, node_len, req_node, group, num_slots_of(wide), align, rows, share,
                 tables["wide" if wide else "narrow"], slack=slack, diagonal=diagonal, masked_nodes=masked_nodes)
        p["share"], p["max_rows"] = share, rows
        if best is None or p["makespan"] < best["makespan"]:
            best = p
    return best
