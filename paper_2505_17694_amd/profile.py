"""Cost-table profiler: measures C_est(rows, len) of the partial-attention kernel on this GPU.

The planner balances work with a profiled table (paper Sec. 5.2: run the
partial attention kernel over a grid of query counts and KV lengths on the
target GPU, record the block execution time, interpolate in between).  One
measurement here is one launch in which every workgroup slot of one KV head
runs exactly one task of the given shape, all slots and heads at once, so the
number is the time of a workgroup under the load the plan will see.  K/V pools
are rotated so that consecutive launches do not find their data in cache.

Two tables are measured because the kernel has two launch variants: "narrow"
(only tasks of at most 16 rows; 4 waves per workgroup, two workgroups per CU)
and "wide" (any task; 8 waves, one workgroup per CU).

The K/V pools are laid out [page][kv_head][token][d]: a (page, head) is one contiguous 4 KB run.

    python -m paper_2505_17694_amd.profile            # writes the package's cost_table_mi355x.json

The build turns that file into the library's built-in tables (build.py: generate_cost_tables), so a
rebuild after profiling is all it takes for the planner to use the new numbers.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys

import numpy as np

FLOOR_NS = 200.0
DEFAULT_OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cost_table_mi355x.json")


def _forest(num_tasks, rows, length, force_wide):
    """`num_tasks` independent nodes of `length` tokens, `rows` requests ending at each (group = 1)."""
    parent = [-1] * num_tasks
    node_len = [length] * num_tasks
    req_node = [n for n in range(num_tasks) for _ in range(rows)]
    if force_wide:          # one tiny 17-row node makes the plan pick the wide kernel variant; it shares a
                            # slot with other tasks and its few microseconds cancel in measure()
        parent.append(-1)
        node_len.append(32)
        req_node += [num_tasks] * 17
    return np.array(parent, np.int32), np.array(node_len, np.int32), np.array(req_node, np.int32)


class _Case:
    """One profiling launch shape: every slot of every KV head runs `per_slot` (rows, length) tasks."""

    def __init__(self, rows: int, length: int, wide: bool, per_slot: int, device: str = "cuda:0"):
        import torch
        from . import binding as B
        from .runtime import PlannedAttention

        class Bag:
            pass

        h_kv, d, ps = 8, 128, 16
        slots = 32 if wide else 64
        force = wide and rows <= 16
        parent, node_len, req_node = _forest(slots * per_slot, rows, length, force)
        forest, paged, head = Bag(), Bag(), Bag()
        forest.parent, forest.node_len, forest.req_node = parent, node_len, req_node
        pages_per = (node_len.astype(np.int64) + ps - 1) // ps
        off = np.zeros(len(parent) + 1, np.int64)
        np.cumsum(pages_per, out=off[1:])
        paged.node_page_off = off.astype(np.int32)
        paged.num_pages = int(off[-1])
        rng = np.random.Generator(np.random.PCG64(rows * 1000003 + length))
        paged.page_ids = rng.permutation(paged.num_pages).astype(np.int32)
        # [page][kv_head][token][d]: a (page, head) is one contiguous 4 KB run
        paged.page_stride, paged.token_stride, paged.head_stride = ps * h_kv * d, d, ps * d
        head.num_q_heads = head.num_kv_heads = h_kv
        head.head_dim, head.dtype, head.page_size, head.scale = d, B.CODEC_DTYPE_BF16, ps, 1.0 / math.sqrt(d)

        pool_elems = paged.num_pages * ps * h_kv * d
        copies = max(1, min(16, int((2 << 30) // max(1, 4 * pool_elems))))
        gen = torch.Generator(device=device)
        gen.manual_seed(1)
        self.q = torch.randn((len(req_node), h_kv, d), device=device, generator=gen).to(torch.bfloat16)
        self.pools = [(torch.randn(pool_elems, device=device, generator=gen).to(torch.bfloat16),
                       torch.randn(pool_elems, device=device, generator=gen).to(torch.bfloat16)) for _ in range(copies)]
        # a flat table keeps the planner from dividing: one task per node, one node per slot
        flat = ([1], [1], [[1000]])
        self.pa = PlannedAttention(forest, paged, head, device=device, num_slots=slots,
                                   split_align=32, max_rows=256, share=1, cost_table=flat)
        view = self.pa.export()
        assert len(view["tasks"]) == len(parent), "the profiling plan must not divide nodes"
        per = np.bincount([t["slot"] for t in view["tasks"]][:slots * per_slot], minlength=slots)
        assert per.max() == per_slot, "every slot must get the same number of tasks"
        self.turn = 0
        self.stream = torch.cuda.current_stream()
        for _ in range(2):
            self.launch()

    def launch(self):
        """One launch of the partial-attention kernel on the next pool copy -> (start, end) events."""
        import torch
        k, v = self.pools[self.turn % len(self.pools)]
        self.turn += 1
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(self.stream)
        self.pa.partial_attention(self.q, k, v)
        b.record(self.stream)
        return a, b

    def close(self):
        self.pa.close()


def measure(rows: int, length: int, wide: bool, pairs: int = 12) -> float:
    """Cost (ns) of one (rows, length) task inside a busy persistent workgroup.

    The difference between a launch with three tasks per slot and one with one task per slot, halved:
    launch latency and the ramp at both ends of a launch drop out.  The two launches alternate (`pairs`
    times) so that clock and temperature drift hits both alike; the median difference is returned.
    """
    import torch
    one, three = _Case(rows, length, wide, 1), _Case(rows, length, wide, 3)
    ev = [(one.launch(), three.launch()) for _ in range(pairs)]
    torch.cuda.synchronize()
    diffs = sorted(c[0].elapsed_time(c[1]) - a[0].elapsed_time(a[1]) for a, c in ev)
    one.close()
    three.close()
    return max(diffs[len(diffs) // 2] * 1e6 / 2.0, 1.0)


def profile(row_grid, len_grid, wide: bool, verbose: bool = True):
    cost = []
    for r in row_grid:
        row = []
        for n in len_grid:
            # the difference of two launches cannot resolve a task that a wave runs in the shadow of the
            # others: no task is priced below FLOOR_NS (a record read and a partial row written)
            ns = max(measure(r, n, wide), FLOOR_NS)
            row.append(int(round(ns)))
            if verbose:
                print(f"[profile] {'wide' if wide else 'narrow'} rows={r:4d} len={n:6d}: {ns / 1e3:9.2f} us",
                      file=sys.stderr, flush=True)
        cost.append(row)
    return {"row_grid": list(row_grid), "len_grid": list(len_grid), "cost": cost}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=DEFAULT_OUT, help="'' = print only")
    ap.add_argument("--lens", default="32,128,512,2048,8192,32768")
    ap.add_argument("--wide-rows", default="1,16,17,32,64,128,256")
    ap.add_argument("--narrow-rows", default="1,16")
    args = ap.parse_args()
    lens = [int(x) for x in args.lens.split(",")]
    tables = {"unit": "ns per workgroup, every slot busy",
              "narrow": profile([int(x) for x in args.narrow_rows.split(",")], lens, wide=False),
              "wide": profile([int(x) for x in args.wide_rows.split(",")], lens, wide=True)}
    text = json.dumps(tables, indent=1)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text + "\n")
    print(text)


if __name__ == "__main__":
    main()
