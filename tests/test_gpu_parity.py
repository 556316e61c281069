"""GPU parity: the HIP path through the C ABI against the fp64 definition oracle.

Bar (both sides on the same 16-bit-rounded inputs): max |out - oracle| <= 1e-2,
the bound the build is held to for fp16/bf16 I/O with fp32 accumulation.  A
tighter mixed bar (2e-3 + 2^-7 |oracle|) is asserted as well; it is what the
arithmetic supports: P is rounded to 16 bits before the second product and the
output is rounded once to 16 bits (relative 2^-9 for bf16), everything else is
fp32.
"""
import numpy as np
import pytest
import torch

from oracle import attention as A
from workloads import (HeadConfig, Forest, make_workload, make_small_config, make_config,
                       two_level_forest, three_level_forest, unshared_forest, random_forest,
                       concat_forests, degenerate_forest, draft_tree_forest, draft_masked_forest,
                       DTYPE_FP16, DTYPE_BF16)

pytestmark = pytest.mark.gpu

TOL = 1e-2


def _C():
    import paper_2505_17694_amd as C
    return C


def run_gpu(w, share=1, **opts):
    C = _C()
    wd = w.to("cuda:0")
    pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", share=share, **opts)
    out = pa.decode(wd.q, wd.k_pool, wd.v_pool)
    torch.cuda.synchronize()
    res = out.to(torch.float64).cpu().numpy()
    view = pa.export()
    pa.close()
    return res, view


def check(w, share=1, sel=None, **opts):
    print(f"[case] {w.name} share={share} opts={opts} B={w.forest.num_requests} "
          f"nodes={w.forest.num_nodes} heads={w.head.num_q_heads}/{w.head.num_kv_heads}", flush=True)
    got, view = run_gpu(w, share, **opts)
    if sel is None:
        ref, _ = A.decode_attention_workload(w)
        g = got
    else:
        ref, _ = A.decode_attention_workload(w, sel=sel)
        g = np.stack([got[r, h] for r, h in sel])
    assert not np.any(np.isnan(g)), "NaN in the output (a masked position leaked?)"
    err = np.abs(g - ref)
    assert err.max() <= TOL, f"max abs err {err.max():.3e}"
    assert np.all(err <= 2e-3 + 2.0 ** -7 * np.abs(ref)), f"mixed bar: worst {err.max():.3e}"
    return got, view


@pytest.mark.parametrize("name,shrink,req_shrink", [
    ("cfg1", 4, 1), ("cfg2", 8, 2), ("cfg3", 16, 2), ("cfg4", 8, 8),
    ("cfg5a", 64, 4), ("cfg5b", 64, 8), ("cfg5c", 64, 8)])
@pytest.mark.parametrize("share", [1, 0])
def test_shrunken_configurations(name, shrink, req_shrink, share):
    w = make_small_config(name, shrink, req_shrink, poison=True)
    check(w, share=share)


@pytest.mark.parametrize("lens", [[1], [15], [16], [17], [31], [32], [33], [63, 64, 65], [127, 129, 1, 2]])
@pytest.mark.parametrize("dtype", [DTYPE_FP16, DTYPE_BF16])
def test_ragged_single_nodes(lens, dtype):
    """Lengths around the 16-token tile and the 32-token block; waves that get no block at all."""
    w = make_workload(f"ragged{lens}", unshared_forest(lens), HeadConfig(8, 2, 128, dtype), seed=5, poison=True)
    check(w)


@pytest.mark.parametrize("hq,hkv", [(8, 8), (4, 1), (28, 4), (16, 2), (64, 1)])
def test_head_layouts(hq, hkv):
    """MHA, MQA and GQA groups 7, 8 and 64 (rows per request not a divisor of the 16-row tile)."""
    f = three_level_forest(70, [130, 45], 3, [5, 33, 64, 1, 17, 48])
    w = make_workload(f"heads{hq}/{hkv}", f, HeadConfig(hq, hkv, 128, DTYPE_BF16), seed=8, poison=True)
    check(w)
    check(w, share=0)


@pytest.mark.parametrize("d", [64, 256])
@pytest.mark.parametrize("case", ["cfg2", "cfg3", "ragged", "mha-drafted-masked", "mqa", "queue-fused", "flat-fp16",
                                  "group2", "group6"])
def test_other_head_dimensions(d, case):
    """64 and 256 channels per head: the stream task shape only (row tiles of at most 32 and 16 rows,
    whatever max_rows asks for), every plan option, masks, the single-launch mode and the reduction kernel (groups
    of 1, 2, 3 and 6 heads take its one-row form with 64 channels, groups of 4, 8 and 16 four rows a wave)."""
    if case in ("group2", "group6"):
        g = int(case[5:])
        f, hq, hkv, dtype, opts = three_level_forest(50, [70, 33], 2, [9, 40, 1, 130]), 2 * g, 2, DTYPE_BF16, {}
    elif case == "cfg2":
        f, hq, hkv, dtype, opts = make_small_config("cfg2", 8, 2).forest, 32, 8, DTYPE_BF16, {}
    elif case == "cfg3":
        f, hq, hkv, dtype, opts = make_small_config("cfg3", 16, 2).forest, 32, 8, DTYPE_BF16, {"extensions": 3}
    elif case == "ragged":
        f, hq, hkv, dtype, opts = unshared_forest([1, 15, 16, 17, 31, 33, 63, 65, 127, 129, 1030]), 8, 2, DTYPE_FP16, \
            {"num_slots": 3, "split_align": 32}
    elif case == "mha-drafted-masked":
        f, hq, hkv, dtype, opts = draft_masked_forest(300, [900, 33, 260], 40, seed=5), 8, 8, DTYPE_BF16, {"fused": 1}
    elif case == "mqa":
        f, hq, hkv, dtype, opts = three_level_forest(70, [130, 45], 3, [5, 33, 64, 1, 17, 48]), 16, 1, DTYPE_BF16, \
            {"max_rows": 200}
    elif case == "queue-fused":
        f, hq, hkv, dtype, opts = random_forest(30, 4, 2.0, 200, 1.0, 1, 3000, seed=7), 12, 4, DTYPE_BF16, \
            {"schedule": 1, "fused": 1, "num_slots": 2, "split_align": 64}
    else:
        f, hq, hkv, dtype, opts = two_level_forest(2100, [40, 90, 33, 7]), 8, 2, DTYPE_FP16, {"share": 0}
    w = make_workload(f"d{d}-{case}", f, HeadConfig(hq, hkv, d, dtype), seed=600 + d, poison=True,
                      layout="htd" if d == 64 else "thd")
    _, view = check(w, **opts)
    assert max(t["n_req"] * (hq // hkv) for t in view["tasks"]) <= (32 if d == 64 else 16)


@pytest.mark.parametrize("hq,hkv,requests", [(8, 2, 5), (8, 2, 7), (8, 2, 8), (4, 4, 17), (4, 4, 31), (4, 4, 33), (12, 4, 10)])
@pytest.mark.parametrize("dtype", [DTYPE_BF16, DTYPE_FP16])
def test_two_row_tiles_with_64_channels(hq, hkv, requests, dtype):
    """Tasks of 17 .. 32 rows of 64 channels (two row tiles per wave): 20, 28, 32, 17, 31, 30 rows and a
    33-row set that splits into 32 + 1; ragged nodes of one block and of many, long enough for a team of
    waves and short enough for runs of single-wave tasks beside them."""
    f = two_level_forest(1500, [1 + 37 * (i % 4) for i in range(requests)])
    f = concat_forests(concat_forests(f, two_level_forest(33, [20] * requests)), unshared_forest([70, 2100, 5]))
    w = make_workload(f"d64-rows-{hq}-{hkv}-{requests}", f, HeadConfig(hq, hkv, 64, dtype), seed=640 + requests, poison=True,
                      layout="htd")
    for opts in ({}, {"num_slots": 2, "split_align": 32}, {"fused": 1}, {"schedule": 1, "num_slots": 3}):
        _, view = check(w, **opts)
        rows = [t["n_req"] * (hq // hkv) for t in view["tasks"]]
        assert max(rows) <= 32 and max(rows) > 16


@pytest.mark.parametrize("max_rows", [8, 16, 32, 48, 64, 100, 128, 200, 256])
def test_row_tiles(max_rows):
    """70 requests x group 4 = 280 rows under the root: stream and dense task shapes, row tiling."""
    f = two_level_forest(300, [7 + (i % 5) for i in range(70)])
    w = make_workload(f"rows{max_rows}", f, HeadConfig(16, 4, 128, DTYPE_BF16), seed=12, poison=True)
    _, view = check(w, max_rows=max_rows)
    assert max(t["n_req"] * 4 for t in view["tasks"]) <= max_rows


@pytest.mark.parametrize("requests", [5, 16, 17, 32, 33, 64])
def test_dense_tasks_of_every_block_count(requests):
    """One undivided task per root, 20 .. 256 rows: 1 .. 70 blocks of 32 tokens, odd and even counts,
    counts around the depth of the block ring, ragged last blocks; from 1024 tokens on, the two waves of
    a row group take alternate blocks in tasks of at most 128 rows, so the odd-block wave may have one
    block less than the other."""
    lens = [1, 33, 65, 96, 200, 256, 257, 289, 300, 330, 353, 511, 545, 577, 1023, 1024, 1025, 1090, 1290, 1312,
            1345, 2210]
    f = two_level_forest(lens[0], [43] * requests)
    for n in lens[1:]:
        f = concat_forests(f, two_level_forest(n, [40 + n % 4] * requests))      # private suffixes: stream path
    w = make_workload(f"dense{requests}", f, HeadConfig(8, 2, 128, DTYPE_BF16), seed=31 + requests, poison=True)
    _, view = check(w, num_slots=3, split_align=4096)
    roots = [t for t in view["tasks"] if t["n_req"] == requests]
    assert sorted(t["kv_len"] for t in roots) == lens


@pytest.mark.parametrize("slots,align", [(1, 32), (7, 32), (64, 32), (64, 64), (256, 32)])
def test_division_granularity(slots, align):
    """From everything on one slot to slices of a single block: merged result must not change."""
    f = concat_forests(two_level_forest(2100, [40, 90, 33]), unshared_forest([700, 31]))
    w = make_workload(f"div{slots}/{align}", f, HeadConfig(8, 2, 128, DTYPE_FP16), seed=3, poison=True)
    _, view = check(w, num_slots=slots, split_align=align)
    if slots >= 64:
        assert max(it["b"] for it in view["items"]) > 4


@pytest.mark.parametrize("layout,page_size", [("htd", 16), ("thd", 32), ("htd", 64), ("thd", 128),
                                              ("hktd", 16), ("hktd", 32)])
def test_layouts_and_page_sizes(layout, page_size):
    f = three_level_forest(200, [333, 90], 2, [5, 70, 130, 17])
    head = HeadConfig(8, 2, 128, DTYPE_BF16, page_size=page_size)
    w = make_workload(f"{layout}{page_size}", f, head, seed=21, poison=True, layout=layout)
    check(w, split_align=max(32, page_size), num_slots=16)


def test_irregular_forest_with_internal_requests():
    f = random_forest(48, 5, 2.0, 100, 1.0, 1, 3000, seed=17)
    inner = [int(f.parent[n]) for n in f.req_node[:6] if f.parent[n] >= 0]
    f = Forest(f.parent, f.node_len, np.concatenate([f.req_node, np.array(inner, dtype=np.int32)]))
    w = make_workload("irregular", f, HeadConfig(32, 8, 128, DTYPE_BF16), seed=4, poison=True)
    check(w, num_slots=16, split_align=32)
    check(w, share=0, num_slots=16, split_align=32)


def test_degenerate_tree():
    w = make_workload("spine", degenerate_forest(6, 500, 60), HeadConfig(8, 2, 128, DTYPE_FP16), seed=2, poison=True)
    check(w, num_slots=8, split_align=32)


def test_large_logits_and_peaked_softmax():
    """Q scaled by 8: logits of order +-90, outputs of order 1; LSE merging must stay stable."""
    f = two_level_forest(1500, [64, 200, 31, 7])
    w = make_workload("stress", f, HeadConfig(8, 2, 128, DTYPE_BF16), seed=9, poison=True, q_scale=8.0)
    got, _ = check(w, num_slots=32, split_align=32)
    assert np.abs(got).max() > 0.5


def test_request_order_permutation_is_equivariant():
    f = two_level_forest(600, [33, 70, 5, 128, 90])
    w = make_workload("perm", f, HeadConfig(8, 2, 128, DTYPE_BF16), seed=13)
    base, _ = run_gpu(w, num_slots=8, split_align=32)
    perm = np.array([3, 0, 4, 1, 2])
    f2 = Forest(f.parent, f.node_len, f.req_node[perm])
    w2 = make_workload("perm2", f2, w.head, seed=13, paged=w.paged)
    w2.q[:] = w.q[torch.from_numpy(perm)]
    w2.k_pool[:] = w.k_pool
    w2.v_pool[:] = w.v_pool
    got, _ = check(w2, num_slots=8, split_align=32)
    # same tasks on the shared root up to row order; each request's own rows see identical arithmetic
    assert np.max(np.abs(got - base[perm])) <= 2.0 ** -7 * np.abs(base).max()


def test_same_plan_decodes_repeatedly_and_with_new_queries():
    C = _C()
    w = make_small_config("cfg2", 8, 2, poison=True)
    wd = w.to("cuda:0")
    pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0")
    a = pa.decode(wd.q, wd.k_pool, wd.v_pool).clone()
    b = pa.decode(wd.q, wd.k_pool, wd.v_pool).clone()
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))      # bit-identical replays
    w.q[:] = torch.randn(w.q.shape, generator=torch.Generator().manual_seed(5)).to(w.q.dtype)
    out = pa.decode(w.q.to("cuda:0"), wd.k_pool, wd.v_pool)
    torch.cuda.synchronize()
    ref, _ = A.decode_attention_workload(w)
    assert np.max(np.abs(out.double().cpu().numpy() - ref)) <= TOL
    pa.close()


@pytest.mark.parametrize("share,schedule", [(1, 0), (0, 0), (1, 1)])
def test_plan_carried_over_to_grown_lengths(share, schedule):
    """codec_plan_refresh_lengths: same division and schedule, longer last slices, new page lists (and, for
    the run-time queue, entries ordered by the new costs and counters back at zero)."""
    C = _C()
    f_old = three_level_forest(700, [1300, 450], 3, [5, 33, 64, 1, 17, 48])
    head = HeadConfig(16, 4, 128, DTYPE_BF16)
    rng = np.random.Generator(np.random.PCG64(3))
    growth = rng.integers(0, 40, size=f_old.num_nodes).astype(np.int32)
    growth[-1] = 1                                          # the usual decode step: one more token
    f_new = Forest(f_old.parent, f_old.node_len + growth, f_old.req_node)
    w_new = make_workload("grown", f_new, head, seed=31, poison=True)
    w_old = make_workload("before", f_old, head, seed=31, paged=w_new.paged)
    w_old.q[:] = w_new.q
    w_old.k_pool[:] = w_new.k_pool
    w_old.v_pool[:] = w_new.v_pool
    wd = w_new.to("cuda:0")
    pa = C.PlannedAttention(f_old, w_new.paged, head, device="cuda:0", share=share, num_slots=4 if schedule else 16,
                            split_align=32, schedule=schedule)
    tasks_before = pa.export()["tasks"]
    for w, lens in ((w_old, None), (w_new, f_new.node_len)):
        if lens is not None:
            pa.refresh(lens)
        out = pa.decode(wd.q, wd.k_pool, wd.v_pool)
        torch.cuda.synchronize()
        ref, _ = A.decode_attention_workload(w)
        got = out.to(torch.float64).cpu().numpy()
        assert not np.any(np.isnan(got))
        assert np.abs(got - ref).max() <= TOL
    tasks_after = pa.export()["tasks"]
    assert [(t["kv_begin"], t["slot"]) for t in tasks_after] == [(t["kv_begin"], t["slot"]) for t in tasks_before]
    assert sum(t["kv_len"] for t in tasks_after) > sum(t["kv_len"] for t in tasks_before)
    pa.close()


def test_best_candidate_plan_on_the_gpu():
    """share = 2 on a forest where private leaves dominate and on one where the shared root does."""
    low = two_level_forest(960, [2900, 3100, 2800, 3000])
    high = two_level_forest(6000, [40] * 24)
    head = HeadConfig(32, 8, 128, DTYPE_BF16)
    picked = []
    for i, f in enumerate((low, high)):
        w = make_workload(f"best{i}", f, head, seed=40 + i, poison=True)
        _, view = check(w, share=2)
        picked.append((view["share"], view["max_rows"]))
    assert picked[1] == (1, 256)


@pytest.mark.parametrize("slots,expect", [(2, 1), (64, 0)])
def test_automatic_schedule_on_the_gpu(slots, expect):
    """schedule = 2: with two slots the forest below has far more than six queue entries per slot and
    runs from the queue, with 64 slots it stays on the static lists; both against the oracle."""
    f = random_forest(40, 4, 2.0, 300, 1.0, 8, 4000, seed=77)
    w = make_workload(f"auto{slots}", f, HeadConfig(16, 4, 128, DTYPE_BF16), seed=78, poison=True)
    _, view = check(w, schedule=2, num_slots=slots, split_align=64)
    assert view["schedule"] == expect, (view["schedule"], len(view["queue_off"]) - 1, view["num_slots"])


@pytest.mark.parametrize("slots", [1, 3])
@pytest.mark.parametrize("upside_down", [False, True])
def test_many_short_tasks_per_slot(slots, upside_down):
    """Long runs of single-wave tasks in a slot's list, before, between and behind team and dense tasks.

    With the upside-down cost table short tasks count as the most expensive, so longest-first
    scheduling puts them in front of the long ones; lengths around the single-wave limit (2048) and
    request counts around the 16-row limit mix the three task shapes in every slot.
    """
    lens = [7, 40, 2048, 33, 2049, 64, 300, 5, 3000, 96, 17, 1000, 31, 640, 1, 129] * 3
    f = concat_forests(two_level_forest(1500, lens), two_level_forest(200, [50, 60, 70, 80, 90]))
    head = HeadConfig(8, 2, 128, DTYPE_BF16)                    # group 4: the 5-request root has 20 rows
    w = make_workload(f"short{slots}", f, head, seed=23, poison=True)
    table = ([1, 256], [1, 4096], [[5000, 100], [6000, 200]]) if upside_down else None
    _, view = check(w, num_slots=slots, split_align=32, cost_table=table)
    per_slot = np.bincount([t["slot"] for t in view["tasks"]], minlength=slots)
    assert per_slot.max() >= 16


def test_limits_of_the_interface():
    """Largest page size (4096 tokens), largest GQA group (64: four requests fill a 256-row task), and a
    context of a million tokens divided over every slot (sampled outputs: the oracle needs seconds per pair)."""
    head = HeadConfig(8, 2, 128, DTYPE_BF16, page_size=4096)
    w = make_workload("page4096", two_level_forest(5000, [4097, 100, 4096]), head, seed=51, poison=True)
    check(w, split_align=4096, num_slots=4)
    head = HeadConfig(64, 1, 128, DTYPE_FP16)
    w = make_workload("group64", two_level_forest(700, [33, 5, 90, 64, 17]), head, seed=52, poison=True)
    _, view = check(w, num_slots=8, split_align=32)
    assert max(t["n_req"] * 64 for t in view["tasks"]) == 256
    head = HeadConfig(8, 8, 128, DTYPE_BF16)
    w = make_workload("million", unshared_forest([1 << 20]), head, seed=53, device="cuda:0")
    C = _C()
    pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0")
    out = pa.decode(w.q, w.k_pool, w.v_pool)
    torch.cuda.synchronize()
    view = pa.export()
    pa.close()
    assert len(view["tasks"]) >= view["num_slots"]
    sel = [(0, 0), (0, 5)]
    ref, _ = A.decode_attention_workload(w, sel=sel)
    got = np.stack([out[r, h].to(torch.float64).cpu().numpy() for r, h in sel])
    assert np.abs(got - ref).max() <= TOL


@pytest.mark.parametrize("schedule,fused", [(0, 0), (1, 0), (0, 1), (1, 1)])
def test_decode_replayed_from_a_hip_graph(schedule, fused):
    """The decode call is two kernel launches on the caller's stream and nothing else, so it can be
    captured; every replay (with eager work and new queries in between) must equal the eager result.
    With the run-time queue, and in single-launch mode (fused = 1: one launch, the reduction inside it),
    the kernel itself puts its counters back (no memset node)."""
    C = _C()
    w = make_small_config("cfg3", 16, 2, poison=True)
    wd = w.to("cuda:0")
    pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", schedule=schedule, fused=fused)
    q = wd.q.clone()
    out = torch.empty_like(q)
    pa.decode(q, wd.k_pool, wd.v_pool, out)                         # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pa.decode(q, wd.k_pool, wd.v_pool, out)
    gen = torch.Generator(device="cuda:0").manual_seed(9)
    for i in range(4):
        q.copy_(torch.randn(q.shape, device="cuda:0", generator=gen).to(q.dtype))      # eager work in between
        graph.replay()
        torch.cuda.synchronize()
        replayed = out.clone()
        eager = pa.decode(q, wd.k_pool, wd.v_pool)
        torch.cuda.synchronize()
        assert torch.equal(replayed.view(torch.int16), eager.view(torch.int16)), f"replay {i}"
    w.q[:] = q.cpu()
    ref, _ = A.decode_attention_workload(w)
    assert np.abs(out.double().cpu().numpy() - ref).max() <= TOL
    pa.close()


@pytest.mark.parametrize("seed", range(24))
def test_random_forests_heads_and_plan_options(seed):
    """Seeded draws over tree shape, head layout, dtype, page size and layout, and every plan option
    (slot count, slice alignment, row tile, plan kind, schedule): each against the oracle."""
    rng = np.random.Generator(np.random.PCG64(4000 + seed))
    leaves = int(rng.integers(1, 40))
    f = random_forest(leaves, int(rng.integers(1, 6)), float(rng.uniform(0.3, 3.0)),
                      int(rng.choice([20, 120, 600])), float(rng.uniform(0.3, 1.4)), 1,
                      int(rng.choice([200, 1500, 5000])), seed=500 + seed)
    if rng.random() < 0.3:                                    # some requests end at inner nodes
        inner = [int(f.parent[n]) for n in f.req_node[:4] if f.parent[n] >= 0]
        f = Forest(f.parent, f.node_len, np.concatenate([f.req_node, np.array(inner, dtype=np.int32)]))
    hq, hkv = [(8, 8), (8, 2), (32, 8), (12, 4), (16, 1), (64, 8), (6, 3)][int(rng.integers(0, 7))]
    dtype = DTYPE_BF16 if rng.random() < 0.6 else DTYPE_FP16
    page_size = int(rng.choice([16, 32, 64]))
    layout = "htd" if rng.random() < 0.5 else "thd"
    head = HeadConfig(hq, hkv, 128, dtype, page_size=page_size)
    w = make_workload(f"random{seed}", f, head, seed=900 + seed, poison=True, layout=layout)
    opts = {"num_slots": int(rng.choice([0, 1, 5, 17])),
            "split_align": int(rng.choice([1, 2, 8])) * max(32, page_size),
            "max_rows": int(rng.choice([0, 0, 16, 64, 128, 200])),
            "schedule": int(rng.integers(0, 2)), "extensions": int(rng.integers(0, 4)),
            "fused": int(rng.integers(0, 2))}
    if opts["max_rows"] and opts["max_rows"] < hq // hkv:
        opts["max_rows"] = 0
    check(w, share=int(rng.choice([1, 1, 0, 2])), **opts)


@pytest.mark.parametrize("drafted,hq,hkv,share,schedule", [
    (1, 8, 2, 1, 0), (7, 32, 8, 1, 0), (24, 32, 8, 1, 1), (24, 8, 8, 2, 0), (40, 16, 1, 1, 0), (12, 32, 8, 0, 0)])
def test_drafted_token_trees(drafted, hq, hkv, share, schedule):
    """Multi-token decoding: verification of tree-structured drafts.  Every drafted token is a node
    of one token, a request ends at every one of them and at the context they hang from, so what a
    query may see is its path (the visibility of the streaming softmax of Sec. 4.2 reduces to the
    tree).  Inner nodes carry requests, nodes are as short as they get, and many requests share
    the one-token nodes near the context."""
    f = draft_tree_forest(300, [900, 33, 2100, 260], drafted, seed=70 + drafted)
    assert f.num_requests == 4 * (drafted + 1)
    w = make_workload(f"drafted{drafted}", f, HeadConfig(hq, hkv, 128, DTYPE_BF16), seed=71 + drafted, poison=True)
    check(w, share=share, schedule=schedule)


@pytest.mark.parametrize("drafted,hq,hkv,opts", [
    (1, 8, 2, {}), (7, 32, 8, {}), (24, 32, 8, {"schedule": 1}), (24, 8, 8, {"share": 2}),
    (40, 16, 1, {"fused": 1}), (33, 32, 8, {"share": 0}), (64, 32, 8, {"extensions": 3}),
    (70, 12, 4, {"num_slots": 3, "split_align": 32}), (100, 16, 4, {"schedule": 1, "fused": 1})])
def test_masked_draft_nodes(drafted, hq, hkv, opts):
    """Multi-token decoding with visibility masks (Sec. 4.1): the drafted tokens of a sequence sit in one
    node, every drafted token's query ends there and sees itself and the drafted tokens before it on
    its branch.  1 .. 100 drafted tokens: one to four mask words per query, partly filled last words,
    row tiles of one to sixteen requests, tasks run by a wave alone and by the workgroup."""
    f = draft_masked_forest(300, [900, 33, 2100, 260], drafted, seed=170 + drafted)
    assert f.num_requests == 4 * (drafted + 1)
    dtype = DTYPE_BF16 if drafted % 2 else DTYPE_FP16
    w = make_workload(f"masked{drafted}", f, HeadConfig(hq, hkv, 128, dtype), seed=171 + drafted, poison=True)
    _, view = check(w, **opts)
    ends = {int(f.req_node[r]) for r in range(f.num_requests) if f.visible(r) is not None}
    assert all(it["rows"] <= 16 and it["b"] == 1 for it in view["items"] if it["node"] in ends)


def test_masks_that_hide_whole_blocks_and_long_masked_nodes():
    """A masked node of 700 tokens (22 blocks), queries that see a single token each, at the front, in the
    middle, at the very end: whole 32-token blocks with nothing visible, before and after the first
    visible one; a query whose mask is all ones; a request without a mask ending at the same node."""
    n = 700
    words = (n + 31) // 32
    picks = [[0], [699], [350], [31, 32], [5, 690], list(range(n)), [64 + i for i in range(40)]]
    masks = []
    for vis in picks:
        m = [0] * words
        for t in vis:
            m[t // 32] |= 1 << (t % 32)
        masks.append(m)
    masks.append([])                                        # the last request sees the whole node
    off = np.zeros(len(masks) + 1, dtype=np.int32)
    np.cumsum([len(m) for m in masks], out=off[1:])
    f = Forest(np.array([-1, 0]), np.array([90, n]), np.full(len(masks), 1), off,
               np.array([x for m in masks for x in m], dtype=np.uint32))
    w = make_workload("sparse-masks", f, HeadConfig(8, 4, 128, DTYPE_BF16), seed=77, poison=True)
    check(w)
    check(w, num_slots=1, schedule=1)


@pytest.mark.parametrize("slices", [1, 6, 7, 8, 14, 15, 16, 23, 40])
def test_reduction_lists_of_every_length(slices):
    """A request's partial rows number slices + 1 or slices + 2 here (root cut evenly, one or two leaf
    slices): 2, 7 .. 10, 15 .. 18, 24, 25, 41, 42 over the cases.  The reduction kernel reads the first
    eight rows and the count from one line per request, rows nine to fifteen from the same line, and
    lists of sixteen and more from the CSR arrays: every boundary is hit from both sides."""
    f = two_level_forest(32 * slices * 3, [33, 7, 64])
    w = make_workload(f"parts{slices}", f, HeadConfig(8, 2, 128, DTYPE_BF16), seed=300 + slices, poison=True)
    got, view = check(w, num_slots=5, split_align=32, fixed_slices=slices)
    lens = {int(view["req_part_off"][r + 1] - view["req_part_off"][r]) for r in range(3)}
    assert lens == ({2} if slices == 1 else {slices + 1, slices + 2}), lens


def _queue_cases():
    short = [7, 40, 2048, 33, 2049, 64, 300, 5, 3000, 96, 17, 1000, 31, 640, 1, 129] * 3
    dense = two_level_forest(1, [43] * 17)
    for n in [33, 300, 545, 1024, 1090, 2210]:
        dense = concat_forests(dense, two_level_forest(n, [40 + n % 4] * 17))
    return {
        "cfg2": (lambda: make_small_config("cfg2", 8, 2, poison=True), {}),
        "cfg3": (lambda: make_small_config("cfg3", 16, 2, poison=True), {}),
        "cfg4": (lambda: make_small_config("cfg4", 8, 8, poison=True), {}),
        "cfg5c": (lambda: make_small_config("cfg5c", 64, 8, poison=True), {}),
        "cfg3-flat": (lambda: make_small_config("cfg3", 16, 2, poison=True), {"share": 0}),
        "short-1-slot": (lambda: make_workload("q-short", concat_forests(two_level_forest(1500, short),
                                                                         two_level_forest(200, [50, 60, 70, 80, 90])),
                                               HeadConfig(8, 2, 128, DTYPE_BF16), seed=23, poison=True),
                         {"num_slots": 1, "split_align": 32}),
        "short-3-slots": (lambda: make_workload("q-short3", two_level_forest(1500, short),
                                                HeadConfig(8, 2, 128, DTYPE_BF16), seed=24, poison=True),
                          {"num_slots": 3, "split_align": 32}),
        "dense-2-slots": (lambda: make_workload("q-dense", dense, HeadConfig(8, 2, 128, DTYPE_BF16), seed=25,
                                                poison=True), {"num_slots": 2, "split_align": 4096}),
        "more-slots-than-entries": (lambda: make_workload("q-few", two_level_forest(100, [5, 9]),
                                                          HeadConfig(8, 8, 128, DTYPE_FP16), seed=26, poison=True),
                                    {"num_slots": 64}),
        "mqa-one-head": (lambda: make_workload("q-mqa", three_level_forest(70, [130, 45], 3, [5, 33, 64, 1, 17, 48]),
                                               HeadConfig(4, 1, 128, DTYPE_BF16), seed=27, poison=True), {}),
    }


@pytest.mark.parametrize("name", sorted(_queue_cases()))
def test_run_time_queue_equals_the_static_schedule(name):
    """schedule = 1 runs the same tasks, writes the same partial rows and merges them in the same order as
    the static schedule; what differs is the workgroup that runs a task and whether a short task is
    run by one wave or by a team (which changes the order of its fp32 sums).  Every launch is held
    against the oracle with both bars of this file, and the launches of the queue against each other bit
    for bit (the kernel leaves the queue's counters at zero behind it; which workgroup takes which entry
    changes no task's own arithmetic)."""
    C = _C()
    make, opts = _queue_cases()[name]
    w = make()
    wd = w.to("cuda:0")
    static = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", **opts)
    queued = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", schedule=1, **opts)
    view = queued.export()
    assert view["schedule"] == 1
    want = static.decode(wd.q, wd.k_pool, wd.v_pool).double().cpu().numpy()
    ref, _ = A.decode_attention_workload(w)
    assert np.all(np.abs(want - ref) <= 2e-3 + 2.0 ** -7 * np.abs(ref))
    outs = []
    for launch in range(3):
        got = queued.decode(wd.q, wd.k_pool, wd.v_pool)
        torch.cuda.synchronize()
        outs.append(got.clone())
        g = got.double().cpu().numpy()
        assert not np.any(np.isnan(g)), f"launch {launch}"
        assert np.abs(g - ref).max() <= TOL, f"launch {launch}: {np.abs(g - ref).max():.3e}"
        assert np.all(np.abs(g - ref) <= 2e-3 + 2.0 ** -7 * np.abs(ref)), f"launch {launch}: mixed bar"
    # partial attention alone, twice in a row, then the reduction: the counters do not depend on the
    # reduction kernel
    queued.partial_attention(wd.q, wd.k_pool, wd.v_pool)
    queued.partial_attention(wd.q, wd.k_pool, wd.v_pool)
    out = torch.empty_like(wd.q)
    queued.partial_reduction(out)
    torch.cuda.synchronize()
    outs.append(out)
    for i, o in enumerate(outs[1:]):
        assert torch.equal(o.view(torch.int16), outs[0].view(torch.int16)), f"launch {i + 1} differs from launch 0"
    static.close()
    queued.close()


def _fused_cases():
    cases = dict(_queue_cases())
    cases["cfg1"] = (lambda: make_small_config("cfg1", 4, 1, poison=True), {})
    cases["cfg5a"] = (lambda: make_small_config("cfg5a", 64, 4, poison=True), {})
    cases["drafted"] = (lambda: make_workload("f-drafted", draft_tree_forest(300, [900, 33, 2100, 260], 24, seed=94),
                                               HeadConfig(32, 8, 128, DTYPE_BF16), seed=95, poison=True), {})
    cases["long-lists"] = (lambda: make_workload("f-lists", two_level_forest(32 * 23 * 3, [33, 7, 64]),
                                                  HeadConfig(8, 2, 128, DTYPE_BF16), seed=96, poison=True),
                           {"num_slots": 5, "split_align": 32, "fixed_slices": 23})
    return cases


@pytest.mark.parametrize("schedule", [0, 1])
@pytest.mark.parametrize("name", sorted(_fused_cases()))
def test_single_launch_equals_two_launches(name, schedule):
    """fused = 1: the workgroup that delivers a request's last partial result reduces the request inside
    the attention launch.  The reduction folds the same rows in the same order as the reduction kernel,
    so the output equals the two-launch output bit for bit, launch after launch (the arrival counters
    are back at zero after every launch), whichever workgroup happens to be last; and it is held against
    the oracle with both bars of this file."""
    C = _C()
    make, opts = _fused_cases()[name]
    w = make()
    wd = w.to("cuda:0")
    two = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", schedule=schedule, **opts)
    one = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", schedule=schedule, fused=1, **opts)
    assert one.export()["fused"] == 1 and two.export()["fused"] == 0
    want = two.decode(wd.q, wd.k_pool, wd.v_pool)
    torch.cuda.synchronize()
    ref, _ = A.decode_attention_workload(w)
    for launch in range(3):
        got = torch.full_like(wd.q, float("nan"))
        one.decode(wd.q, wd.k_pool, wd.v_pool, got)
        torch.cuda.synchronize()
        g = got.double().cpu().numpy()
        assert not np.any(np.isnan(g)), f"launch {launch}: a request was never reduced"
        assert np.abs(g - ref).max() <= TOL, f"launch {launch}: {np.abs(g - ref).max():.3e}"
        assert np.all(np.abs(g - ref) <= 2e-3 + 2.0 ** -7 * np.abs(ref)), f"launch {launch}: mixed bar"
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), f"launch {launch} differs from two launches"
    # the two phase calls of a fused plan stay separate and leave the counters alone
    out = torch.empty_like(wd.q)
    one.partial_attention(wd.q, wd.k_pool, wd.v_pool)
    one.partial_reduction(out)
    got = one.decode(wd.q, wd.k_pool, wd.v_pool)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), want.view(torch.int16))
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    one.close()
    two.close()


def test_tree_equals_flat_on_the_gpu():
    w = make_small_config("cfg3", 16, 2, poison=True)
    tree, _ = run_gpu(w, share=1)
    flat, _ = run_gpu(w, share=0)
    assert np.max(np.abs(tree - flat)) <= TOL


def test_error_paths_on_the_device_side():
    C = _C()
    w = make_small_config("cfg1", 4, 1)
    wd = w.to("cuda:0")
    pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0")
    p = w.paged
    out = torch.empty_like(wd.q)
    args = (wd.q.data_ptr(), wd.k_pool.data_ptr(), wd.v_pool.data_ptr())
    ws = pa.workspace
    # pool smaller than the largest page id, workspace too small, misaligned query pointer
    assert C.codec_decode_attention(pa.plan, *args, 3, p.page_stride, p.token_stride, p.head_stride,
                                    out.data_ptr(), ws.data_ptr(), ws.numel()) == C.CODEC_ERR_INVALID_ARGUMENT
    assert C.codec_decode_attention(pa.plan, *args, p.num_pages, p.page_stride, p.token_stride, p.head_stride,
                                    out.data_ptr(), ws.data_ptr(), 16) == C.CODEC_ERR_WORKSPACE_TOO_SMALL
    assert C.codec_decode_attention(pa.plan, args[0] + 2, args[1], args[2], p.num_pages, p.page_stride,
                                    p.token_stride, p.head_stride, out.data_ptr(), ws.data_ptr(),
                                    ws.numel()) == C.CODEC_ERR_INVALID_ARGUMENT
    pa.close()


def test_cost_table_profiler_agrees_with_the_built_in_table():
    """The profiler that writes the built-in table, on two grid points of the wide variant (a stream
    task and a dense task): what it measures on this machine is within 25 % of what the library plans with."""
    C = _C()
    from paper_2505_17694_amd import profile
    row_grid, len_grid, cost = C.codec_default_cost_table(1)
    for rows, length in ((16, 2048), (256, 2048)):
        got = profile.measure(rows, length, wide=True)
        want = cost[row_grid.index(rows)][len_grid.index(length)]
        print(f"[case] profiler rows={rows} len={length}: measured {got:.0f} ns, table {want} ns", flush=True)
        assert 0.75 * want <= got <= 1.25 * want, (rows, length, got, want)


# ---- full-size configurations, in the launch configuration the benchmark times -------------------

def _sample_pairs(w, n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    B, H = w.forest.num_requests, w.head.num_q_heads
    idx = rng.choice(B * H, size=min(n, B * H), replace=False)
    return [(int(i // H), int(i % H)) for i in idx]


# what bench.py times: layout "htd"; the prefix-shared plan with both planner extensions ("tree", the
# headline), the solver of Sec. 5.1 as printed, the flat plan, the run-time queue, the library's own
# choice of plan and schedule
BENCH_VARIANTS = [
    {"share": 1, "schedule": 0, "extensions": 3},
    {"share": 1, "schedule": 0, "extensions": 0},
    {"share": 0, "schedule": 0, "extensions": 0},
    {"share": 1, "schedule": 1, "extensions": 3},
    {"share": 2, "schedule": 2, "extensions": 3, "fused": 2},
    {"share": 1, "schedule": 0, "extensions": 3, "fused": 1},
]


@pytest.mark.parametrize("name,layout,n_pairs", [
    ("cfg1", "htd", 10 ** 9), ("cfg2", "htd", 10 ** 9), ("cfg3", "htd", 10 ** 9), ("cfg4", "htd", 10 ** 9),
    ("cfg5a", "htd", 10 ** 9), ("cfg5b", "htd", 10 ** 9), ("cfg5c", "htd", 10 ** 9),
    ("cfg3", "thd", 1024), ("cfg4", "hktd", 1024)])
def test_full_size_configurations(name, layout, n_pairs):
    """Inputs are generated on the GPU and copied back for the oracle.  In the benchmark's layout every
    (request, head) pair of every configuration is compared (the oracle needs about ten seconds for
    the largest); the other two layouts are sampled."""
    w = make_config(name, device="cuda:0", layout=layout)
    C = _C()
    print(f"[case] full {name} {layout} unique_kv_bytes={w.unique_kv_bytes}", flush=True)
    sel = _sample_pairs(w, n_pairs, seed=77)
    ref, _ = A.decode_attention_workload(w, sel=sel)
    print(f"[case] full {name} {layout}: oracle done on {len(sel)} pairs", flush=True)
    for opts in BENCH_VARIANTS:
        pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", **opts)
        out = pa.decode(w.q, w.k_pool, w.v_pool)
        torch.cuda.synchronize()
        got = out.to(torch.float64).cpu().numpy()
        pa.close()
        g = np.stack([got[r, h] for r, h in sel])
        err = np.abs(g - ref)
        print(f"[case] full {name} {layout} {opts} max_err={err.max():.3e}", flush=True)
        assert not np.any(np.isnan(got))
        assert err.max() <= TOL
        assert np.all(err <= 2e-3 + 2.0 ** -7 * np.abs(ref))


@pytest.mark.parametrize("sweep,point", [("draft_masked", "drafted=64"), ("draft", "drafted=16"), ("batch", "requests=64"),
                                         ("depth", "levels=6"), ("shape", "DT"), ("ratio", "shared=0.9")])
def test_full_size_sweep_points(sweep, point):
    """Points of the synthetic sweeps that `bench.py --sweep` times, at full size in the benchmark's
    layout, on 512 sampled (request, head) pairs: a masked node of 64 drafted tokens per sequence, one-token
    draft nodes, a 122880-token root under 64 requests (256 rows per KV head), a six-level binary tree, the
    degenerate tree, 90 % sharing."""
    from workloads.sweeps import sweep_points, sweep_head, SWEEP_SEED
    forest = dict(sweep_points(sweep))[point]
    w = make_workload(f"{sweep}/{point}", forest, sweep_head(), seed=SWEEP_SEED, device="cuda:0", layout="htd")
    C = _C()
    print(f"[case] sweep {sweep} {point} unique_kv_bytes={w.unique_kv_bytes} requests={forest.num_requests}", flush=True)
    sel = _sample_pairs(w, 512, seed=78)
    ref, _ = A.decode_attention_workload(w, sel=sel)
    for opts in ({"share": 1, "extensions": 3}, {"share": 2, "schedule": 2, "extensions": 3}, {"share": 0}):
        pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", **opts)
        out = pa.decode(w.q, w.k_pool, w.v_pool)
        torch.cuda.synchronize()
        got = out.to(torch.float64).cpu().numpy()
        pa.close()
        g = np.stack([got[r, h] for r, h in sel])
        err = np.abs(g - ref)
        print(f"[case] sweep {sweep} {point} {opts} max_err={err.max():.3e}", flush=True)
        assert not np.any(np.isnan(got))
        assert err.max() <= TOL
        assert np.all(err <= 2e-3 + 2.0 ** -7 * np.abs(ref))
