"""The C ABI without a GPU: exported symbols, status codes and every host-side error path."""
import ctypes
import re
import os

import numpy as np
import pytest

import paper_2505_17694_amd as C
from workloads import two_level_forest, HeadConfig, build_paged_kv, DTYPE_BF16

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "codec.h")).read()
    declared = set(re.findall(r"\b(codec_[a-z_]+)\s*\(", header))
    assert declared == set(C.EXPORTED_SYMBOLS)
    lib = ctypes.CDLL(C.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings_are_distinct():
    names = {C.codec_status_string(s) for s in range(0, -8, -1)}
    assert len(names) == 8 and C.codec_status_string(-99) == "unknown status"


def _create(f=None, head=None, **kw):
    f = f or two_level_forest(100, [20, 30])
    head = head or HeadConfig(8, 2, 128, DTYPE_BF16)
    paged = kw.pop("paged", None) or build_paged_kv(f, head, seed=1)
    args = dict(num_slots=4, split_align=32, max_rows=64, share=1, cost_table=None)
    args.update(kw)
    return C.codec_plan_create(f.parent, f.node_len, f.req_node, paged.node_page_off, paged.page_ids,
                               head.num_q_heads, head.num_kv_heads, head.head_dim, head.dtype,
                               head.page_size, head.scale, **args)


def test_create_ok_and_sizes():
    st, plan = _create()
    assert st == C.CODEC_OK
    assert C.codec_plan_device_bytes(plan) % 256 == 0 and C.codec_plan_device_bytes(plan) > 0
    assert C.codec_plan_workspace_bytes(plan) >= 2 * 3 * 4 * 130 * 4
    assert C.codec_plan_destroy(plan) == C.CODEC_OK
    assert C.codec_plan_destroy(None) == C.CODEC_OK


@pytest.mark.parametrize("head,status", [
    (HeadConfig(8, 2, 96), C.CODEC_ERR_UNSUPPORTED),           # head dimensions: 64, 128, 256
    (HeadConfig(8, 2, 512), C.CODEC_ERR_UNSUPPORTED),
    (HeadConfig(64, 2, 64), C.CODEC_ERR_UNSUPPORTED),           # 64 and 256 channels: groups of at most 16
    (HeadConfig(34, 2, 256), C.CODEC_ERR_UNSUPPORTED),
    (HeadConfig(8, 2, 128, dtype=2), C.CODEC_ERR_UNSUPPORTED),
    (HeadConfig(8, 2, 128, page_size=24), C.CODEC_ERR_UNSUPPORTED),
    (HeadConfig(8, 2, 128, page_size=48), C.CODEC_ERR_UNSUPPORTED),
    (HeadConfig(8, 3, 128), C.CODEC_ERR_INVALID_ARGUMENT),
    (HeadConfig(130, 1, 128), C.CODEC_ERR_UNSUPPORTED),
    (HeadConfig(8, 2, 128, scale=-1.0), C.CODEC_ERR_INVALID_ARGUMENT),
])
def test_bad_head_configs(head, status):
    good = HeadConfig(8, 2, 128, page_size=head.page_size if head.page_size in (16, 32, 64) else 16)
    paged = build_paged_kv(two_level_forest(100, [20, 30]), good, seed=1)
    assert _create(head=head, paged=paged)[0] == status


@pytest.mark.parametrize("kw", [dict(num_slots=-1), dict(split_align=48), dict(split_align=16),
                                dict(max_rows=257), dict(max_rows=2), dict(share=3), dict(share=-1), dict(fixed_slices=-1),
                                dict(cost_table=([1, 1], [10], [[1], [2]])),
                                dict(cost_table=([1], [10, 5], [[1, 2]])),
                                dict(cost_table=([1], [10], [[0]]))])
def test_bad_options(kw):
    assert _create(**kw)[0] == C.CODEC_ERR_INVALID_ARGUMENT


def test_bad_forests():
    from workloads import Forest
    head = HeadConfig(8, 2, 128)
    good = two_level_forest(100, [20, 30])
    paged = build_paged_kv(good, head, seed=1)
    for parent, lens, req in [([0, 0, 0], [100, 20, 30], [1, 2]),        # self parent
                              ([2, 0, 1], [100, 20, 30], [1, 2]),        # cycle
                              ([-1, 0, 7], [100, 20, 30], [1, 2]),       # parent out of range
                              ([-1, 0, 0], [100, 0, 30], [1, 2]),        # empty node
                              ([-1, 0, 0], [100, 20, 30], [1, 3])]:      # request beyond the forest
        f = Forest(np.array(parent), np.array(lens), np.array(req))
        assert _create(f=f, paged=paged)[0] == C.CODEC_ERR_INVALID_TREE
    # page list shorter than ceil(len / page_size)
    short = build_paged_kv(two_level_forest(100, [20, 30]), head, seed=1)
    short.node_page_off = short.node_page_off.copy()
    short.node_page_off[1:] -= 1
    assert _create(f=good, paged=short)[0] == C.CODEC_ERR_INVALID_TREE
    neg = build_paged_kv(good, head, seed=1)
    neg.page_ids = neg.page_ids.copy(); neg.page_ids[3] = -5
    assert _create(f=good, paged=neg)[0] == C.CODEC_ERR_INVALID_TREE


def test_decode_argument_checks_happen_before_any_device_work():
    st, plan = _create()
    ws = C.codec_plan_workspace_bytes(plan)
    # not uploaded yet
    assert C.codec_decode_attention(plan, 256, 256, 256, 1000, 16 * 2 * 128, 2 * 128, 128, 256, 256, ws) \
        == C.CODEC_ERR_NOT_UPLOADED
    assert C.codec_decode_attention(plan, 0, 256, 256, 1000, 4096, 256, 128, 256, 256, ws) \
        == C.CODEC_ERR_INVALID_ARGUMENT
    assert C.codec_plan_upload(plan, 0, 1 << 20) == C.CODEC_ERR_INVALID_ARGUMENT
    assert C.codec_plan_upload(plan, 256, 16) == C.CODEC_ERR_WORKSPACE_TOO_SMALL
    assert C.codec_plan_upload(plan, 264, 1 << 20) == C.CODEC_ERR_INVALID_ARGUMENT      # misaligned
    C.codec_plan_destroy(plan)


def test_empty_batch_is_a_valid_plan():
    from workloads import Forest
    f = Forest(np.zeros(0), np.zeros(0), np.zeros(0))
    head = HeadConfig(8, 2, 128)
    st, plan = C.codec_plan_create(f.parent, f.node_len, f.req_node, np.zeros(1, np.int32), np.zeros(0, np.int32),
                                   8, 2, 128, 1, 16, head.scale, 4, 32, 64, 1, None)
    assert st == C.CODEC_OK
    st, view = C.codec_plan_export(plan)
    assert view["tasks"] == [] and view["part_rows"] == 0
    # an empty batch decodes to nothing, without touching the device
    assert C.codec_decode_attention(plan, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) == C.CODEC_OK
    C.codec_plan_destroy(plan)


def test_runtime_refuses_pools_smaller_than_the_strides_reach():
    """The binding checks on the host that the page table and strides stay inside the K/V tensors
    before anything is launched: a compacted copy of a strided view is half as long as the kernels
    would walk."""
    from workloads import make_workload, three_level_forest
    f = three_level_forest(70, [130, 45], 3, [5, 33, 64, 1, 17, 48])
    head = HeadConfig(8, 2, 128, DTYPE_BF16)
    w = make_workload("one-pool", f, head, seed=3, layout="hktd")
    pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cpu")
    pa._check_pool(w.k_pool, "k_pool")
    pa._check_pool(w.v_pool, "v_pool")
    with pytest.raises(ValueError, match="k_pool"):
        pa._check_pool(w.k_pool.contiguous(), "k_pool")
    with pytest.raises(ValueError, match="v_pool"):
        pa.decode(w.q, w.k_pool, w.v_pool[:-1].contiguous())        # refused before any pointer is used
    two = make_workload("two-pools", f, head, seed=3, layout="htd")
    with pytest.raises(ValueError):
        pa._check_pool(two.k_pool, "k_pool")                         # the other layout's pool: half the stride
    pa.close()


def test_entry_points_added_for_measurement_and_for_callers_without_a_workspace_check_their_arguments():
    """Argument errors that are caught before any HIP call."""
    assert C.codec_static_scratch_bytes() == 64 << 20
    assert C.codec_decode_attention_static(None, 16, 16, 16, 1, 2048, 128, 128, 16) == C.CODEC_ERR_INVALID_ARGUMENT
    ok = dict(buffer_ptr=4096, nbytes=1 << 20, pattern=1, nontemporal=1, workgroups=64, sink_ptr=4096)
    for bad in (dict(buffer_ptr=0), dict(sink_ptr=0), dict(nbytes=3 << 20), dict(nbytes=2048), dict(pattern=2),
                dict(workgroups=0), dict(buffer_ptr=4100)):
        args = dict(ok)
        args.update(bad)
        assert C.codec_stream_read_probe(**args) == C.CODEC_ERR_INVALID_ARGUMENT, bad
    # a plan that was never uploaded: the static entry point refuses like the workspace one
    st, plan = _create()
    assert st == C.CODEC_OK
    assert C.codec_decode_attention_static(plan, 16, 16, 16, 64, 2048, 128, 128, 16) == C.CODEC_ERR_NOT_UPLOADED
    C.codec_plan_destroy(plan)
