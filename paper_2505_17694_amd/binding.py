"""ctypes binding of libcodec.so: the C ABI of include/codec.h under the same names.

Argument marshalling only.  Every step of the decode path runs inside the
library; PyTorch is used by callers for device memory and streams.  If the
library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t,
                    c_void_p, byref)

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcodec.so")

CODEC_OK = 0
CODEC_ERR_INVALID_ARGUMENT = -1
CODEC_ERR_INVALID_TREE = -2
CODEC_ERR_UNSUPPORTED = -3
CODEC_ERR_WORKSPACE_TOO_SMALL = -4
CODEC_ERR_HIP = -5
CODEC_ERR_NOT_UPLOADED = -6
CODEC_ERR_OUT_OF_MEMORY = -7
CODEC_DTYPE_FP16 = 0
CODEC_DTYPE_BF16 = 1
CODEC_PLAN_EXT_SLACK = 1
CODEC_PLAN_EXT_DIAGONAL = 2

# every symbol include/codec.h declares
EXPORTED_SYMBOLS = [
    "codec_plan_create", "codec_plan_destroy", "codec_plan_export", "codec_cost_estimate",
    "codec_default_cost_table", "codec_plan_device_bytes", "codec_plan_upload",
    "codec_plan_workspace_bytes", "codec_decode_attention", "codec_partial_attention",
    "codec_partial_reduction", "codec_status_string", "codec_last_error_message",
    "codec_plan_refresh_lengths", "codec_decode_attention_static", "codec_static_scratch_bytes",
    "codec_stream_read_probe",
]

_i32p = POINTER(c_int32)
_i64p = POINTER(c_int64)


class codec_head_config(Structure):
    _fields_ = [("num_q_heads", c_int32), ("num_kv_heads", c_int32), ("head_dim", c_int32),
                ("dtype", c_int32), ("page_size", c_int32), ("scale", c_float)]


class codec_tree(Structure):
    _fields_ = [("num_nodes", c_int32), ("parent", _i32p), ("node_len", _i32p),
                ("num_requests", c_int32), ("req_node", _i32p),
                ("node_page_off", _i32p), ("page_ids", _i32p),
                ("req_mask_off", _i32p), ("req_mask", POINTER(ctypes.c_uint32))]


class codec_cost_table(Structure):
    _fields_ = [("num_row_points", c_int32), ("num_len_points", c_int32),
                ("row_grid", _i32p), ("len_grid", _i32p), ("cost", _i64p)]


class codec_plan_options(Structure):
    _fields_ = [("num_slots", c_int32), ("split_align", c_int32), ("max_rows", c_int32),
                ("share", c_int32), ("cost", POINTER(codec_cost_table)), ("fixed_slices", c_int32),
                ("schedule", c_int32), ("fused", c_int32), ("extensions", c_int32)]


class codec_item(Structure):
    _fields_ = [("node", c_int32), ("q_off", c_int32), ("n_req", c_int32), ("rows", c_int32),
                ("len", c_int32), ("ub", c_int32), ("b", c_int32), ("reserved", c_int32),
                ("cost", c_int64)]


class codec_task(Structure):
    _fields_ = [("item", c_int32), ("node", c_int32), ("kv_begin", c_int32), ("kv_len", c_int32),
                ("q_off", c_int32), ("n_req", c_int32), ("part_row_base", c_int32),
                ("slot", c_int32), ("cost", c_int64)]


class codec_plan_view(Structure):
    _fields_ = [("num_items", c_int32), ("items", POINTER(codec_item)),
                ("num_tasks", c_int32), ("tasks", POINTER(codec_task)),
                ("num_slots", c_int32), ("slot_off", _i32p), ("slot_tasks", _i32p),
                ("num_nodes", c_int32), ("node_q_off", _i32p), ("node_q", _i32p),
                ("num_requests", c_int32), ("req_part_off", _i32p), ("req_part", _i32p),
                ("cost_l", c_int64), ("makespan", c_int64), ("part_rows", c_int32),
                ("split_align", c_int32), ("max_rows", c_int32), ("share", c_int32),
                ("schedule", c_int32), ("fused", c_int32), ("num_entries", c_int32), ("queue_off", _i32p), ("queue_tasks", _i32p)]


class codec_kv_layout(Structure):
    _fields_ = [("num_pages", c_int64), ("page_stride", c_int64), ("token_stride", c_int64),
                ("head_stride", c_int64)]


# PyTorch wheels carry their own copy of the HIP runtime.  Device pointers and streams handed to the
# library come from PyTorch, so both must use the same runtime instance: load PyTorch's first, and
# libcodec.so's dependency on libamdhip64 then resolves to the copy already in the process.
try:
    import torch  # noqa: F401
except ImportError:
    pass

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_17694_amd.build` "
                      "(there is no CPU fallback)")
_lib = ctypes.CDLL(LIB_PATH)

_lib.codec_plan_create.restype = c_int
_lib.codec_plan_create.argtypes = [POINTER(codec_tree), POINTER(codec_head_config),
                                   POINTER(codec_plan_options), POINTER(c_void_p)]
_lib.codec_plan_destroy.restype = c_int
_lib.codec_plan_destroy.argtypes = [c_void_p]
_lib.codec_plan_export.restype = c_int
_lib.codec_plan_export.argtypes = [c_void_p, POINTER(codec_plan_view)]
_lib.codec_plan_refresh_lengths.restype = c_int
_lib.codec_plan_refresh_lengths.argtypes = [c_void_p, _i32p, _i32p, _i32p]
_lib.codec_cost_estimate.restype = c_int64
_lib.codec_cost_estimate.argtypes = [POINTER(codec_cost_table), c_int32, c_int32]
_lib.codec_default_cost_table.restype = POINTER(codec_cost_table)
_lib.codec_default_cost_table.argtypes = [c_int32]
_lib.codec_plan_device_bytes.restype = c_size_t
_lib.codec_plan_device_bytes.argtypes = [c_void_p]
_lib.codec_plan_upload.restype = c_int
_lib.codec_plan_upload.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
_lib.codec_plan_workspace_bytes.restype = c_size_t
_lib.codec_plan_workspace_bytes.argtypes = [c_void_p]
_lib.codec_decode_attention.restype = c_int
_lib.codec_decode_attention.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p,
                                        POINTER(codec_kv_layout), c_void_p, c_void_p, c_size_t,
                                        c_void_p]
_lib.codec_partial_attention.restype = c_int
_lib.codec_partial_attention.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p,
                                         POINTER(codec_kv_layout), c_void_p, c_size_t, c_void_p]
_lib.codec_partial_reduction.restype = c_int
_lib.codec_partial_reduction.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p, c_void_p]
_lib.codec_decode_attention_static.restype = c_int
_lib.codec_decode_attention_static.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p,
                                               POINTER(codec_kv_layout), c_void_p, c_void_p]
_lib.codec_static_scratch_bytes.restype = c_size_t
_lib.codec_static_scratch_bytes.argtypes = []
_lib.codec_stream_read_probe.restype = c_int
_lib.codec_stream_read_probe.argtypes = [c_void_p, c_size_t, c_int32, c_int32, c_int32, c_void_p, c_void_p]
_lib.codec_status_string.restype = c_char_p
_lib.codec_status_string.argtypes = [c_int]
_lib.codec_last_error_message.restype = c_char_p
_lib.codec_last_error_message.argtypes = []


class CodecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = codec_last_error_message() if status == CODEC_ERR_HIP else ""
        super().__init__(f"{where}: {codec_status_string(status)} ({status})" + (f": {detail}" if detail else ""))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a, ct=c_int32):
    return a.ctypes.data_as(POINTER(ct)) if a is not None and a.size else None


def make_cost_table(row_grid, len_grid, cost):
    """Marshal a cost table; returns (struct, keepalive) - keep both alive while the struct is used."""
    rg, lg = _i32(row_grid), _i32(len_grid)
    c = np.ascontiguousarray(cost, dtype=np.int64).reshape(-1)
    t = codec_cost_table(len(rg), len(lg), _ptr(rg), _ptr(lg), _ptr(c, c_int64))
    return t, (rg, lg, c)


def codec_status_string(status: int) -> str:
    return _lib.codec_status_string(int(status)).decode()


def codec_last_error_message() -> str:
    return _lib.codec_last_error_message().decode()


def codec_plan_create(parent, node_len, req_node, node_page_off, page_ids,
                      num_q_heads, num_kv_heads, head_dim, dtype, page_size, scale,
                      num_slots=0, split_align=0, max_rows=0, share=1, cost_table=None, fixed_slices=0,
                      schedule=0, extensions=0, fused=0, req_mask_off=None, req_mask=None):
    """Returns (status, plan handle or None).  ``cost_table``: (row_grid, len_grid, cost) or None;
    ``req_mask_off`` / ``req_mask``: per-request visibility masks (see codec_tree) or None."""
    parent, node_len, req_node = _i32(parent), _i32(node_len), _i32(req_node)
    node_page_off, page_ids = _i32(node_page_off), _i32(page_ids)
    mask_off = mask_words = None
    if req_mask_off is not None:
        mask_off = _i32(req_mask_off)
        mask_words = np.ascontiguousarray(req_mask if req_mask is not None else [], dtype=np.uint32)
    tree = codec_tree(len(parent), _ptr(parent), _ptr(node_len), len(req_node), _ptr(req_node),
                      _ptr(node_page_off), _ptr(page_ids),
                      _ptr(mask_off) if mask_off is not None else None,
                      _ptr(mask_words, ctypes.c_uint32) if mask_words is not None else None)
    head = codec_head_config(num_q_heads, num_kv_heads, head_dim, dtype, page_size, scale)
    keep = None
    ct_ptr = None
    if cost_table is not None:
        ct, keep = make_cost_table(*cost_table)
        ct_ptr = ctypes.pointer(ct)
    opt = codec_plan_options(num_slots, split_align, max_rows, share, ct_ptr, fixed_slices, schedule,
                             fused, extensions)
    handle = c_void_p()
    st = _lib.codec_plan_create(byref(tree), byref(head), byref(opt), byref(handle))
    del keep
    return st, (handle if st == CODEC_OK else None)


def codec_plan_destroy(plan) -> int:
    return _lib.codec_plan_destroy(plan)


def _arr(ptr, n, dtype=np.int32):
    if n == 0:
        return np.zeros(0, dtype=dtype)
    return np.ctypeslib.as_array(ptr, shape=(n,)).copy()


def codec_plan_export(plan):
    """Returns (status, dict of numpy copies of the plan view)."""
    v = codec_plan_view()
    st = _lib.codec_plan_export(plan, byref(v))
    if st != CODEC_OK:
        return st, None
    items = [{f: getattr(v.items[i], f) for f, _ in codec_item._fields_ if f != "reserved"}
             for i in range(v.num_items)]
    tasks = [{f: getattr(v.tasks[i], f) for f, _ in codec_task._fields_} for i in range(v.num_tasks)]
    out = {
        "items": items, "tasks": tasks, "num_slots": v.num_slots,
        "slot_off": _arr(v.slot_off, v.num_slots + 1), "slot_tasks": _arr(v.slot_tasks, v.num_tasks),
        "node_q_off": _arr(v.node_q_off, v.num_nodes + 1),
        "req_part_off": _arr(v.req_part_off, v.num_requests + 1),
        "cost_l": v.cost_l, "makespan": v.makespan, "part_rows": v.part_rows,
        "split_align": v.split_align, "max_rows": v.max_rows, "share": v.share,
        "schedule": v.schedule, "fused": v.fused, "queue_off": _arr(v.queue_off, v.num_entries + 1),
        "queue_tasks": _arr(v.queue_tasks, v.num_tasks),
    }
    out["node_q"] = _arr(v.node_q, int(out["node_q_off"][-1]) if v.num_nodes else 0)
    out["req_part"] = _arr(v.req_part, int(out["req_part_off"][-1]))
    return st, out


def codec_plan_refresh_lengths(plan, node_len, node_page_off, page_ids) -> int:
    node_len, node_page_off, page_ids = _i32(node_len), _i32(node_page_off), _i32(page_ids)
    return _lib.codec_plan_refresh_lengths(plan, _ptr(node_len), _ptr(node_page_off), _ptr(page_ids))


def codec_cost_estimate(cost_table, rows: int, length: int) -> int:
    if cost_table is None:
        return int(_lib.codec_cost_estimate(None, rows, length))
    ct, keep = make_cost_table(*cost_table)
    r = int(_lib.codec_cost_estimate(byref(ct), rows, length))
    del keep
    return r


def codec_default_cost_table(wide: int):
    """Returns (row_grid, len_grid, cost[rows][lens]) of a built-in table as Python lists."""
    t = _lib.codec_default_cost_table(int(wide)).contents
    rg = [t.row_grid[i] for i in range(t.num_row_points)]
    lg = [t.len_grid[i] for i in range(t.num_len_points)]
    cost = [[t.cost[i * t.num_len_points + j] for j in range(t.num_len_points)]
            for i in range(t.num_row_points)]
    return rg, lg, cost


def codec_plan_device_bytes(plan) -> int:
    return int(_lib.codec_plan_device_bytes(plan))


def codec_plan_upload(plan, device_meta_ptr: int, device_meta_bytes: int, stream: int = 0) -> int:
    return _lib.codec_plan_upload(plan, c_void_p(device_meta_ptr), device_meta_bytes, c_void_p(stream))


def codec_plan_workspace_bytes(plan) -> int:
    return int(_lib.codec_plan_workspace_bytes(plan))


def codec_decode_attention(plan, q_ptr: int, k_ptr: int, v_ptr: int, num_pages: int,
                           page_stride: int, token_stride: int, head_stride: int, out_ptr: int,
                           workspace_ptr: int, workspace_bytes: int, stream: int = 0) -> int:
    lay = codec_kv_layout(num_pages, page_stride, token_stride, head_stride)
    return _lib.codec_decode_attention(plan, c_void_p(q_ptr), c_void_p(k_ptr), c_void_p(v_ptr),
                                       byref(lay), c_void_p(out_ptr), c_void_p(workspace_ptr),
                                       workspace_bytes, c_void_p(stream))


def codec_partial_attention(plan, q_ptr: int, k_ptr: int, v_ptr: int, num_pages: int,
                            page_stride: int, token_stride: int, head_stride: int,
                            workspace_ptr: int, workspace_bytes: int, stream: int = 0) -> int:
    lay = codec_kv_layout(num_pages, page_stride, token_stride, head_stride)
    return _lib.codec_partial_attention(plan, c_void_p(q_ptr), c_void_p(k_ptr), c_void_p(v_ptr),
                                        byref(lay), c_void_p(workspace_ptr), workspace_bytes,
                                        c_void_p(stream))


def codec_partial_reduction(plan, workspace_ptr: int, workspace_bytes: int, out_ptr: int,
                            stream: int = 0) -> int:
    return _lib.codec_partial_reduction(plan, c_void_p(workspace_ptr), workspace_bytes,
                                        c_void_p(out_ptr), c_void_p(stream))


def codec_decode_attention_static(plan, q_ptr: int, k_ptr: int, v_ptr: int, num_pages: int,
                                  page_stride: int, token_stride: int, head_stride: int, out_ptr: int,
                                  stream: int = 0) -> int:
    lay = codec_kv_layout(num_pages, page_stride, token_stride, head_stride)
    return _lib.codec_decode_attention_static(plan, c_void_p(q_ptr), c_void_p(k_ptr), c_void_p(v_ptr),
                                              byref(lay), c_void_p(out_ptr), c_void_p(stream))


def codec_static_scratch_bytes() -> int:
    return int(_lib.codec_static_scratch_bytes())


def codec_stream_read_probe(buffer_ptr: int, nbytes: int, pattern: int, nontemporal: int, workgroups: int,
                            sink_ptr: int, stream: int = 0) -> int:
    return _lib.codec_stream_read_probe(c_void_p(buffer_ptr), nbytes, pattern, nontemporal, workgroups,
                                        c_void_p(sink_ptr), c_void_p(stream))
