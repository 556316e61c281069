"""Thin holder of a plan and the PyTorch tensors that back it (marshalling only)."""
from __future__ import annotations

import torch

from . import binding as B


class PlannedAttention:
    """Owns a codec plan plus its device metadata and workspace tensors.

    ``forest``/``paged``/``head`` are plain attribute bags (see ``workloads``):
    forest.parent, forest.node_len, forest.req_node (and, optionally, forest.req_mask_off and
    forest.req_mask: per-request visibility masks); paged.node_page_off,
    paged.page_ids, paged.num_pages and the three strides; head.num_q_heads,
    num_kv_heads, head_dim, dtype, page_size, scale.
    """

    def __init__(self, forest, paged, head, device="cuda:0", num_slots=0, split_align=0,
                 max_rows=0, share=1, cost_table=None, fixed_slices=0, schedule=0,
                 extensions=0, fused=0):
        st, plan = B.codec_plan_create(forest.parent, forest.node_len, forest.req_node,
                                       paged.node_page_off, paged.page_ids,
                                       head.num_q_heads, head.num_kv_heads, head.head_dim,
                                       head.dtype, head.page_size, head.scale,
                                       num_slots, split_align, max_rows, share, cost_table, fixed_slices, schedule,
                                       extensions, fused,
                                       getattr(forest, "req_mask_off", None), getattr(forest, "req_mask", None))
        if st != B.CODEC_OK:
            raise B.CodecError(st, "codec_plan_create")
        self.plan = plan
        self.paged = paged
        self.head = head
        self.device = torch.device(device)
        self.num_requests = len(forest.req_node)
        self.meta = None
        self.workspace = None
        if self.device.type == "cuda":
            self.meta = torch.empty(B.codec_plan_device_bytes(plan), dtype=torch.uint8, device=self.device)
            stream = torch.cuda.current_stream(self.device).cuda_stream
            st = B.codec_plan_upload(plan, self.meta.data_ptr(), self.meta.numel(), stream)
            if st != B.CODEC_OK:
                raise B.CodecError(st, "codec_plan_upload")
            self.workspace = torch.empty(B.codec_plan_workspace_bytes(plan), dtype=torch.uint8,
                                         device=self.device)

    def refresh(self, node_len, paged=None):
        """New node lengths (and page lists) for the same forest: keeps the division and the schedule."""
        if paged is not None:
            self.paged = paged
        st = B.codec_plan_refresh_lengths(self.plan, node_len, self.paged.node_page_off, self.paged.page_ids)
        if st != B.CODEC_OK:
            raise B.CodecError(st, "codec_plan_refresh_lengths")
        if self.device.type == "cuda":
            need = B.codec_plan_device_bytes(self.plan)
            if self.meta.numel() < need:
                self.meta = torch.empty(need, dtype=torch.uint8, device=self.device)
            stream = torch.cuda.current_stream(self.device).cuda_stream
            st = B.codec_plan_upload(self.plan, self.meta.data_ptr(), self.meta.numel(), stream)
            if st != B.CODEC_OK:
                raise B.CodecError(st, "codec_plan_upload")

    def export(self):
        st, view = B.codec_plan_export(self.plan)
        if st != B.CODEC_OK:
            raise B.CodecError(st, "codec_plan_export")
        return view

    def _check_pool(self, pool: torch.Tensor, what: str) -> None:
        """The kernels address `pool` through the plan's strides from its first element: the farthest
        element they can touch must lie inside the tensor's storage (a view whose strides differ from
        the plan's, e.g. a compacted copy of a strided view, would send them outside)."""
        p, h = self.paged, self.head
        last = ((p.num_pages - 1) * p.page_stride + (h.page_size - 1) * p.token_stride
                + (h.num_kv_heads - 1) * p.head_stride + h.head_dim)
        have = pool.untyped_storage().nbytes() // pool.element_size() - pool.storage_offset()
        if pool.device != self.device or pool.element_size() != 2 or last > have:
            raise ValueError(f"{what}: {have} elements from the tensor's first one on {pool.device}, "
                             f"the page table and strides reach {last} on {self.device}")

    def _check_rows(self, t: torch.Tensor, what: str) -> None:
        """q and out are dense [num_requests][num_q_heads][head_dim] tensors of the plan's dtype on its device."""
        h = self.head
        want = (self.num_requests, h.num_q_heads, h.head_dim)
        dtype = torch.float16 if h.dtype == B.CODEC_DTYPE_FP16 else torch.bfloat16
        if (tuple(t.shape) != want or t.dtype != dtype or t.device != self.device
                or not t.is_contiguous()):
            raise ValueError(f"{what}: need a contiguous {dtype} tensor of shape {want} on {self.device}, "
                             f"got {t.dtype} {tuple(t.shape)} on {t.device}, contiguous={t.is_contiguous()}")

    def decode(self, q: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor,
               out: torch.Tensor = None, stream=None) -> torch.Tensor:
        self._check_pool(k_pool, "k_pool")
        self._check_pool(v_pool, "v_pool")
        self._check_rows(q, "q")
        if out is None:
            out = torch.empty_like(q)
        self._check_rows(out, "out")
        s = (stream or torch.cuda.current_stream(self.device)).cuda_stream
        p = self.paged
        st = B.codec_decode_attention(self.plan, q.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr(),
                                      p.num_pages, p.page_stride, p.token_stride, p.head_stride,
                                      out.data_ptr(), self.workspace.data_ptr(),
                                      self.workspace.numel(), s)
        if st != B.CODEC_OK:
            raise B.CodecError(st, "codec_decode_attention")
        return out

    def partial_attention(self, q, k_pool, v_pool, stream=None) -> None:
        self._check_pool(k_pool, "k_pool")
        self._check_pool(v_pool, "v_pool")
        self._check_rows(q, "q")
        s = (stream or torch.cuda.current_stream(self.device)).cuda_stream
        p = self.paged
        st = B.codec_partial_attention(self.plan, q.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr(),
                                       p.num_pages, p.page_stride, p.token_stride, p.head_stride,
                                       self.workspace.data_ptr(), self.workspace.numel(), s)
        if st != B.CODEC_OK:
            raise B.CodecError(st, "codec_partial_attention")

    def partial_reduction(self, out, stream=None) -> None:
        self._check_rows(out, "out")
        s = (stream or torch.cuda.current_stream(self.device)).cuda_stream
        st = B.codec_partial_reduction(self.plan, self.workspace.data_ptr(), self.workspace.numel(),
                                       out.data_ptr(), s)
        if st != B.CODEC_OK:
            raise B.CodecError(st, "codec_partial_reduction")

    def close(self):
        if self.plan is not None:
            B.codec_plan_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
