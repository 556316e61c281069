"""The entry point that allocates nothing (codec_decode_attention_static) against codec_decode_attention.

Both run the same two kernels; the first keeps the partial results in the caller's workspace, the
second in the library's static scratch array.  Outputs must be bit-identical (and within the
parity bar of the oracle), on two calls in a row, the second on a smaller input: the array keeps
the first call's contents.
"""
import numpy as np
import pytest
import torch

from oracle import attention as A
from workloads import make_small_config

pytestmark = pytest.mark.gpu


def _both(C, w):
    wd = w.to("cuda:0")
    pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0")
    assert C.codec_plan_workspace_bytes(pa.plan) <= C.codec_static_scratch_bytes()
    want = pa.decode(wd.q, wd.k_pool, wd.v_pool)
    torch.cuda.synchronize()
    got = torch.full_like(wd.q, float("nan"))
    p = w.paged
    st = C.codec_decode_attention_static(pa.plan, wd.q.data_ptr(), wd.k_pool.data_ptr(), wd.v_pool.data_ptr(),
                                         p.num_pages, p.page_stride, p.token_stride, p.head_stride,
                                         got.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == C.CODEC_OK, C.codec_status_string(st)
    torch.cuda.synchronize()
    pa.close()
    return want, got


def test_static_scratch_entry_point_equals_the_workspace_one():
    import paper_2505_17694_amd as C
    assert C.codec_static_scratch_bytes() == 64 << 20
    for name, shrink, req_shrink in (("cfg3", 8, 1), ("cfg2", 16, 4)):       # the second input is smaller
        w = make_small_config(name, shrink, req_shrink, poison=True)
        print(f"[case] static scratch {w.name}", flush=True)
        want, got = _both(C, w)
        assert torch.equal(want.view(torch.int16), got.view(torch.int16))
        ref, _ = A.decode_attention_workload(w)
        err = np.abs(got.double().cpu().numpy() - ref)
        assert err.max() <= 1e-2 and np.all(err <= 2e-3 + 2.0 ** -7 * np.abs(ref))


def test_static_scratch_rejects_plans_beyond_its_size():
    """A plan whose partial results need more than the array: a clear error, nothing launched."""
    import paper_2505_17694_amd as C
    from workloads import HeadConfig, make_workload, two_level_forest, DTYPE_BF16
    # 1100 requests x 64 query heads under one root cut into many slices: partial rows beyond 64 MiB
    f = two_level_forest(8192, [16] * 1100)
    w = make_workload("big-scratch", f, HeadConfig(64, 8, 128, DTYPE_BF16), seed=3, device="cuda:0")
    pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", fixed_slices=8)
    need = C.codec_plan_workspace_bytes(pa.plan)
    assert need > C.codec_static_scratch_bytes(), need
    out = torch.zeros_like(w.q)
    p = w.paged
    st = C.codec_decode_attention_static(pa.plan, w.q.data_ptr(), w.k_pool.data_ptr(), w.v_pool.data_ptr(),
                                         p.num_pages, p.page_stride, p.token_stride, p.head_stride,
                                         out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == C.CODEC_ERR_WORKSPACE_TOO_SMALL
    assert "scratch" in C.codec_last_error_message()
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
    pa.close()
