"""Pins for the fp64 definition oracle (oracle/attention_oracle.c).

The oracle is checked against things other than itself: brute-force Python
loops over a materialised context, PyTorch's fp64 softmax on single-sequence
cases, closed forms, and invariances the definition implies (Eq. 1-2 and the
prefix-path/concatenation model of Sec. 4.1).
"""
import math

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import attention as A
from workloads import (HeadConfig, make_workload, two_level_forest, three_level_forest,
                       unshared_forest, random_forest, draft_tree_forest, draft_masked_forest, concat_forests,
                       DTYPE_FP16, DTYPE_BF16, Forest)
from helpers import request_context, q_float64, set_token, token_slot, pool_row


def brute_force(w):
    """Eq. 1-2 by explicit loops on the materialised per-request context."""
    h = w.head
    Q = q_float64(w)
    B = w.forest.num_requests
    out = np.zeros((B, h.num_q_heads, h.head_dim))
    lse = np.zeros((B, h.num_q_heads))
    for r in range(B):
        for hq in range(h.num_q_heads):
            K, V = request_context(w, r, hq // h.group)
            scores = []
            for t in range(K.shape[0]):
                acc = 0.0
                for c in range(h.head_dim):
                    acc += Q[r, hq, c] * K[t, c]
                scores.append(acc * h.scale)
            mx = max(scores)
            e = [math.exp(s - mx) for s in scores]
            z = sum(e)
            for c in range(h.head_dim):
                out[r, hq, c] = sum(e[t] * V[t, c] for t in range(len(e))) / z
            lse[r, hq] = mx + math.log(z)
    return out, lse


def test_decode16_all_bit_patterns():
    """16-bit decoding equals numpy's float16 and PyTorch's bfloat16 on every finite pattern."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref16 = bits.view(np.float16).astype(np.float64)
    refbf = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    for b in range(0, 65536, 7):          # stride keeps the ctypes loop short; ends are covered below
        for dt, ref in ((DTYPE_FP16, ref16), (DTYPE_BF16, refbf)):
            got = A.decode16(b, dt)
            assert (math.isnan(got) and math.isnan(ref[b])) or got == ref[b], (b, dt)
    assert A.decode16(0x3C00, DTYPE_FP16) == 1.0
    assert A.decode16(0x0001, DTYPE_FP16) == 2.0 ** -24       # smallest subnormal
    assert A.decode16(0x7BFF, DTYPE_FP16) == 65504.0
    assert A.decode16(0xC000, DTYPE_FP16) == -2.0
    assert A.decode16(0x3F80, DTYPE_BF16) == 1.0
    assert A.decode16(0x4049, DTYPE_BF16) == 3.140625
    assert A.decode16(0xFFFF, DTYPE_FP16) != A.decode16(0xFFFF, DTYPE_FP16)  # NaN


@pytest.mark.parametrize("dtype,hq,hkv", [(DTYPE_FP16, 2, 2), (DTYPE_BF16, 4, 2), (DTYPE_BF16, 3, 1)])
def test_brute_force_tiny_tree(dtype, hq, hkv):
    """MHA, GQA and MQA on a three-level tree with ragged page tails, d = 8."""
    f = three_level_forest(5, [7, 3], 2, [2, 9, 1, 4])
    head = HeadConfig(hq, hkv, 8, dtype, page_size=4)
    w = make_workload("tiny", f, head, seed=11, poison=True)
    out, lse = A.decode_attention_workload(w)
    ref, ref_lse = brute_force(w)
    assert np.max(np.abs(out - ref)) < 1e-13
    assert np.max(np.abs(lse - ref_lse)) < 1e-12


def test_brute_force_random_forest_internal_request():
    """Irregular forest; one request ends at an internal node (its context is another's prefix)."""
    f = random_forest(6, 4, 1.5, 6, 0.8, 1, 20, seed=5)
    inner = int(f.parent[f.req_node[0]])
    if inner < 0:
        inner = int(f.req_node[0])
    f = Forest(f.parent, f.node_len, np.concatenate([f.req_node, [inner]]))
    w = make_workload("rand", f, HeadConfig(4, 2, 8, DTYPE_FP16, page_size=2), seed=3, poison=True)
    out, _ = A.decode_attention_workload(w)
    ref, _ = brute_force(w)
    assert np.max(np.abs(out - ref)) < 1e-13


def test_brute_force_drafted_token_trees():
    """Multi-token decoding: a request at every drafted token (one-token nodes) and at every context;
    a query sees its path only, so a drafted token on another branch must not leak in.  The second
    part plants a huge key on a sibling branch and checks that only its own branch notices."""
    f = draft_tree_forest(5, [7, 3], 6, seed=2)
    w = make_workload("drafts", f, HeadConfig(4, 2, 8, DTYPE_BF16, page_size=4), seed=9, poison=True)
    out, lse = A.decode_attention_workload(w)
    ref, ref_lse = brute_force(w)
    assert np.max(np.abs(out - ref)) < 1e-13 and np.max(np.abs(lse - ref_lse)) < 1e-12
    # the first drafted token with a sibling: a key of 100s in it changes the requests below it only
    parents = [int(p) for p in f.parent]
    node = next(n for n in range(f.num_nodes) if f.node_len[n] == 1 and parents.count(parents[n]) > 1)
    page, slot = token_slot(w, node, 0)
    for kvh in range(w.head.num_kv_heads):
        pool_row(w.k_pool, w, page, slot, kvh)[:] = 100.0
    out2, _ = A.decode_attention_workload(w)
    below = [r for r in range(f.num_requests) if node in f.path(r)]
    others = [r for r in range(f.num_requests) if node not in f.path(r)]
    assert below and others
    assert np.array_equal(out2[others], out[others])
    assert all(np.max(np.abs(out2[r] - out[r])) > 1e-6 for r in below)


def test_brute_force_with_visibility_masks():
    """Sec. 4.1 visibility: a request with a mask over its last node attends to the visible tokens only
    (brute-force loops over the materialised visible context); 40 drafted tokens need two mask words."""
    f = concat_forests(draft_masked_forest(5, [7, 3], 6, seed=2), draft_masked_forest(0, [9], 40, seed=5))
    w = make_workload("masked", f, HeadConfig(4, 2, 8, DTYPE_BF16, page_size=4), seed=9, poison=True)
    out, lse = A.decode_attention_workload(w)
    ref, ref_lse = brute_force(w)
    assert np.max(np.abs(out - ref)) < 1e-13 and np.max(np.abs(lse - ref_lse)) < 1e-12
    # masks really hide something: with every bit set the drafted requests give other results
    full = Forest(f.parent, f.node_len, f.req_node, f.req_mask_off, np.full_like(f.req_mask, 0xFFFFFFFF))
    w_all = make_workload("masked", full, w.head, seed=9, poison=True)
    out_all, _ = A.decode_attention_workload(w_all)
    unmasked = Forest(f.parent, f.node_len, f.req_node)
    out_none, _ = A.decode_attention_workload(make_workload("masked", unmasked, w.head, seed=9, poison=True))
    assert np.array_equal(out_all, out_none)                # all bits set = no mask at all
    hidden = [r for r in range(f.num_requests) if f.visible(r) is not None and not f.visible(r).all()]
    assert len(hidden) > 20 and all(np.max(np.abs(out[r] - out_none[r])) > 1e-9 for r in hidden)


def test_masked_draft_node_equals_tree_of_one_token_nodes():
    """Two statements of one verification step: every drafted token a node of its own (what a query sees
    is its path: pinned by brute force above), or all drafted tokens of a sequence in one node with a
    mask per query.  Same drafted trees, the same K/V rows copied token by token: identical outputs, the
    visible tokens being summed in the same order."""
    head = HeadConfig(4, 2, 16, DTYPE_FP16, page_size=4)
    tree = draft_tree_forest(11, [19, 6, 33], 9, seed=12)
    packed = draft_masked_forest(11, [19, 6, 33], 9, seed=12)
    assert tree.num_requests == packed.num_requests == 3 * 10
    a = make_workload("tree", tree, head, seed=4, poison=True)
    b = make_workload("packed", packed, head, seed=5, poison=True)
    b.q[:] = a.q
    # node numbering: tree = prompt, then per sequence context + 9 one-token nodes; packed = prompt, then
    # per sequence context + one 9-token node
    pairs = [((0, t), (0, t)) for t in range(11)]
    for i, n in enumerate([19, 6, 33]):
        ta, tb = 1 + i * 10, 1 + i * 2
        pairs += [((ta, t), (tb, t)) for t in range(n)]
        pairs += [((ta + 1 + k, 0), (tb + 1, k)) for k in range(9)]
    _copy_logical(a, b, pairs)
    out_a, lse_a = A.decode_attention_workload(a)
    out_b, lse_b = A.decode_attention_workload(b)
    assert np.array_equal(out_a, out_b) and np.array_equal(lse_a, lse_b)


def test_planted_key_is_seen_through_the_mask_only():
    """A key with a huge logit planted in drafted token k: the requests whose mask has bit k answer with
    (almost exactly) that token's V row, every other request's output does not move by one bit."""
    f = draft_masked_forest(4, [10, 5], 7, seed=21)
    head = HeadConfig(2, 2, 8, DTYPE_FP16, page_size=4)
    w = make_workload("planted", f, head, seed=6, poison=True)
    w.q[:] = torch.ones_like(w.q)
    base, _ = A.decode_attention_workload(w)
    draft_node, k = 2, 3                                   # first sequence's draft node, its fourth token
    marker = torch.arange(8, dtype=torch.float32) - 3.0
    for kvh in range(2):
        set_token(w, draft_node, k, kvh, k_row=torch.full((8,), 30.0), v_row=marker)
    out, _ = A.decode_attention_workload(w)
    sees = [r for r in range(f.num_requests) if f.req_node[r] == draft_node and f.visible(r)[k]]
    blind = [r for r in range(f.num_requests) if r not in sees]
    assert sees and len(blind) > len(sees)
    assert np.array_equal(out[blind], base[blind])
    for r in sees:
        assert np.max(np.abs(out[r] - marker.double().numpy())) < 1e-9


def test_request_that_sees_nothing_is_rejected():
    """A mask that hides every token of a request whose path is its last node alone: no context at all."""
    g = Forest(np.array([-1]), np.array([5]), np.array([0]), np.array([0, 1]), np.array([0], dtype=np.uint32))
    w = make_workload("blind", g, HeadConfig(2, 2, 8, DTYPE_FP16, page_size=4), seed=1)
    with pytest.raises(ValueError):
        A.decode_attention_workload(w)


def test_single_sequence_equals_torch_softmax():
    """Unshared single-node requests reduce to ordinary attention: library routine."""
    f = unshared_forest([37, 1, 130])
    head = HeadConfig(8, 2, 128, DTYPE_BF16)
    w = make_workload("single", f, head, seed=7, poison=True)
    out, lse = A.decode_attention_workload(w)
    Q = torch.from_numpy(q_float64(w))
    for r in range(3):
        for hq in range(8):
            K, V = request_context(w, r, hq // 4)
            s = (torch.from_numpy(K) @ Q[r, hq]) * head.scale
            ref = torch.softmax(s, dim=0) @ torch.from_numpy(V)
            assert torch.max(torch.abs(ref - torch.from_numpy(out[r, hq]))) < 1e-13
            assert abs(lse[r, hq] - logsumexp(s.numpy())) < 1e-12


def test_zero_query_gives_mean_of_values():
    f = two_level_forest(21, [5, 12])
    w = make_workload("zeroq", f, HeadConfig(4, 2, 16, DTYPE_FP16, page_size=4), seed=1, poison=True)
    w.q.zero_()
    out, lse = A.decode_attention_workload(w)
    for r in range(2):
        for hq in range(4):
            K, V = request_context(w, r, hq // 2)
            assert np.max(np.abs(out[r, hq] - V.mean(axis=0))) < 1e-14
            assert abs(lse[r, hq] - math.log(V.shape[0])) < 1e-13


def test_dominant_key_selects_its_value_row():
    """One key aligned with q at logit +60 above the rest: output is that token's V row."""
    f = two_level_forest(16, [6, 6])
    head = HeadConfig(2, 2, 16, DTYPE_FP16, page_size=4, scale=1.0)
    w = make_workload("peak", f, head, seed=2, poison=True)
    w.q.zero_(); w.k_pool[~torch.isnan(w.k_pool)] = 0
    w.q[:, :, 0] = 8.0
    set_token(w, 0, 9, 0, k_row=[8.0] + [0.0] * 15)        # root token 9, kv head 0: logit 64
    set_token(w, 2, 3, 1, k_row=[7.5] + [0.0] * 15)        # leaf of request 1, kv head 1: logit 60
    out, _ = A.decode_attention_workload(w)
    page, slot = token_slot(w, 0, 9)
    v_root = pool_row(w.v_pool, w, page, slot, 0).double().numpy()
    page, slot = token_slot(w, 2, 3)
    v_leaf = pool_row(w.v_pool, w, page, slot, 1).double().numpy()
    for r in range(2):
        assert np.max(np.abs(out[r, 0] - v_root)) < 1e-14
    assert np.max(np.abs(out[1, 1] - v_leaf)) < 1e-14
    # request 0 never sees request 1's leaf: on kv head 1 all its logits are 0 -> mean of V
    K, V = request_context(w, 0, 1)
    assert np.max(np.abs(out[0, 1] - V.mean(axis=0))) < 1e-14


def test_duplicate_requests_get_identical_rows():
    f = two_level_forest(33, [9, 9, 4])
    w = make_workload("dup", f, HeadConfig(4, 4, 32, DTYPE_BF16, page_size=8), seed=4)
    # make request 1 a copy of request 0: same query and same leaf contents
    w.q[1] = w.q[0]
    for t in range(9):
        for kvh in range(4):
            p0, s0 = token_slot(w, 1, t)
            set_token(w, 2, t, kvh, k_row=pool_row(w.k_pool, w, p0, s0, kvh).clone(),
                      v_row=pool_row(w.v_pool, w, p0, s0, kvh).clone())
    out, _ = A.decode_attention_workload(w)
    assert np.array_equal(out[0], out[1])
    assert not np.array_equal(out[0], out[2])


def _copy_logical(src, dst, pairs):
    """pairs: ((src_node, src_t), (dst_node, dst_t)) token copies over all KV heads."""
    for (sn, st), (dn, dt_) in pairs:
        ps, ss = token_slot(src, sn, st)
        for kvh in range(src.head.num_kv_heads):
            set_token(dst, dn, dt_, kvh, k_row=pool_row(src.k_pool, src, ps, ss, kvh).clone(),
                      v_row=pool_row(src.v_pool, src, ps, ss, kvh).clone())


def test_invariant_to_how_the_context_is_cut_into_nodes():
    """The same 50-token context as one node, or as 23 + 27 over two nodes."""
    head = HeadConfig(4, 2, 16, DTYPE_FP16, page_size=4)
    a = make_workload("a", unshared_forest([50]), head, seed=9, poison=True)
    fb = Forest(np.array([-1, 0]), np.array([23, 27]), np.array([1]))
    b = make_workload("b", fb, head, seed=10, poison=True)
    b.q[:] = a.q
    _copy_logical(a, b, [((0, t), (0, t)) for t in range(23)] + [((0, 23 + t), (1, t)) for t in range(27)])
    oa, la = A.decode_attention_workload(a)
    ob, lb = A.decode_attention_workload(b)
    assert np.max(np.abs(oa - ob)) < 1e-15
    assert np.max(np.abs(la - lb)) < 1e-13


def test_invariant_to_physical_page_order_and_layout():
    f = three_level_forest(19, [11, 6], 2, [3, 8, 5, 2])
    head = HeadConfig(4, 2, 16, DTYPE_BF16, page_size=4)
    a = make_workload("a", f, head, seed=21, poison=True)
    b = make_workload("b", f, head, seed=99, poison=True, layout="htd")   # other permutation, other layout
    b.q[:] = a.q
    _copy_logical(a, b, [((n, t), (n, t)) for n in range(f.num_nodes) for t in range(int(f.node_len[n]))])
    oa, _ = A.decode_attention_workload(a)
    ob, _ = A.decode_attention_workload(b)
    assert np.array_equal(oa, ob)


def test_one_pool_for_keys_and_values_changes_nothing():
    """The layout with K and V of a page and head side by side holds the values of the layout with two
    pools (same seed); the oracle, addressing both through their strides, returns the same bits."""
    f = three_level_forest(70, [130, 45], 3, [5, 33, 64, 1, 17, 48])
    head = HeadConfig(8, 2, 128, DTYPE_BF16)
    a = make_workload("two", f, head, seed=3, poison=True, layout="htd")
    b = make_workload("one", f, head, seed=3, poison=True, layout="hktd")
    assert b.kv_pool is not None and b.paged.page_stride == 2 * a.paged.page_stride
    assert b.k_pool.data_ptr() == b.kv_pool.data_ptr()
    assert b.v_pool.data_ptr() == b.kv_pool.data_ptr() + 2 * head.page_size * head.head_dim
    oa, la = A.decode_attention_workload(a)
    ob, lb = A.decode_attention_workload(b)
    assert np.array_equal(oa, ob) and np.array_equal(la, lb)


def test_selection_matches_full_run_and_threads_do_not_matter():
    f = two_level_forest(40, [7, 13, 2])
    w = make_workload("sel", f, HeadConfig(4, 2, 32, DTYPE_BF16, page_size=8), seed=6, poison=True)
    full, lse = A.decode_attention_workload(w, nthreads=1)
    sel = [(2, 3), (0, 0), (1, 2)]
    part, plse = A.decode_attention_workload(w, sel=sel, nthreads=3)
    for i, (r, hq) in enumerate(sel):
        assert np.array_equal(part[i], full[r, hq])
        assert plse[i] == lse[r, hq]


def test_rejects_cyclic_forest():
    f = Forest(np.array([1, 0]), np.array([4, 4]), np.array([0]))
    w = make_workload("cyc", unshared_forest([4, 4]), HeadConfig(2, 2, 8, DTYPE_FP16, page_size=4), seed=1)
    with pytest.raises(ValueError):
        A.decode_attention(f.parent, f.node_len, f.req_node, w.paged.node_page_off, w.paged.page_ids,
                           4, 2, 2, 8, DTYPE_FP16, 1.0, w.q_bits(), w.k_bits(), w.v_bits(),
                           w.paged.page_stride, w.paged.token_stride, w.paged.head_stride)
