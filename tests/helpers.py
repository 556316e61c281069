"""Test-side plumbing: logical views of paged K/V, written independently of the oracle."""
import numpy as np
import torch

from workloads import bits_to_float64


def token_slot(w, node, t):
    """(page, in-page slot) of logical token t of a node."""
    p = w.paged
    return int(p.page_ids[p.node_page_off[node] + t // p.page_size]), t % p.page_size


def pool_row(pool, w, page, slot, kvh):
    return pool[page, slot, kvh] if w.paged.layout == "thd" else pool[page, kvh, slot]


def request_context(w, r, kvh):
    """Concatenated (K, V) float64 [N_r, d] of request r for one KV head, root first: the tokens of the
    nodes on its path, without those of its last node that its visibility mask (if any) hides."""
    ks, vs = [], []
    f = w.forest
    words = None
    if getattr(f, "req_mask_off", None) is not None and f.req_mask_off[r + 1] > f.req_mask_off[r]:
        words = [int(x) for x in f.req_mask[f.req_mask_off[r]:f.req_mask_off[r + 1]]]
    for node in f.path(r):
        for t in range(int(f.node_len[node])):
            if words is not None and node == int(f.req_node[r]) and not (words[t // 32] >> (t % 32)) & 1:
                continue
            page, slot = token_slot(w, node, t)
            ks.append(pool_row(w.k_pool, w, page, slot, kvh))
            vs.append(pool_row(w.v_pool, w, page, slot, kvh))
    K = torch.stack(ks).to(torch.float64).numpy()
    V = torch.stack(vs).to(torch.float64).numpy()
    return K, V


def set_token(w, node, t, kvh, k_row=None, v_row=None):
    page, slot = token_slot(w, node, t)
    if k_row is not None:
        pool_row(w.k_pool, w, page, slot, kvh)[:] = torch.as_tensor(k_row).to(w.k_pool.dtype)
    if v_row is not None:
        pool_row(w.v_pool, w, page, slot, kvh)[:] = torch.as_tensor(v_row).to(w.v_pool.dtype)


def q_float64(w):
    return w.q.to(torch.float64).numpy()
