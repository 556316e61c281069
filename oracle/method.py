"""The paper's method, step by step, in fp64 numpy.  TEST INFRASTRUCTURE ONLY.

* ``pac``  - partial attention computation (Alg. 2): attention of a query
  set against one KV chunk, returning the normalised output with the row
  maximum m and the sum of exponentials s.
* ``por``  - partial output reduction (Alg. 3): binary merge of two partial
  results of the same queries.
* ``streaming_update`` - the running (M, D, U) accumulators of Sec. 4.1
  "Streaming softmax across nodes".  The paper prints only M <- max(M, m); the
  D and U updates used here are the ones that keep numerator and denominator
  in the frame of the new maximum (D <- D e^{M-Mh} + d e^{m-Mh}, same for U),
  which is what Alg. 3 computes for normalised outputs.
* ``codec`` - Alg. 4: PAC for every node against the queries of all requests
  below it, then per-query reduction of the node results along the path.
* ``replay_tasks`` - the same with an explicit task list (node chunk x request
  range) and per-request partial lists, to check that a plan covers every
  (request, token) once.

Nothing here is shared with the HIP library.
"""
from __future__ import annotations

import numpy as np


def widen(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Exact fp16 (dtype 0) / bf16 (dtype 1) bit patterns -> float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == 0:
        return bits.view(np.float16).astype(np.float64)
    with np.errstate(invalid="ignore"):     # signalling-NaN patterns may appear in poisoned padding
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def pac(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float, visible=None):
    """Alg. 2 on Q [n_q, d], K, V [n, d] -> (O [n_q, d], m [n_q], s [n_q]).

    ``visible`` [n_q, n] bool: the visibility mask of Sec. 4.1 (an invisible position gets the score
    -inf and contributes 0); every query must see at least one position.
    """
    S = (Q @ K.T) * scale
    if visible is not None:
        S = np.where(visible, S, -np.inf)
    m = S.max(axis=1)
    P = np.exp(S - m[:, None])
    s = P.sum(axis=1)
    O = (P @ V) / s[:, None]
    return O, m, s


def por(O1, m1, s1, O2, m2, s2):
    """Alg. 3: merge two partial results of the same queries."""
    m = np.maximum(m1, m2)
    w1 = s1 * np.exp(m1 - m)
    w2 = s2 * np.exp(m2 - m)
    s = w1 + w2
    O = (O1 * w1[..., None] + O2 * w2[..., None]) / s[..., None]
    return O, m, s


def streaming_update(M, D, U, m, d, u):
    """Sec. 4.1 accumulators: fold one node's (m, d, u) into the running (M, D, U)."""
    Mh = np.maximum(M, m)
    a = np.where(np.isneginf(M), 0.0, np.exp(M - Mh))
    b = np.exp(m - Mh)
    return Mh, D * a + d * b, U * a[..., None] + u * b[..., None]


def paths_and_queries(parent, req_node):
    """Prefix path of every request (root first) and, per node, the requests below it."""
    n_nodes = len(parent)
    paths = []
    node_q = [[] for _ in range(n_nodes)]
    for r, leaf in enumerate(req_node):
        p = []
        n = int(leaf)
        while n != -1:
            p.append(n)
            n = int(parent[n])
        p.reverse()
        paths.append(p)
        for n in p:
            node_q[n].append(r)
    return paths, node_q


def gather_node_kv(w, node: int, kvh: int, t0: int, t1: int):
    """K and V rows [t0, t1) of ``node`` for KV head ``kvh`` as float64 [t1-t0, d]."""
    p, h = w.paged, w.head
    kb, vb = w.k_bits().reshape(-1), w.v_bits().reshape(-1)
    t = np.arange(t0, t1, dtype=np.int64)
    page = p.page_ids[p.node_page_off[node] + t // p.page_size].astype(np.int64)
    base = page * p.page_stride + (t % p.page_size) * p.token_stride + kvh * p.head_stride
    idx = base[:, None] + np.arange(h.head_dim, dtype=np.int64)[None, :]
    return widen(kb[idx], h.dtype), widen(vb[idx], h.dtype)


def _visibility(f, node: int, reqs, g: int, t0: int, t1: int):
    """Rows (request x head of the group) x tokens [t0, t1) of ``node``: which positions each row sees
    (Sec. 4.1).  A request's mask covers its last node only; None when no row of the task is masked."""
    if getattr(f, "req_mask_off", None) is None:
        return None
    rows = []
    any_mask = False
    for r in reqs:
        vis = f.visible(int(r)) if int(f.req_node[int(r)]) == node else None
        any_mask |= vis is not None
        row = np.ones(t1 - t0, dtype=bool) if vis is None else vis[t0:t1]
        rows += [row] * g
    return np.stack(rows) if any_mask else None


def codec(w):
    """Alg. 4 on a workload -> out [B, h_q, d] float64 (tree sharing, node-level partials)."""
    f, h = w.forest, w.head
    g = h.group
    Q = widen(w.q_bits(), h.dtype)                     # [B, h_q, d]
    paths, node_q = paths_and_queries(f.parent, f.req_node)
    B = f.num_requests
    out = np.zeros((B, h.num_q_heads, h.head_dim))
    for kvh in range(h.num_kv_heads):
        # O_tree: one partial per node, rows = (request in I_n) x (head in group)
        tree = {}
        for n in range(f.num_nodes):
            if not node_q[n]:
                continue
            K, V = gather_node_kv(w, n, kvh, 0, int(f.node_len[n]))
            Qn = Q[node_q[n], kvh * g:(kvh + 1) * g, :].reshape(-1, h.head_dim)
            tree[n] = pac(Qn, K, V, h.scale, _visibility(f, n, node_q[n], g, 0, int(f.node_len[n])))
        for r in range(B):
            acc = None
            for n in paths[r]:
                O, m, s = tree[n]
                a = node_q[n].index(r) * g
                part = (O[a:a + g], m[a:a + g], s[a:a + g])
                acc = part if acc is None else por(*acc, *part)
            out[r, kvh * g:(kvh + 1) * g, :] = acc[0]
    return out


def replay_tasks(w, tasks, node_q_flat, req_part_off, req_part):
    """Run an explicit task list on the CPU.

    ``tasks``: rows of (node, kv_begin, kv_len, q_off, n_req, part_row_base);
    the task's queries are requests ``node_q_flat[q_off : q_off + n_req]`` and
    its partial rows are ``part_row_base + i * g + j`` for its i-th request and
    the j-th head of the group.  ``req_part[req_part_off[r] : req_part_off[r+1]]``
    lists, for request r, the first partial row of each of its partials.
    """
    f, h = w.forest, w.head
    g, d = h.group, h.head_dim
    Q = widen(w.q_bits(), h.dtype)
    total_rows = max(int(t[5]) + int(t[4]) * g for t in tasks) if len(tasks) else 0
    out = np.zeros((f.num_requests, h.num_q_heads, d))
    for kvh in range(h.num_kv_heads):
        PO = np.full((total_rows, d), np.nan)
        PM = np.full(total_rows, np.nan)
        PS = np.full(total_rows, np.nan)
        for (node, kv_begin, kv_len, q_off, n_req, base) in tasks:
            reqs = node_q_flat[q_off:q_off + n_req]
            K, V = gather_node_kv(w, int(node), kvh, int(kv_begin), int(kv_begin + kv_len))
            Qt = Q[reqs, kvh * g:(kvh + 1) * g, :].reshape(-1, d)
            O, m, s = pac(Qt, K, V, h.scale, _visibility(f, int(node), reqs, g, int(kv_begin), int(kv_begin + kv_len)))
            rows = slice(int(base), int(base) + n_req * g)
            assert np.all(np.isnan(PM[rows])), "two tasks write the same partial rows"
            PO[rows], PM[rows], PS[rows] = O, m, s
        for r in range(f.num_requests):
            acc = None
            for e in range(int(req_part_off[r]), int(req_part_off[r + 1])):
                a = int(req_part[e])
                part = (PO[a:a + g], PM[a:a + g], PS[a:a + g])
                assert not np.any(np.isnan(part[1])), "partial row never written"
                acc = part if acc is None else por(*acc, *part)
            out[r, kvh * g:(kvh + 1) * g, :] = acc[0]
    return out
