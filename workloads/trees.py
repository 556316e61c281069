"""Prefix forests: which KV-cache node is a prefix of which, and where requests end.

A forest is three int32 arrays.  ``parent[i]`` is the node whose tokens come
directly before node ``i``'s tokens (-1 for a top-level prefix, i.e. a child of
the virtual root that joins unrelated prefixes), ``node_len[i]`` is the number
of tokens the node holds and ``req_node[r]`` is the last node on request
``r``'s root-to-leaf path.  Shapes follow the workloads the paper evaluates
(two-level document-QA trees, full k-ary trees, a degenerate left-spine tree)
and the configurations this build is measured on.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np


@dataclass
class Forest:
    parent: np.ndarray      # int32 [N]
    node_len: np.ndarray    # int32 [N]
    req_node: np.ndarray    # int32 [B]
    # optional visibility masks over the tokens of each request's LAST node: request r owns the 32-bit
    # words req_mask[req_mask_off[r] : req_mask_off[r + 1]] (none: it sees every token); bit t % 32 of
    # word t // 32 says whether it sees token t of node req_node[r]
    req_mask_off: Optional[np.ndarray] = None   # int32 [B + 1]
    req_mask: Optional[np.ndarray] = None       # uint32

    def __post_init__(self):
        self.parent = np.ascontiguousarray(self.parent, dtype=np.int32)
        self.node_len = np.ascontiguousarray(self.node_len, dtype=np.int32)
        self.req_node = np.ascontiguousarray(self.req_node, dtype=np.int32)
        assert self.parent.shape == self.node_len.shape
        if self.req_mask_off is not None:
            self.req_mask_off = np.ascontiguousarray(self.req_mask_off, dtype=np.int32)
            self.req_mask = np.ascontiguousarray(self.req_mask, dtype=np.uint32)
            assert self.req_mask_off.shape == (self.req_node.shape[0] + 1,)

    def visible(self, r: int) -> Optional[np.ndarray]:
        """bool [node_len of r's last node], or None when request r carries no mask."""
        if self.req_mask_off is None or self.req_mask_off[r + 1] == self.req_mask_off[r]:
            return None
        words = self.req_mask[self.req_mask_off[r]:self.req_mask_off[r + 1]]
        n = int(self.node_len[self.req_node[r]])
        t = np.arange(n)
        return ((words[t // 32] >> (t % 32).astype(np.uint32)) & 1).astype(bool)

    @property
    def num_nodes(self) -> int:
        return int(self.parent.shape[0])

    @property
    def num_requests(self) -> int:
        return int(self.req_node.shape[0])

    def path(self, r: int) -> List[int]:
        """Root-to-leaf node ids of request r (input plumbing for generators and reports)."""
        out = []
        n = int(self.req_node[r])
        while n >= 0:
            out.append(n)
            n = int(self.parent[n])
        return out[::-1]


def two_level_forest(root_len: int, leaf_lens: Sequence[int]) -> Forest:
    """One shared prefix, one private suffix per request (document QA)."""
    b = len(leaf_lens)
    parent = np.array([-1] + [0] * b, dtype=np.int32)
    node_len = np.array([root_len] + list(leaf_lens), dtype=np.int32)
    req_node = np.arange(1, b + 1, dtype=np.int32)
    return Forest(parent, node_len, req_node)


def three_level_forest(root_len: int, mid_lens: Sequence[int], leaves_per_mid: int,
                       leaf_lens: Sequence[int]) -> Forest:
    """Root shared by all, each mid node shared by ``leaves_per_mid`` requests."""
    nm = len(mid_lens)
    assert len(leaf_lens) == nm * leaves_per_mid
    parent = [-1] + [0] * nm
    node_len = [root_len] + list(mid_lens)
    req_node = []
    for m in range(nm):
        for j in range(leaves_per_mid):
            parent.append(1 + m)
            node_len.append(int(leaf_lens[m * leaves_per_mid + j]))
            req_node.append(len(parent) - 1)
    return Forest(np.array(parent), np.array(node_len), np.array(req_node))


def unshared_forest(lens: Sequence[int]) -> Forest:
    """Every request has its own single node under the virtual root (no sharing)."""
    b = len(lens)
    return Forest(np.full(b, -1, dtype=np.int32), np.array(lens, dtype=np.int32),
                  np.arange(b, dtype=np.int32))


def full_kary_forest(k: int, depth: int, node_len_of_depth) -> Forest:
    """Full k-ary tree with ``depth`` levels; one request per leaf.

    ``node_len_of_depth(level)`` gives the token count of a node at ``level`` (1 = root).
    """
    parent, node_len, level_nodes = [-1], [int(node_len_of_depth(1))], [0]
    for lvl in range(2, depth + 1):
        nxt = []
        for p in level_nodes:
            for _ in range(k):
                parent.append(p)
                node_len.append(int(node_len_of_depth(lvl)))
                nxt.append(len(parent) - 1)
        level_nodes = nxt
    return Forest(np.array(parent), np.array(node_len), np.array(level_nodes))


def degenerate_forest(depth: int, spine_len: int, leaf_len: int) -> Forest:
    """Left-spine tree: at every level only the left child has children.

    Each spine node has a right child that is a leaf; the last spine node is
    itself a leaf.  One request per leaf.
    """
    parent, node_len, req_node = [-1], [spine_len], []
    spine = 0
    for _ in range(depth - 1):
        parent.append(spine); node_len.append(leaf_len); req_node.append(len(parent) - 1)
        parent.append(spine); node_len.append(spine_len); spine = len(parent) - 1
    req_node.append(spine)
    return Forest(np.array(parent), np.array(node_len), np.array(req_node))


def random_forest(num_leaves: int, max_depth: int, poisson_mean: float,
                  median_len: int, sigma: float, min_len: int, max_len: int,
                  seed: int) -> Forest:
    """Seeded irregular forest: child count 1+Poisson(mean), log-normal node lengths.

    Breadth-first growth.  A new top-level prefix is started whenever the
    frontier is empty; a popped node below ``max_depth`` gets 1+Poisson
    children, clipped so the number of leaves never exceeds ``num_leaves``;
    growth stops when exactly ``num_leaves`` leaves exist.  One request per leaf.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    parent: List[int] = []
    depth: List[int] = []
    nchild: List[int] = []
    frontier: List[int] = []          # nodes that may still get children
    leaves = 0                        # current number of childless nodes

    def new_node(p: int, d: int) -> int:
        parent.append(p); depth.append(d); nchild.append(0)
        return len(parent) - 1

    head = 0
    while leaves < num_leaves:
        if head >= len(frontier):
            frontier.append(new_node(-1, 1))
            leaves += 1
            continue
        n = frontier[head]; head += 1
        if depth[n] >= max_depth:
            continue
        # giving c children to a childless node turns one leaf into c leaves
        c = min(1 + int(rng.poisson(poisson_mean)), num_leaves - leaves + 1)
        for _ in range(c):
            frontier.append(new_node(n, depth[n] + 1))
        nchild[n] = c
        leaves += c - 1
    n_nodes = len(parent)
    z = rng.standard_normal(n_nodes)
    lens = np.clip(np.rint(np.exp(np.log(float(median_len)) + sigma * z)), min_len, max_len)
    req_node = [i for i in range(n_nodes) if nchild[i] == 0]
    assert len(req_node) == num_leaves, (len(req_node), num_leaves)
    return Forest(np.array(parent), lens.astype(np.int32), np.array(req_node))


def draft_tree_forest(prompt_len: int, context_lens: Sequence[int], draft_tokens: int, seed: int) -> Forest:
    """Verification step of tree-structured speculative decoding (multi-token decoding).

    A prompt of ``prompt_len`` tokens is shared by all sequences (0: none); sequence i has
    ``context_lens[i]`` tokens of its own; on top of each sits a seeded random tree of
    ``draft_tokens`` drafted tokens, every one a node of length 1 whose parent is the token it was
    drafted after (an earlier draft token of the sequence, or the sequence's context).  A query
    sees exactly the tokens on its path, so which drafted tokens a query may attend to is given by
    the tree itself.  There is one request per context node (the last accepted token) and one per
    draft token: requests end at internal nodes as well as at leaves.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    parent: List[int] = []
    node_len: List[int] = []
    req_node: List[int] = []
    top = -1
    if prompt_len > 0:
        parent.append(-1); node_len.append(prompt_len); top = 0
    for ctx_len in context_lens:
        parent.append(top); node_len.append(int(ctx_len))
        ctx = len(parent) - 1
        req_node.append(ctx)
        drafted = [ctx]
        for _ in range(draft_tokens):
            # half of the tokens extend the newest branch, the others start a sibling branch
            # somewhere in the tree drafted so far
            after = drafted[-1] if rng.random() < 0.5 else drafted[int(rng.integers(len(drafted)))]
            parent.append(after); node_len.append(1)
            drafted.append(len(parent) - 1)
            req_node.append(len(parent) - 1)
    return Forest(np.array(parent), np.array(node_len), np.array(req_node))


def draft_masked_forest(prompt_len: int, context_lens: Sequence[int], draft_tokens: int, seed: int) -> Forest:
    """The verification step of ``draft_tree_forest`` with the drafted tokens of a sequence packed into
    ONE node and visibility masks in place of one-token nodes.

    Same seeded draft trees and the same request order as ``draft_tree_forest`` (a request for the
    sequence's context, then one per drafted token in the order they were drafted).  The drafted tokens
    of a sequence form a node of ``draft_tokens`` tokens below the sequence's context, token k being the
    k-th drafted one; the request of drafted token k ends at that node and sees, of its tokens, token k
    and the drafted tokens k was drafted after (its ancestors in the draft tree): bit j of its mask.
    A token is always drafted after an earlier one, so a request's visible tokens come in the order of
    its path in the one-token-node formulation.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    parent: List[int] = []
    node_len: List[int] = []
    req_node: List[int] = []
    masks: List[List[int]] = []
    words = (draft_tokens + 31) // 32
    top = -1
    if prompt_len > 0:
        parent.append(-1); node_len.append(prompt_len); top = 0
    for ctx_len in context_lens:
        parent.append(top); node_len.append(int(ctx_len))
        ctx = len(parent) - 1
        req_node.append(ctx)
        masks.append([])
        if draft_tokens == 0:
            continue
        parent.append(ctx); node_len.append(draft_tokens)
        draft = len(parent) - 1
        after_of: List[int] = []                  # per drafted token: the drafted token before it, -1 = the context
        order = [-1]                              # the tokens drafted so far, the context first (as in draft_tree_forest)
        for k in range(draft_tokens):
            after = order[-1] if rng.random() < 0.5 else order[int(rng.integers(len(order)))]
            after_of.append(after)
            order.append(k)
            bits = [0] * words
            t = k
            while t != -1:
                bits[t // 32] |= 1 << (t % 32)
                t = after_of[t]
            req_node.append(draft)
            masks.append(bits)
    off = np.zeros(len(req_node) + 1, dtype=np.int32)
    np.cumsum([len(m) for m in masks], out=off[1:])
    flat = np.array([w for m in masks for w in m], dtype=np.uint32)
    return Forest(np.array(parent), np.array(node_len), np.array(req_node), off, flat)


def concat_forests(a: Forest, b: Forest) -> Forest:
    """Both forests under one virtual root; b's node ids are shifted by a.num_nodes."""
    shift = a.num_nodes
    pb = b.parent.copy()
    pb[pb >= 0] += shift
    off = words = None
    if a.req_mask_off is not None or b.req_mask_off is not None:
        ao = a.req_mask_off if a.req_mask_off is not None else np.zeros(a.num_requests + 1, dtype=np.int32)
        bo = b.req_mask_off if b.req_mask_off is not None else np.zeros(b.num_requests + 1, dtype=np.int32)
        aw = a.req_mask if a.req_mask is not None else np.zeros(0, dtype=np.uint32)
        bw = b.req_mask if b.req_mask is not None else np.zeros(0, dtype=np.uint32)
        off = np.concatenate([ao, bo[1:] + ao[-1]])
        words = np.concatenate([aw, bw])
    return Forest(np.concatenate([a.parent, pb]),
                  np.concatenate([a.node_len, b.node_len]),
                  np.concatenate([a.req_node, b.req_node + shift]), off, words)


def forest_stats(f: Forest) -> dict:
    """Token counts used in reports: unique tokens, per-request-summed tokens, sharing ratio."""
    n_q = np.zeros(f.num_nodes, dtype=np.int64)
    for r in range(f.num_requests):
        for n in f.path(r):
            n_q[n] += 1
    used = n_q > 0
    unique = int(f.node_len[used].astype(np.int64).sum())
    flat = int((f.node_len.astype(np.int64) * n_q).sum())
    return {"num_nodes": f.num_nodes, "num_requests": f.num_requests,
            "unique_tokens": unique, "flat_tokens": flat,
            "mean_sharing": (flat / unique) if unique else 0.0,
            "max_n_q": int(n_q.max()) if f.num_nodes else 0,
            "max_node_len": int(f.node_len.max()) if f.num_nodes else 0}
