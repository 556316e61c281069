"""Synthetic sweeps with the shapes of the paper's comparison workloads (Sec. 7, "Comparison with SOTA",
"Ablation Studies", "Impact of Division Granularity").

Forests only; tensors come from ``make_workload`` like every other input.  Each sweep is a list of
(label, forest); all use GQA 32 / 8, head_dim 128, bf16, 16-token pages.  Lengths are multiples of 16.

* ``seqlen``   two-level tree, 32768-token shared root, 32 requests, unshared part 512 .. 8192 tokens
* ``batch``    two-level tree, 122880-token (120k) shared root, 256-token suffixes, 1 .. 64 requests
* ``depth``    full binary tree of 2 .. 6 levels, 8192 tokens per node, one request per leaf
* ``ratio``    two-level tree, 16 requests of 122880 tokens each, shared fraction 0 .. 0.99 of a context
* ``shape``    full 2-, 3-, 4-, 5-ary trees of 3 levels and a 6-level degenerate tree, about 2^18 unique
               tokens each ("the same workload" over different shapes)
* ``ablation`` a full binary tree (6 levels) and a degenerate tree (8 levels) with 204800-token (200k)
               contexts, for the tree on/off x division on/off grid
* ``draft``    verification of drafted token trees (multi-token decoding): 16 sequences of 8192 tokens
               under a shared 2048-token prompt, each with a random tree of 0 .. 64 one-token draft nodes
               and one request per draft token; not one of the paper's sweeps, its motivation names the
               use case
* ``draft_masked``  the same verification steps with the drafted tokens of a sequence packed into one
               node and a visibility mask per query (Sec. 4.1) in place of the one-token nodes
"""
from __future__ import annotations

from typing import List, Tuple

from .trees import (Forest, two_level_forest, full_kary_forest, degenerate_forest, unshared_forest,
                    draft_tree_forest, draft_masked_forest)
from .tensors import HeadConfig, DTYPE_BF16

SWEEP_NAMES = ["seqlen", "batch", "depth", "ratio", "shape", "ablation", "draft", "draft_masked"]
SWEEP_SEED = 2000


def sweep_head() -> HeadConfig:
    return HeadConfig(32, 8, 128, DTYPE_BF16)


def _r16(x: float) -> int:
    return max(16, int(round(x / 16.0)) * 16)


def sweep_points(name: str) -> List[Tuple[str, Forest]]:
    if name == "seqlen":
        return [(f"unshared={n}", two_level_forest(32768, [n] * 32)) for n in (512, 1024, 2048, 4096, 8192)]
    if name == "batch":
        return [(f"requests={b}", two_level_forest(122880, [256] * b)) for b in (1, 2, 4, 8, 16, 32, 64)]
    if name == "depth":
        return [(f"levels={d}", full_kary_forest(2, d, lambda lvl: 8192)) for d in (2, 3, 4, 5, 6)]
    if name == "ratio":
        pts = []
        for r in (0.0, 0.25, 0.5, 0.75, 0.9, 0.99):
            shared = _r16(122880 * r) if r > 0 else 0
            own = 122880 - shared
            f = unshared_forest([own] * 16) if shared == 0 else two_level_forest(shared, [own] * 16)
            pts.append((f"shared={r:g}", f))
        return pts
    if name == "shape":
        pts = []
        for k in (2, 3, 4, 5):
            nodes = 1 + k + k * k
            pts.append((f"{k}T", full_kary_forest(k, 3, lambda lvl, n=nodes: _r16(262144 / n))))
        pts.append(("DT", degenerate_forest(6, _r16(262144 / 11), _r16(262144 / 11))))
        return pts
    if name == "ablation":
        return [("balanced", full_kary_forest(2, 6, lambda lvl: _r16(204800 / 6))),
                ("degenerate", degenerate_forest(8, _r16(204800 / 8), _r16(204800 / 8)))]
    if name == "draft":
        # verification of drafted token trees (the speculative-decoding use of prefix sharing named
        # in the motivation): 16 sequences of 8192 tokens under a prompt of 2048
        return [(f"drafted={t}", draft_tree_forest(2048, [8192] * 16, t, SWEEP_SEED + t)) for t in (0, 4, 16, 64)]
    if name == "draft_masked":
        return [(f"drafted={t}", draft_masked_forest(2048, [8192] * 16, t, SWEEP_SEED + t)) for t in (0, 4, 16, 64)]
    raise KeyError(name)
