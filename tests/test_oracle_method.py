"""Pins for the step-by-step method oracle (oracle/method.py): Alg. 2-4 and Sec. 4.1.

The partial-attention / partial-reduction pipeline must reproduce the
definition oracle exactly (up to fp64 rounding), and the reduction must not
depend on order or bracketing (Sec. 4.3, "Parallelization of the tree
reduction operation").
"""
import itertools

import numpy as np
import pytest

from oracle import attention as A
from oracle import method as M
from workloads import (HeadConfig, make_workload, make_small_config, two_level_forest,
                       three_level_forest, degenerate_forest, full_kary_forest, unshared_forest,
                       concat_forests, DTYPE_FP16, DTYPE_BF16)


def _rand_parts(rng, n_parts, n_q=5, d=16, n=13):
    Q = rng.standard_normal((n_q, d))
    parts, Ks, Vs = [], [], []
    for _ in range(n_parts):
        K = rng.standard_normal((n, d)) * 3
        V = rng.standard_normal((n, d))
        Ks.append(K); Vs.append(V)
        parts.append(M.pac(Q, K, V, 0.4))
    return Q, Ks, Vs, parts


def test_widen_matches_numpy_and_torch():
    import torch
    bits = np.arange(0, 65536, 3, dtype=np.uint32).astype(np.uint16)
    a = M.widen(bits, 0)
    b = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(a[~np.isnan(b)], b[~np.isnan(b)])
    c = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).double().numpy()
    a = M.widen(bits, 1)
    assert np.array_equal(a[~np.isnan(c)], c[~np.isnan(c)])


def test_pac_is_softmax_attention():
    from scipy.special import softmax
    rng = np.random.default_rng(0)
    Q, Ks, Vs, parts = _rand_parts(rng, 1)
    O, m, s = parts[0]
    ref = softmax(Q @ Ks[0].T * 0.4, axis=1) @ Vs[0]
    assert np.max(np.abs(O - ref)) < 1e-14
    assert np.all(s >= 1.0)                      # the maximum itself contributes e^0


def test_por_commutative_and_associative():
    rng = np.random.default_rng(1)
    _, _, _, (a, b, c) = _rand_parts(rng, 3)
    ab, ba = M.por(*a, *b), M.por(*b, *a)
    for x, y in zip(ab, ba):
        assert np.array_equal(x, y) or np.max(np.abs(x - y)) < 1e-15
    left = M.por(*M.por(*a, *b), *c)
    right = M.por(*a, *M.por(*b, *c))
    assert np.max(np.abs(left[0] - right[0])) < 1e-14
    assert np.max(np.abs(left[1] - right[1])) == 0
    assert np.max(np.abs(left[2] - right[2]) / left[2]) < 1e-14


def test_merge_of_any_split_equals_unsplit_attention():
    rng = np.random.default_rng(2)
    Q, Ks, Vs, parts = _rand_parts(rng, 4)
    whole = M.pac(Q, np.concatenate(Ks), np.concatenate(Vs), 0.4)
    for perm in itertools.permutations(range(4)):
        acc = parts[perm[0]]
        for i in perm[1:]:
            acc = M.por(*acc, *parts[i])
        assert np.max(np.abs(acc[0] - whole[0])) < 1e-14
        lse_acc = acc[1] + np.log(acc[2])
        lse_whole = whole[1] + np.log(whole[2])
        assert np.max(np.abs(lse_acc - lse_whole)) < 1e-13
    # balanced bracketing too
    bal = M.por(*M.por(*parts[0], *parts[1]), *M.por(*parts[2], *parts[3]))
    assert np.max(np.abs(bal[0] - whole[0])) < 1e-14


def test_streaming_accumulators_equal_binary_reduction():
    rng = np.random.default_rng(3)
    Q, Ks, Vs, parts = _rand_parts(rng, 3)
    Mx = np.full(5, -np.inf); D = np.zeros(5); U = np.zeros((5, 16))
    for (O, m, s) in parts:
        Mx, D, U = M.streaming_update(Mx, D, U, m, s, O * s[:, None])
    acc = parts[0]
    for p in parts[1:]:
        acc = M.por(*acc, *p)
    assert np.max(np.abs(U / D[:, None] - acc[0])) < 1e-14
    assert np.array_equal(Mx, acc[1])


def test_large_logits_stay_finite():
    """Partials whose maxima differ by hundreds must merge without overflow."""
    rng = np.random.default_rng(4)
    Q = rng.standard_normal((2, 8))
    K1, K2 = rng.standard_normal((6, 8)) * 200, rng.standard_normal((6, 8)) * 0.01
    V1, V2 = rng.standard_normal((6, 8)), rng.standard_normal((6, 8))
    a, b = M.pac(Q, K1, V1, 1.0), M.pac(Q, K2, V2, 1.0)
    merged = M.por(*a, *b)
    whole = M.pac(Q, np.concatenate([K1, K2]), np.concatenate([V1, V2]), 1.0)
    assert np.all(np.isfinite(merged[0]))
    assert np.max(np.abs(merged[0] - whole[0])) < 1e-13


FORESTS = {
    "two_level": lambda: two_level_forest(45, [7, 1, 19, 4]),
    "three_level": lambda: three_level_forest(9, [21, 5], 3, [3, 8, 1, 2, 6, 11]),
    "degenerate": lambda: degenerate_forest(4, 10, 3),
    "binary_depth4": lambda: full_kary_forest(2, 4, lambda lvl: 3 * lvl + 1),
    "mixed_with_unshared": lambda: concat_forests(two_level_forest(12, [5, 6]), unshared_forest([17, 2])),
}


@pytest.mark.parametrize("name", sorted(FORESTS))
@pytest.mark.parametrize("dtype,hq,hkv", [(DTYPE_FP16, 2, 2), (DTYPE_BF16, 8, 2)])
def test_tree_merged_result_equals_definition(name, dtype, hq, hkv):
    w = make_workload(name, FORESTS[name](), HeadConfig(hq, hkv, 16, dtype, page_size=4), seed=31,
                      poison=True)
    ref, _ = A.decode_attention_workload(w)
    got = M.codec(w)
    assert np.max(np.abs(got - ref)) < 1e-13


def test_tree_merged_equals_definition_on_shrunken_config():
    w = make_small_config("cfg4", shrink=32, req_shrink=16)
    ref, _ = A.decode_attention_workload(w)
    got = M.codec(w)
    assert np.max(np.abs(got - ref)) < 1e-13


def test_masked_pac_is_attention_over_the_visible_positions():
    """Alg. 2 with the visibility mask of Sec. 4.1: a row's result equals plain softmax attention (scipy)
    over the positions it sees."""
    from scipy.special import softmax
    rng = np.random.default_rng(11)
    Q, K, V = rng.standard_normal((6, 16)), rng.standard_normal((21, 16)), rng.standard_normal((21, 16))
    vis = rng.random((6, 21)) < 0.4
    vis[np.arange(6), rng.integers(0, 21, size=6)] = True           # everybody sees something
    O, m, s = M.pac(Q, K, V, 0.25, vis)
    for i in range(6):
        idx = np.nonzero(vis[i])[0]
        sc = (K[idx] @ Q[i]) * 0.25
        assert np.allclose(O[i], softmax(sc) @ V[idx], atol=1e-14)
        assert np.isclose(m[i], sc.max()) and np.isclose(s[i], np.exp(sc - sc.max()).sum())


def test_tree_merged_result_with_masks_equals_definition():
    """Alg. 4 with masked drafted-token nodes (node-level partials, per-query reduction) = the definition."""
    from workloads import draft_masked_forest, DTYPE_BF16
    f = draft_masked_forest(20, [33, 9, 70], 37, seed=8)
    w = make_workload("masked-codec", f, HeadConfig(4, 2, 16, DTYPE_BF16, page_size=8), seed=3, poison=True)
    ref, _ = A.decode_attention_workload(w)
    assert np.max(np.abs(M.codec(w) - ref)) < 1e-13
