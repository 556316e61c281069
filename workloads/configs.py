"""The measured configurations, as seeded synthetic workloads.

Names: cfg1 .. cfg4, cfg5a (shared long prefix), cfg5b (unshared control
batch), cfg5c (both in one forest).  ``make_small_config`` gives shrunken
versions with the same structure (several tiles, ragged tails) that a plain CPU
implementation finishes in seconds.
"""
from __future__ import annotations

import numpy as np

from .trees import (Forest, two_level_forest, three_level_forest, random_forest,
                    unshared_forest, concat_forests)
from .tensors import HeadConfig, Workload, make_workload, DTYPE_FP16, DTYPE_BF16

CONFIG_NAMES = ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5a", "cfg5b", "cfg5c"]
_INDEX = {"cfg1": 0, "cfg2": 1, "cfg3": 2, "cfg4": 3, "cfg5a": 4, "cfg5b": 4, "cfg5c": 4}


def config_seed(name: str) -> int:
    return 1000 + _INDEX[name]


def config_head(name: str) -> HeadConfig:
    if name == "cfg1":
        return HeadConfig(8, 8, 128, DTYPE_FP16)
    if name in ("cfg2", "cfg3", "cfg4"):
        return HeadConfig(32, 8, 128, DTYPE_BF16)
    return HeadConfig(64, 8, 128, DTYPE_BF16)


def config_forest(name: str, shrink: int = 1, req_shrink: int = 1) -> Forest:
    """Forest of a configuration.

    ``shrink`` > 1 divides node lengths, ``req_shrink`` > 1 divides request
    (and mid-node) counts; both keep the structure and leave ragged lengths.
    """
    seed = config_seed(name)
    s, sr = shrink, req_shrink
    if name == "cfg1":
        return two_level_forest(max(1024 // s, 48), [max(64 // s, 5)] * 4)
    if name == "cfg2":
        return two_level_forest(max(4096 // s, 100), [max(256 // s, 19)] * max(64 // sr, 3))
    if name == "cfg3":
        rng = np.random.Generator(np.random.PCG64(seed))
        nm, lpm = max(16 // sr, 2), max(16 // sr, 3)
        leaf = rng.integers(max(32 // s, 1), max(512 // s, 40) + 1, size=nm * lpm)
        return three_level_forest(max(2048 // s, 70), [max(8192 // s, 150)] * nm, lpm, leaf)
    if name == "cfg4":
        return random_forest(max(512 // sr, 12), 5, 2.0, max(512 // s, 24), 1.0,
                             max(16 // s, 1), max(32768 // s, 300), seed)
    a = two_level_forest(max(131072 // s, 400), [max(1024 // s, 33)] * max(64 // sr, 3))
    b = unshared_forest([max(32768 // s, 210)] * max(64 // sr, 2))
    if name == "cfg5a":
        return a
    if name == "cfg5b":
        return b
    if name == "cfg5c":
        return concat_forests(a, b)
    raise KeyError(name)


def make_config(name: str, device: str = "cpu", layout: str = "thd", poison: bool = False) -> Workload:
    return make_workload(name, config_forest(name), config_head(name), config_seed(name),
                         device=device, layout=layout, poison=poison)


def make_small_config(name: str, shrink: int = 16, req_shrink: int = 1, device: str = "cpu",
                      layout: str = "thd", poison: bool = True) -> Workload:
    return make_workload(name + f"/len{shrink}/req{req_shrink}", config_forest(name, shrink, req_shrink),
                         config_head(name), config_seed(name), device=device, layout=layout,
                         poison=poison)
