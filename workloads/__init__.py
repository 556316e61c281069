"""Seeded synthetic inputs for prefix-tree decode attention.

This package only builds inputs: prefix forests, page tables and random Q/K/V
tensors.  It holds none of the method's arithmetic (no attention, no softmax,
no planning), so both the CPU oracle's tests and the HIP path's tests can draw
their inputs from it without sharing any code of the method itself.
"""
from .trees import (Forest, two_level_forest, three_level_forest, random_forest,
                    unshared_forest, full_kary_forest, degenerate_forest, draft_tree_forest, draft_masked_forest,
                    concat_forests, forest_stats)
from .tensors import (HeadConfig, PagedKV, Workload, build_paged_kv, make_workload,
                      bits_to_float64, float_to_bits, DTYPE_FP16, DTYPE_BF16)
from .configs import CONFIG_NAMES, make_config, make_small_config

__all__ = [
    "Forest", "two_level_forest", "three_level_forest", "random_forest", "unshared_forest",
    "full_kary_forest", "degenerate_forest", "draft_tree_forest", "draft_masked_forest", "concat_forests", "forest_stats",
    "HeadConfig", "PagedKV", "Workload", "build_paged_kv", "make_workload",
    "bits_to_float64", "float_to_bits", "DTYPE_FP16", "DTYPE_BF16",
    "CONFIG_NAMES", "make_config", "make_small_config",
]
