"""Workload statistics in the paper's terms (Table 1)."""


def kv_pruned_fraction(max_cache: float, output_len: float) -> float:
    """Table 1: KV pruned = 1 - max_cache / output_len."""
    return 1.0 - max_cache / output_len
