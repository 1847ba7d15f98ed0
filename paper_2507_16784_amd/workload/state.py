"""Seeded initial paging state: which physical pages a preloaded batch owns.

A serving runtime that has been up for a while holds its sequences in
scattered physical pages.  This recipe shuffles the page ids with the seeded
generator, hands each sequence the next ceil(len / page_size) ids for its
logical pages 0, 1, 2, ..., and leaves the rest as the free stack (bottom
first, in shuffled order).  Index bookkeeping only.
"""
from typing import List, Sequence

from .rng import Stream


def scattered_pages(seed: int, num_pages: int, page_size: int, seq_lens: Sequence[int]):
    """Returns (tables, free_ids): tables[b] = physical ids of sequence b's pages."""
    perm = Stream(seed).permutation(num_pages)
    tables: List[List[int]] = []
    at = 0
    for n in seq_lens:
        k = (n + page_size - 1) // page_size
        if at + k > num_pages:
            raise ValueError("pool too small for the preloaded batch")
        tables.append(perm[at : at + k])
        at += k
    return tables, perm[at:]
