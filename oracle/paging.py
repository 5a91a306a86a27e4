"""CPU oracle: reference page allocation for per-candidate suffix KV.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The shared prefix is one block outside the pool.  Each candidate's suffix tokens go
to fixed-size pages taken from a free list.  Rule: before a decode step appends one
token per candidate, candidates are visited in ascending index; one whose suffix
length is a multiple of the page size takes the page at the head of the free list.
"""
from __future__ import annotations

import numpy as np


def page_tables(n_cands: int, n_steps: int, page_tokens: int, free_list) -> np.ndarray:
    """Page table after n_steps lock-step decode steps: [n_cands][ceil(n_steps/page_tokens)]."""
    free = list(free_list)
    n_pages = -(-n_steps // page_tokens)
    table = -np.ones((n_cands, max(n_pages, 1)), dtype=np.int32)
    head = 0
    for t in range(n_steps):                  # suffix length before the append is t
        if t % page_tokens == 0:
            for b in range(n_cands):
                table[b, t // page_tokens] = free[head]
                head += 1
    return table[:, :n_pages] if n_pages else table[:, :0]


def slot_of(table: np.ndarray, b: int, j: int, page_tokens: int):
    """(page id, offset in page) of candidate b's j-th suffix token."""
    return int(table[b, j // page_tokens]), j % page_tokens
